"""Seeded synthetic inputs shared by tests, smoke and bench (no method arithmetic)."""
