"""CPU fp64 oracle for the stage step and the cluster average.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; it is
used by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of
bench.py.  It shares no code with the HIP path.
"""
