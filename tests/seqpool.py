"""Test harness: evaluates the oracle's decoder block function and its reverse-mode derivative
one SEQUENCE per worker process, so that a full-size fp64 stage step finishes in seconds.

Nothing here is method arithmetic: every number comes from oracle/blocks.py, called by
seqpool_worker.py on one sequence.  What the split relies on: LayerNorm and the Linear layers
act on one token, causal attention on the tokens of one sequence, so out and grad_in of a
sequence depend on that sequence only, and the parameter gradient of a microbatch is the sum
of its sequences' gradients (pinned in tests/test_oracle_stage.py: the pooled stage equals
oracle.stage.Stage on the stacked microbatch).

Workers are separate interpreters (started with subprocess: they never touch the GPU); arrays
travel through anonymous shared memory (memfd), commands through the workers' pipes.
"""
import json
import mmap
import os
import subprocess
import sys

import numpy as np

from oracle import stage as ostage

HERE = os.path.dirname(os.path.abspath(__file__))


def _shared(nbytes):
    fd = os.memfd_create("rv_seqpool")
    os.ftruncate(fd, max(nbytes, 8))
    return fd, mmap.mmap(fd, max(nbytes, 8))


class SeqPool:
    def __init__(self, n_blocks, d, h, f, S, mb, eps=1e-5, workers=None):
        cores = len(os.sched_getaffinity(0))
        self.nw = nw = max(1, min(mb, workers or cores))
        self.mb, self.S, self.d = mb, S, d
        self.P = n_blocks * (4 * d * d + 2 * d * f + 9 * d + f)
        act = mb * S * d * 8
        sizes = {"W": self.P * 8, "X": act, "DY": act, "Y": act, "DX": act, "G": nw * self.P * 8}
        self._maps, fds = {}, {}
        for k, n in sizes.items():
            fds[k], self._maps[k] = _shared(n)
        view = lambda k, shape: np.frombuffer(self._maps[k], dtype=np.float64, count=int(np.prod(shape))).reshape(shape)
        self.W = view("W", (self.P,))
        self.X, self.DY, self.Y, self.DX = (view(k, (mb, S, d)) for k in ("X", "DY", "Y", "DX"))
        self.G = view("G", (nw, self.P))
        env = dict(os.environ)
        threads = str(max(1, cores // nw))
        for v in ("OPENBLAS_NUM_THREADS", "OMP_NUM_THREADS", "MKL_NUM_THREADS"):
            env[v] = threads
        self.procs = []
        for r in range(nw):
            spec = dict(rank=r, nw=nw, n_blocks=n_blocks, d=d, h=h, f=f, S=S, mb=mb, eps=eps, P=self.P, fds=fds)
            self.procs.append(subprocess.Popen(
                [sys.executable, "-u", os.path.join(HERE, "seqpool_worker.py"), json.dumps(spec)],
                stdin=subprocess.PIPE, stdout=subprocess.PIPE, env=env, pass_fds=list(fds.values()), text=True))
        for fd in fds.values():
            os.close(fd)
        self._wait("ready")

    def _wait(self, word):
        for p in self.procs:
            line = p.stdout.readline().strip()
            if line != word:
                raise RuntimeError("oracle worker failed: %r (exit %s)" % (line, p.poll()))

    def _run(self, cmd):
        for p in self.procs:
            p.stdin.write(cmd + "\n"); p.stdin.flush()
        self._wait("ok")

    def forward(self, w, x):
        np.copyto(self.W, w); np.copyto(self.X, x)
        self._run("fwd")
        return self.Y.copy()

    def backward(self, w, x, dy):
        np.copyto(self.W, w); np.copyto(self.X, x); np.copyto(self.DY, dy)
        self._run("bwd")
        return self.DX.copy(), np.add.reduce(self.G, axis=0)     # workers' gradients added in rank order

    def close(self):
        for p in self.procs:
            try:
                p.stdin.write("quit\n"); p.stdin.flush(); p.stdin.close()
            except (BrokenPipeError, ValueError):
                pass
        for p in self.procs:
            try:
                p.wait(timeout=30)
            except subprocess.TimeoutExpired:
                p.kill()
        self.procs = []

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


class PooledStage(ostage.Stage):
    """oracle.stage.Stage (all of its bookkeeping and its update) with the block function and its
    derivative evaluated through a SeqPool."""

    def __init__(self, pool, *a, **k):
        super().__init__(*a, **k)
        self.pool = pool

    def _f(self, w, x):
        return self.pool.forward(w, x)

    def _vjp(self, w, x, dy):
        return self.pool.backward(w, x, dy)
