"""The outer loop of the method (Alg. 2) for ONE stage position held by C clusters (fp64).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Step t samples a cluster i_t (the samples are an input: `picks`).  Its peer runs one
microbatch through Alg. 1 (forward, backward at the forward-time parameters).  If
(t+1) mod kappa != 0 the peer takes its own step x <- x - eta g (Alg. 2, else-branch, Eq. 3).
Otherwise that step is left pending and folded into Parallel Multi-Ring All-Reduce
(Alg. 2, the all-reduce branch): every cluster's parameters become the ring-partitioned mean of
(x_1, ..., x_{i_t} - eta g, ..., x_C), so the mean moves by -(eta/C) g (Eq. 17).
One peer per cluster and staleness 0 inside the sampled peer: the stage-level staleness is
covered by oracle/stage.py; here the interplay of local steps and periodic averaging is.
"""
import numpy as np

from . import average


def cluster_sync(stages, R, pending=None, ring_offsets=None):
    """All-reduce branch of Alg. 2 over the stages' parameter vectors; `pending` is the index of
    the stage whose last backward was deferred (its gradient is folded), or None."""
    xs = [st.w for st in stages]
    if pending is None:
        bufs, rounds, _ = average.multi_ring_allreduce(xs, R, ring_offsets=ring_offsets)
    else:
        p = stages[pending]
        bufs, rounds, _ = average.multi_ring_allreduce(xs, R, grad=p.last_grad, grad_replica=pending, eta=p.eta,
                                                       ring_offsets=ring_offsets)
    for st, b in zip(stages, bufs):
        st.install(b)
    return rounds


def run(stages, picks, kappa, R, batch_fn):
    """Alg. 2.  batch_fn(t, i) -> (x, upstream-gradient function of the stage output).  Returns the
    per-step outputs of the sampled stages."""
    outs = []
    for t, i in enumerate(picks):
        st = stages[i]
        x, dy_fn = batch_fn(t, i)
        y = st.forward(t, x)
        sync = (t + 1) % kappa == 0
        st.backward(t, dy_fn(y), defer=sync)
        if sync:
            cluster_sync(stages, R, pending=i)
        outs.append(y)
    return outs
