"""The outer loop of the method (Alg. 2) for ONE stage position held by C clusters (fp64).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Step t samples a cluster i_t (the samples are an input: `picks`).  Its peer runs one
microbatch through Alg. 1 (forward, backward at the forward-time parameters).  If
(t+1) mod kappa != 0 the peer takes its own step x <- x - eta g (Alg. 2, else-branch, Eq. 3).
Otherwise that step is left pending and folded into Parallel Multi-Ring All-Reduce
(Alg. 2, the all-reduce branch): every cluster's parameters become the ring-partitioned mean of
(x_1, ..., x_{i_t} - eta g, ..., x_C), so the mean moves by -(eta/C) g (Eq. 17).
run(): one peer per cluster and staleness 0 inside the sampled peer: the stage-level staleness
is covered by oracle/stage.py; here the interplay of local steps and periodic averaging is.
run_chains(): every cluster is a chain of peers (section 3.3: cluster i holds x_i = (x_{i,1}, ...,
x_{i,P})); a microbatch runs forward through the chain and its gradient back, and every peer's
backward is one iteration t of Alg. 2 - the peer's own step, or, at an averaging iteration, the
all-reduce of the WHOLE model over the clusters with that peer's step folded into its block.
"""
import numpy as np

from . import average


def cluster_sync(stages, R, pending=None, ring_offsets=None, average_state=False):
    """All-reduce branch of Alg. 2 over the stages' parameter vectors; `pending` is the index of
    the stage whose last backward was deferred (its gradient is folded), or None.
    average_state: the optimiser state (the momentum buffers of section 4.1's optimiser) is
    averaged over the clusters in the same cycle, ring by ring like the parameters."""
    if average_state:
        vs, _, _ = average.multi_ring_allreduce([st.v for st in stages], R, ring_offsets=ring_offsets)
        for st, v in zip(stages, vs):
            st.v = np.array(v, dtype=np.float64)
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


def sync_chains(clusters, R, pending=None):
    """The all-reduce branch for clusters that are chains of peers: every peer position is
    averaged over the clusters (a ring set of its own per position); pending = (cluster, peer)
    of the deferred step, folded into that peer position only."""
    rounds = 0
    for p in range(len(clusters[0])):
        col = [c[p] for c in clusters]
        rounds = cluster_sync(col, R, pending=pending[0] if pending is not None and pending[1] == p else None)
    return rounds


def run_chains(clusters, picks, kappa, R, batch_fn, on_event=None):
    """Alg. 2 with chains.  picks[m] = cluster that takes microbatch m; batch_fn(m, i) -> (x,
    upstream-gradient function of the chain's output).  The iteration counter t advances with
    every peer backward (last peer first); on_event(t, i, p, sync) is called after each."""
    t = 0
    outs = []
    for m, i in enumerate(picks):
        chain = clusters[i]
        x, dy_fn = batch_fn(m, i)
        h = x
        for st in chain:
            h = st.forward(m, h)
        outs.append(h)
        dy = dy_fn(h)
        for p in reversed(range(len(chain))):
            sync = (t + 1) % kappa == 0
            dy = chain[p].backward(m, dy, defer=sync)
            if sync:
                sync_chains(clusters, R, pending=(i, p))
            if on_event is not None:
                on_event(t, i, p, sync)
            t += 1
    return outs
