"""Parameter averaging across C cluster replicas (fp64, plus an fp32 twin).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Definition form: the average the paper's analysis uses, x = (1/C) sum_i x_i
(section 3.4, assumption 4), optionally after one replica has taken its
pending step x_i - eta * g (Alg. 2, the all-reduce branch), which moves the
mean by -(eta/C) g (Eq. 17).

Algorithm form: Parallel Multi-Ring All-Reduce (section 3.2) built from the
ring all-reduce of section 2.3: R rings, each owning one segment of the
vector; inside a ring the segment is cut into C chunks and 2(C-1) rounds of
neighbour-to-neighbour sends first reduce, then propagate.  All rings and all
replicas act simultaneously in a round.

Readings where the text is silent: equal contiguous segments and chunks with
floor boundaries; sums accumulate in ring order and are divided by C once,
when the reduce phase of a chunk completes.
"""
import numpy as np


def ring_partition(n, R, C, ring_offsets=None):
    """bounds[r][j] .. bounds[r][j+1] is chunk j of ring r.  ring_offsets (R+1 element
    offsets) gives rings of unequal size (section 3.2: segment sizes follow the submodel
    boundaries of the clusters); default: R equal segments."""
    out = []
    for r in range(R):
        lo, hi = ((r * n) // R, ((r + 1) * n) // R) if ring_offsets is None else (ring_offsets[r], ring_offsets[r + 1])
        s = hi - lo
        out.append([lo + (j * s) // C for j in range(C + 1)])
    return out


def direct_mean(replicas, grad=None, grad_replica=0, eta=0.0):
    xs = [np.asarray(x, dtype=np.float64) for x in replicas]
    if grad is not None:
        xs = list(xs)
        xs[grad_replica] = xs[grad_replica] - float(eta) * np.asarray(grad, dtype=np.float64)
    acc = np.zeros_like(xs[0])
    for x in xs:
        acc = acc + x
    return acc / float(len(xs))


def multi_ring_allreduce(replicas, R, grad=None, grad_replica=0, eta=0.0, dtype=np.float64, ring_offsets=None):
    """Round-by-round simulation.  Returns (buffers, rounds, sent) where
    buffers[c] is replica c's vector after the cycle, rounds the number of
    rounds played and sent[r][c] the elements replica c sent on ring r."""
    C = len(replicas)
    buf = [np.array(x, dtype=dtype) for x in replicas]
    n = buf[0].size
    if grad is not None:
        step = (np.asarray(grad, dtype=dtype) * dtype(eta)).astype(dtype)
        buf[grad_replica] = (buf[grad_replica] - step).astype(dtype)
    bounds = ring_partition(n, R, C, ring_offsets)
    sent = [[0] * C for _ in range(R)]
    rounds = 0
    # reduce phase: after round s replica c+1 has added chunk (c - s) mod C
    for s in range(C - 1):
        msgs = []
        for r in range(R):
            for c in range(C):
                j = (c - s) % C
                lo, hi = bounds[r][j], bounds[r][j + 1]
                msgs.append((r, (c + 1) % C, lo, hi, buf[c][lo:hi].copy()))
                sent[r][c] += hi - lo
        for r, dst, lo, hi, data in msgs:
            buf[dst][lo:hi] = buf[dst][lo:hi] + data
        rounds += 1
    # chunk j is now complete on replica (j - 1) mod C: one division by C
    for r in range(R):
        for j in range(C):
            lo, hi = bounds[r][j], bounds[r][j + 1]
            o = (j - 1) % C
            buf[o][lo:hi] = buf[o][lo:hi] / dtype(C)
    # propagate phase: replica c forwards chunk (c + 1 - s) mod C
    for s in range(C - 1):
        msgs = []
        for r in range(R):
            for c in range(C):
                j = (c + 1 - s) % C
                lo, hi = bounds[r][j], bounds[r][j + 1]
                msgs.append((r, (c + 1) % C, lo, hi, buf[c][lo:hi].copy()))
                sent[r][c] += hi - lo
        for r, dst, lo, hi, data in msgs:
            buf[dst][lo:hi] = data
        rounds += 1
    return buf, rounds, sent


def ring_order_mean_f32(replicas, R, grad=None, grad_replica=0, eta=0.0, ring_offsets=None):
    """What the rounds above compute, written per chunk, in fp32: chunk j of
    every ring is summed starting at replica j and walking the ring, then
    divided by C.  Same operation order as multi_ring_allreduce(dtype=float32)
    (a test holds the two together)."""
    C = len(replicas)
    xs = [np.asarray(x, dtype=np.float32) for x in replicas]
    n = xs[0].size
    if grad is not None:
        step = np.asarray(grad, dtype=np.float32) * np.float32(eta)
        xs = list(xs)
        xs[grad_replica] = xs[grad_replica] - step
    out = np.empty(n, dtype=np.float32)
    for bnd in ring_partition(n, R, C, ring_offsets):
        for j in range(C):
            lo, hi = bnd[j], bnd[j + 1]
            acc = xs[j % C][lo:hi].copy()
            for s in range(1, C):
                acc = acc + xs[(j + s) % C][lo:hi]
            out[lo:hi] = acc / np.float32(C)
    return out
