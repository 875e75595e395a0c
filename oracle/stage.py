"""One peer's stage step with stale gradients (fp64).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

Follows the peer body of the paper's Alg. 1 with the update of Eq. 2:
forward(mb) evaluates the block at the CURRENT parameters and remembers that
parameter state; backward(mb) computes the exact gradient of the block at the
remembered state (Eq. 2: the gradient is taken at the parameters in force
when that batch's forward ran), applies x <- x - eta * g to this block only
(Eq. 4: the sampling matrix keeps the peer's own block) and returns the
gradient for the preceding peer.

Plainly: a snapshot of the whole vector per in-flight microbatch, the forward
recomputed inside backward.  At most tau+1 microbatches may be in flight.
"""
import numpy as np
from . import blocks


def sgd_step(w, g, eta):
    """Eq. 2 on a block: x <- x - eta * g."""
    return w - eta * g


def momentum_step(w, g, v, eta, momentum, weight_decay):
    """The optimiser of the paper's single-cluster experiments (section 4.1: SGD with momentum and
    weight decay), taken in its usual form d = g + wd w; v <- mu v + d; w <- w - eta v.
    Returns (w, v)."""
    d = g + weight_decay * w
    v = momentum * v + d
    return w - eta * v, v


class StashFull(Exception):
    pass


class UnknownMicrobatch(Exception):
    pass


class DuplicateMicrobatch(Exception):
    pass


class Stage:
    def __init__(self, kind, tau, eta, flat_w, *, dims=None, n_blocks=None, d=None, h=None,
                 f=None, eps=1e-5, momentum=0.0, weight_decay=0.0, accumulate=1):
        assert kind in ("mlp", "decoder")
        self.kind, self.tau, self.eta = kind, int(tau), float(eta)
        self.dims, self.n_blocks, self.d, self.h, self.f, self.eps = dims, n_blocks, d, h, f, eps
        self.w = np.array(flat_w, dtype=np.float64)  # owns a copy
        self.k = 0                                     # number of updates applied
        self.live = {}                                 # mb_id -> (w snapshot, input, k at forward)
        self.last_grad = None
        self.last_staleness = None
        # optimiser of the paper's single-cluster experiments (section 4.1): SGD with
        # momentum and weight decay; both zero = the plain step of Eq. 2
        self.momentum, self.weight_decay = float(momentum), float(weight_decay)
        self.v = np.zeros_like(self.w)
        # gradient accumulation of the paper's multi-cluster experiment (section 4.2: gradients
        # of several microbatches are summed before one update); 1 = update on every backward
        self.accumulate = int(accumulate)
        self.g_sum = np.zeros_like(self.w)
        self.n_sum = 0

    def _f(self, w, x):
        if self.kind == "mlp":
            return blocks.mlp_forward(w, self.dims, x)
        return blocks.decoder_forward(w, self.n_blocks, self.d, self.h, self.f, self.eps, x)

    def _vjp(self, w, x, dy):
        if self.kind == "mlp":
            return blocks.mlp_backward(w, self.dims, x, dy)
        return blocks.decoder_backward(w, self.n_blocks, self.d, self.h, self.f, self.eps, x, dy)

    def forward(self, mb_id, x):
        if mb_id in self.live:
            raise DuplicateMicrobatch(mb_id)
        if len(self.live) >= self.tau + 1:
            raise StashFull(mb_id)
        x = np.array(x, dtype=np.float64)
        w_mb = self.w.copy()
        self.live[mb_id] = (w_mb, x, self.k)
        return self._f(w_mb, x)

    def backward(self, mb_id, dy, defer=False):
        """defer: compute the gradient but leave the update pending (Alg. 2: at an averaging
        step the sampled peer's update is folded into the all-reduce instead)."""
        if mb_id not in self.live:
            raise UnknownMicrobatch(mb_id)
        w_mb, x, k_fwd = self.live.pop(mb_id)
        dx, g = self._vjp(w_mb, x, np.array(dy, dtype=np.float64))
        self.last_grad = g
        self.last_staleness = self.k - k_fwd
        if defer:
            return dx
        self.g_sum = self.g_sum + g
        self.n_sum += 1
        if self.n_sum < self.accumulate:
            return dx                                           # no update yet: k counts updates
        g = self.g_sum
        self.g_sum = np.zeros_like(self.w)
        self.n_sum = 0
        if self.momentum == 0.0 and self.weight_decay == 0.0:
            self.w = sgd_step(self.w, g, self.eta)              # Eq. 2
        else:
            self.w, self.v = momentum_step(self.w, g, self.v, self.eta, self.momentum, self.weight_decay)
        self.k += 1
        return dx

    def install(self, w):
        """Parameters replaced from outside (the cluster average): a new weight version."""
        self.w = np.array(w, dtype=np.float64)
        self.k += 1
