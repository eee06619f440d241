"""Floating-point side of the Hop update (oracle side).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

  reduce_weights   mixing weight of every averaged vector: the communication
                   graph's W (Section 3.1, Eq. 1) times the iteration weight
                   Iter(u) - (k - s) + 1 of Eq. 2, renormalised over the set
                   that was actually accepted.  With equal tags or s = 0 this
                   is W renormalised (the plain mean of the backup-worker
                   figure when W is uniform); with uniform W it is exactly
                   Eq. 2; with everything accepted at tag k it is W itself.
  svm_subgradient  hinge-loss linear SVM minibatch subgradient
                   g = lambda w - (1/B) sum_{m: y_m <x_m, w> < 1} y_m x_m
                   ("Compute", Figure "Standard Decentralized Training" step 1);
                   with loss="log" the log loss the paper's own runs use
                   (Section 7.2): g = lambda w - (1/B) sum_m y_m x_m / (1 + exp(y_m <x_m, w>))
  momentum         Section 7.2's momentum 0.9, as a local velocity per worker:
                   v <- mu v + g, then x_{k+1} = sum_a w'_a x_a - eta v (the
                   velocity is never sent or averaged; a jump leaves it alone)
  reduce_apply     x_{k+1,i} = sum_a w'_a x_a - eta g   (steps 2 and 3 there)
  execute          all records in sequence order over rings of D slots
                   (serial approach of Section 3.2: an APPLY record is the same formula with the
                   single source x_k and weight 1, y_k = x_k - eta g(x_k); a REDUCE record the
                   same without gradient, x_{k+1} = sum_a w'_a y_a; x_k lives in slot D)

State and weights are fp32 (what is stored), sums are carried in fp64.
"""
import numpy as np

from . import rng

STEP = 0
JUMP = 1
APPLY = 2
REDUCE = 3


def reduce_weights(W, i, k, s, src_worker, src_tag):
    """Weights for Reduce at worker i in iteration k.  src_* list the self term
    first (its tag is k), then the accepted neighbours.  Returns (fp64 list,
    fp32 array); every weight is rounded to fp32 once."""
    r = []
    for j, t in zip(src_worker, src_tag):
        f = float(t - (k - s) + 1) if s >= 1 else 1.0
        r.append(float(W[j][i]) * f)
    tot = 0.0
    for v in r:
        tot += v
    w64 = [v / tot for v in r]
    return w64, np.array(w64, dtype=np.float64).astype(np.float32)


def hinge_margins(Xb, yb, w):
    """y_m <x_m, w> for the rows of a dense minibatch, in fp64."""
    return yb.astype(np.float64) * (Xb.astype(np.float64) @ w.astype(np.float64))


def loss_coefficients(yb, margins, B, loss, active=None):
    """c_m with g = lambda w - sum_m c_m x_m.  Hinge: y_m / B where the margin is below 1 (or where
    `active` says so), else 0.  Log loss: y_m / (B (1 + exp(margin)))."""
    if loss == "log":
        with np.errstate(over="ignore"):
            return yb / (float(B) * (1.0 + np.exp(margins))), np.ones(len(yb), dtype=bool)
    act = (margins < 1.0) if active is None else np.asarray(active, dtype=bool)
    return np.where(act, yb, 0.0) / float(B), act


def svm_subgradient_dense(X, y, w, rows, lam, active=None, loss="hinge"):
    """Returns (g fp64 [d], margins fp64 [B], active bool [B]).  `active`
    overrides the hinge indicator (used only to follow the other branch at a
    margin within rounding of the kink)."""
    Xb = X[rows].astype(np.float64)
    yb = y[rows].astype(np.float64)
    w64 = w.astype(np.float64)
    margins = yb * (Xb @ w64)
    coef, act = loss_coefficients(yb, margins, len(rows), loss, active)
    g = float(lam) * w64 - Xb.T @ coef
    return g, margins, act


def svm_subgradient_csr(rowptr, col, val, y, w, rows, lam, active=None, loss="hinge"):
    """Same for CSR features (rowptr int64, col int32 ascending per row)."""
    w64 = w.astype(np.float64)
    B = len(rows)
    margins = np.empty(B, dtype=np.float64)
    for m, r in enumerate(rows):
        lo, hi = int(rowptr[r]), int(rowptr[r + 1])
        margins[m] = float(y[r]) * float(np.dot(val[lo:hi].astype(np.float64), w64[col[lo:hi]]))
    yb = np.array([float(y[r]) for r in rows], dtype=np.float64)
    coef, act = loss_coefficients(yb, margins, B, loss, active)
    g = float(lam) * w64
    for m, r in enumerate(rows):
        if coef[m] != 0.0:
            lo, hi = int(rowptr[r]), int(rowptr[r + 1])
            np.subtract.at(g, col[lo:hi], coef[m] * val[lo:hi].astype(np.float64))
    return g, margins, act


def reduce_apply(vectors, w32, g, eta):
    """sum_a w'_a x_a - eta g in fp64, in record order, rounded to fp32 once.
    g = None for a jump's Reduce (no gradient)."""
    acc = np.zeros(vectors[0].shape, dtype=np.float64)
    for x, w in zip(vectors, w32):
        acc += float(w) * x.astype(np.float64)
    if g is not None:
        acc -= float(np.float32(eta)) * np.asarray(g, dtype=np.float64)
    return acc.astype(np.float32)


class GradZero:
    def __call__(self, i, k, w):
        return None


class GradSynth:
    """Synthetic gradient of the mixing-only workload at the columns `cols`."""

    def __init__(self, seed, variance, cols):
        self.seed, self.variance, self.cols = seed, variance, np.asarray(cols)

    def __call__(self, i, k, w):
        return rng.synth_grad(self.seed, i, k, self.cols, self.variance).astype(np.float64)


class GradSvmDense:
    def __init__(self, seed, X, y, batch, lam, loss="hinge"):
        self.seed, self.X, self.y, self.batch, self.lam, self.loss = seed, X, y, batch, lam, loss
        self.log = {}
        self.force = {}            # (i, k) -> bool[B], see svm_subgradient_dense

    def __call__(self, i, k, w):
        rows = rng.batch_rows(self.seed, i, k, self.batch, self.X[i].shape[0])
        g, m, a = svm_subgradient_dense(self.X[i], self.y[i], w, rows, self.lam,
                                        self.force.get((i, k)), self.loss)
        self.log[(i, k)] = (rows, m, a)
        return g


class GradSvmCsr:
    def __init__(self, seed, data, batch, lam, loss="hinge"):
        """data[i] = (rowptr, col, val, y)"""
        self.seed, self.data, self.batch, self.lam, self.loss = seed, data, batch, lam, loss
        self.log = {}
        self.force = {}

    def __call__(self, i, k, w):
        rowptr, col, val, y = self.data[i]
        rows = rng.batch_rows(self.seed, i, k, self.batch, len(rowptr) - 1)
        g, m, a = svm_subgradient_csr(rowptr, col, val, y, w, rows, self.lam,
                                      self.force.get((i, k)), self.loss)
        self.log[(i, k)] = (rows, m, a)
        return g


def init_rings(p0, N, D, serial=False):
    """x_{0,i} = p_0 in slot 0 of every worker (p0: [d] shared, or [N, d]).  D counts the slots in
    memory; with the serial approach the last of them holds the current parameters, and x_0 goes there."""
    p0 = np.asarray(p0, dtype=np.float32)
    rings = np.zeros((N, D) + p0.shape[-1:], dtype=np.float32)
    for i in range(N):
        rings[i, D - 1 if serial else 0] = p0 if p0.ndim == 1 else p0[i]
    return rings


def momentum_step(vel_i, g, mu):
    """v <- mu v + g in fp64 from the stored fp32 velocity; returns (fp64 value used by Apply, fp32
    value stored).  g = None counts as a zero gradient."""
    v64 = float(np.float32(mu)) * vel_i.astype(np.float64)
    if g is not None:
        v64 = v64 + np.asarray(g, dtype=np.float64)
    return v64, v64.astype(np.float32)


def apply_record(rings, rec, grad, eta, vel=None, mu=0.0):
    """Execute one record against the rings, in place; returns the new vector.  vel: [N, d] fp32
    velocities (updated in place by STEP records) when momentum is on."""
    vecs = [rings[j, sl] for j, sl in zip(rec.src_worker, rec.src_slot)]
    g = None
    if rec.kind == STEP or rec.kind == APPLY:
        g = grad(rec.worker, rec.k, vecs[0])
        if vel is not None:
            g, vel[rec.worker] = momentum_step(vel[rec.worker], g, mu)
    out = reduce_apply(vecs, rec.w32, g, eta)
    rings[rec.worker, rec.out_slot] = out
    return out


def execute(records, rings, grad, eta, on_record=None, vel=None, mu=0.0):
    """Records in sequence order.  Returns version[i] = newest iteration held."""
    version = [0] * rings.shape[0]
    for rec in records:
        out = apply_record(rings, rec, grad, eta, vel, mu)
        if rec.kind == STEP or rec.kind == REDUCE:
            version[rec.worker] = rec.k + 1
        elif rec.kind == JUMP:
            version[rec.worker] = rec.k
        if on_record is not None:
            on_record(rec, out)
    return version


def final_params(rings, version, serial=False):
    """Newest parameters of every worker: ring slot version mod D, or - serial approach, whose rings
    carry one more slot per worker - the current-parameter slot."""
    if serial:
        return np.stack([rings[i, rings.shape[1] - 1] for i in range(rings.shape[0])])
    D = rings.shape[1]
    return np.stack([rings[i, version[i] % D] for i in range(rings.shape[0])])
