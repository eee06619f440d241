"""Seeded synthetic inputs: graphs, mixing matrices, slow-worker sets, data.

This module makes inputs only; it contains none of the method's arithmetic and
imports neither the HIP library nor the CPU oracle.  Whatever it produces is
handed, unchanged, to both.

The five workloads stand in for the paper's experiments (Section 7): a dense
and a very sparse linear SVM in place of the web-spam set, a flat 25 M
parameter vector in place of the CNN, 4 to 64 workers on rings, tori and a ring
with chords, random Exp(1) / deterministic 2-5x slowdowns in place of the
paper's "6x with probability 1/n" and "one worker 4x slower".
"""
import math

import numpy as np
import torch

M64 = (1 << 64) - 1
STREAM_GRAPH = 3
STREAM_SLOWSET = 4
STREAM_DATA = 5

DELAY_NONE, DELAY_EXP1, DELAY_BERNOULLI6, DELAY_TABLE = 0, 1, 2, 3
DEFAULT_SEED = 190201064


def _sm64(z):
    z = (z + 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _mix(seed, stream, a, b, c):
    h = _sm64(seed & M64)
    for w in (stream, a, b, c):
        h = _sm64(h ^ (w & M64))
    return h


# ---------------------------------------------------------------- graphs ----
def ring(n):
    if n == 1:
        return [[]]
    if n == 2:
        return [[1], [0]]
    return [sorted({(i - 1) % n, (i + 1) % n}) for i in range(n)]


def torus(r, c):
    nb = []
    for a in range(r):
        for b_ in range(c):
            s = {((a - 1) % r) * c + b_, ((a + 1) % r) * c + b_,
                 a * c + (b_ - 1) % c, a * c + (b_ + 1) % c}
            s.discard(a * c + b_)
            nb.append(sorted(s))
    return nb


def ring_based(n):
    """Ring plus an edge from every node to the most distant one (Section 7.3.1, graph 2); n even."""
    return [sorted({(i - 1) % n, (i + 1) % n, (i + n // 2) % n} - {i}) for i in range(n)]


def double_ring(n):
    """Two ring-based graphs of n/2 nodes joined node to node (Section 7.3.1, graph 3)."""
    h = n // 2
    half = ring_based(h)
    nb = []
    for side in (0, 1):
        for i in range(h):
            nb.append(sorted([j + side * h for j in half[i]] + [i + (1 - side) * h]))
    return nb


def complete(n):
    return [[j for j in range(n) if j != i] for i in range(n)]


def directed_cycle(order):
    """order = [v0, v1, ...]: edges v0 -> v1 -> ... -> v0; returns in-neighbours."""
    n = len(order)
    nb = [[] for _ in range(n)]
    for p, v in enumerate(order):
        nb[order[(p + 1) % n]].append(v)
    return nb


def ring_with_chords(n, chords_per_node, seed):
    """Ring plus, for every node in turn, `chords_per_node` undirected chords to
    seeded targets that are neither the node itself nor already adjacent."""
    adj = [set(l) for l in ring(n)]
    for i in range(n):
        for c in range(chords_per_node):
            t = 0
            while True:
                j = _mix(seed, STREAM_GRAPH, i, c, t) % n
                t += 1
                if j != i and j not in adj[i]:
                    break
                if t > 64 * n:
                    raise RuntimeError("no free chord target")
            adj[i].add(j)
            adj[j].add(i)
    return [sorted(a) for a in adj]


def to_csr(in_nbrs):
    row_ptr = np.zeros(len(in_nbrs) + 1, dtype=np.int32)
    for i, l in enumerate(in_nbrs):
        row_ptr[i + 1] = row_ptr[i] + len(l)
    col = np.array([j for l in in_nbrs for j in l], dtype=np.int32)
    return row_ptr, col


def uniform_weights(in_nbrs):
    """Every update has the same influence: 1 / (|N_in| + 1) counting the
    self-loop.  W[j][i] = weight of sender j at receiver i."""
    n = len(in_nbrs)
    W = np.zeros((n, n), dtype=np.float32)
    for i, l in enumerate(in_nbrs):
        for j in list(l) + [i]:
            W[j][i] = np.float32(1.0 / (len(l) + 1))
    return W


def metropolis_weights(in_nbrs):
    """Symmetric graph: W_ij = 1 / (1 + max(deg_i, deg_j)), W_ii = 1 - sum."""
    n = len(in_nbrs)
    W = np.zeros((n, n), dtype=np.float64)
    for i, l in enumerate(in_nbrs):
        for j in l:
            W[j][i] = 1.0 / (1 + max(len(l), len(in_nbrs[j])))
    for i in range(n):
        W[i][i] = 1.0 - W[:, i].sum()
    return W.astype(np.float32)


def slow_workers(seed, n, count):
    """First `count` entries of a seeded permutation of the workers."""
    keyed = sorted(range(n), key=lambda i: (_mix(seed, STREAM_SLOWSET, i, 0, 0), i))
    return keyed[:count]


# ------------------------------------------------------------------ data ----
def _gen(seed, tag, worker, device):
    g = torch.Generator(device=device)
    g.manual_seed(_mix(seed, STREAM_DATA, tag, worker, 0) & 0x7FFFFFFFFFFFFFFF)
    return g


def initial_params(seed, d, variance=0.01, device="cpu"):
    g = _gen(seed, 1, 0, device)
    return torch.randn(d, generator=g, device=device, dtype=torch.float32) * math.sqrt(variance)


def hidden_w(seed, d, device="cpu"):
    g = _gen(seed, 2, 0, device)
    return torch.randn(d, generator=g, device=device, dtype=torch.float32)


def _labels(score, g, device):
    eps = torch.randn(score.shape, generator=g, device=device, dtype=torch.float32)
    y = torch.sign(score + 0.1 * eps)
    y[y == 0] = 1.0
    return y


def dense_svm_data(seed, worker, rows, d, wstar, device="cpu", chunk_rows=4096):
    """x ~ N(0,1), y = sign(<w*, x> + 0.1 eps).  Returns (X [rows, d], y [rows])."""
    g = _gen(seed, 3, worker, device)
    X = torch.empty((rows, d), device=device, dtype=torch.float32)
    y = torch.empty(rows, device=device, dtype=torch.float32)
    for lo in range(0, rows, chunk_rows):
        hi = min(rows, lo + chunk_rows)
        X[lo:hi].normal_(generator=g)
        y[lo:hi] = _labels(X[lo:hi] @ wstar, g, device)
    return X, y


_zipf_cdf_cache = {}


def _zipf_cdf(d, a, device):
    key = (d, a, str(device))
    if key not in _zipf_cdf_cache:
        r = torch.arange(1, d + 1, device=device, dtype=torch.float64)
        c = torch.cumsum(r.pow_(-a), 0)
        _zipf_cdf_cache.clear()
        _zipf_cdf_cache[key] = c / c[-1]
    return _zipf_cdf_cache[key]


def csr_svm_data(seed, worker, rows, d, nnz, zipf_a, wstar, device="cpu", chunk_rows=8192):
    """CSR features: every row has `nnz` distinct columns, the first nnz distinct
    values of a Zipf(zipf_a) stream over ranks 1..d (column = rank - 1), sorted
    ascending; values ~ N(0,1); labels from the hidden w*.  Returns
    (rowptr int64 [rows+1], col int32 [rows*nnz], val fp32, y fp32)."""
    g = _gen(seed, 4, worker, device)
    cdf = _zipf_cdf(d, float(zipf_a), device)
    cols = torch.empty((rows, nnz), device=device, dtype=torch.int32)
    big = torch.iinfo(torch.int64).max
    for lo in range(0, rows, chunk_rows):
        hi = min(rows, lo + chunk_rows)
        n = hi - lo
        M = 3 * nnz
        while True:
            u = torch.rand((n, M), generator=g, device=device, dtype=torch.float64)
            cand = torch.searchsorted(cdf, u.reshape(-1)).reshape(n, M).clamp_(max=d - 1)
            order = torch.arange(M, device=device).expand(n, M)
            key = cand * M + order                       # sort by (column, draw order)
            skey, _ = torch.sort(key, dim=1)
            scol, sord = skey // M, skey % M
            first = torch.ones_like(scol, dtype=torch.bool)
            first[:, 1:] = scol[:, 1:] != scol[:, :-1]
            if int(first.sum(1).min()) >= nnz:
                break
            M *= 2
        rank = torch.where(first, sord, torch.full_like(sord, big))
        _, pick = torch.sort(rank, dim=1)
        chosen = torch.gather(scol, 1, pick[:, :nnz])
        cols[lo:hi] = torch.sort(chosen, dim=1)[0].to(torch.int32)
    val = torch.randn((rows, nnz), generator=g, device=device, dtype=torch.float32)
    score = (val * wstar[cols.long()]).sum(1)
    y = _labels(score, g, device)
    rowptr = torch.arange(0, rows + 1, device=device, dtype=torch.int64) * nnz
    return rowptr, cols.reshape(-1), val.reshape(-1), y


# --------------------------------------------------------------- configs ----
def config(n, seed=DEFAULT_SEED, **over):
    """The five synthetic workloads (1-based).  Keyword overrides (d, rows, K,
    batch ...) give the scaled-down parity cases; the schedule depends on none
    of d, rows or the data."""
    if n == 1:
        nb = ring(4)
        c = dict(name="cfg1-ring4-dense", in_nbrs=nb, W=uniform_weights(nb), s=1, b=0,
                 delay_kind=DELAY_NONE, mult=None, skip_on=False, model="dense", d=1024,
                 rows=4096, batch=64, lr=0.01, lam=1e-4, K=50)
    elif n == 2:
        nb = ring(16)
        mult = [1.0] * 16
        for w in slow_workers(seed, 16, 1):
            mult[w] = 4.0
        c = dict(name="cfg2-ring16-dense", in_nbrs=nb, W=uniform_weights(nb), s=2, b=0,
                 delay_kind=DELAY_EXP1, mult=mult, skip_on=True, model="dense", d=65536,
                 rows=16384, batch=128, lr=0.01, lam=1e-4, K=200)
    elif n == 3:
        nb = torus(4, 4)
        c = dict(name="cfg3-torus16-csr", in_nbrs=nb, W=uniform_weights(nb), s=3, b=1,
                 delay_kind=DELAY_EXP1, mult=None, skip_on=False, model="csr", d=1 << 20,
                 rows=32768, nnz=64, zipf_a=1.1, batch=256, lr=0.01, lam=1e-4, K=200)
    elif n == 4:
        nb = ring_with_chords(32, 2, seed)
        mult = [1.0] * 32
        for w in slow_workers(seed, 32, 2):
            mult[w] = 3.0
        c = dict(name="cfg4-chords32-mix", in_nbrs=nb, W=metropolis_weights(nb), s=4, b=1,
                 delay_kind=DELAY_NONE, mult=mult, skip_on=True, model="synth",
                 d=25_000_000, grad_var=1e-3, lr=0.01, lam=0.0, K=100, batch=0, rows=0)
    elif n == 5:
        nb = torus(8, 8)
        mult = [1.0] * 64
        for p, w in enumerate(slow_workers(seed, 64, 16)):
            mult[w] = float(2 + p % 4)
        c = dict(name="cfg5-torus64-csr", in_nbrs=nb, W=uniform_weights(nb), s=8, b=2,
                 delay_kind=DELAY_EXP1, mult=mult, skip_on=True, model="csr", d=1 << 24,
                 rows=65536, nnz=128, zipf_a=1.05, batch=512, lr=0.01, lam=1e-4, K=100)
    else:
        raise ValueError("config 1..5")
    c.update(N=len(nb), seed=seed, max_ig=0, max_skip=10, trigger=1)
    c.update(over)
    return c
