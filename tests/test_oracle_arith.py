"""Pins for the oracle's arithmetic: closed forms and library routines.

None of these needs a GPU.
"""
import numpy as np
import pytest

from oracle import arith, protocol, rng
from paper_1902_01064_amd import inputs


def _run(nb, W, s, b, K, **kw):
    h = protocol.Hop(nb, W, s, b, K, check=False, **kw)
    return h, h.run()


def _svm_problem(N, rows, d, seed=1):
    wstar = inputs.hidden_w(seed, d)
    X, y = [], []
    for i in range(N):
        Xi, yi = inputs.dense_svm_data(seed, i, rows, d, wstar)
        X.append(Xi.numpy())
        y.append(yi.numpy())
    return X, y, inputs.initial_params(seed, d).numpy()


# ---- Figure "Standard Decentralized Training": X_{k+1} = W^T X_k - eta G_k -------
@pytest.mark.parametrize("kind", [rng.DELAY_NONE, rng.DELAY_EXP1])
def test_standard_mode_equals_dense_recurrence(kind):
    nb = inputs.ring_with_chords(6, 1, 4)
    W = inputs.metropolis_weights(nb)
    N, d, K, B, lam, eta, seed = 6, 40, 12, 8, 1e-2, 0.05, 21
    X, y, p0 = _svm_problem(N, 64, d, seed)
    h, recs = _run(nb, W, 0, 0, K, seed=seed, delay_kind=kind, mult=[1, 3, 1, 1, 2, 1])
    rings = arith.init_rings(p0, N, h.D)
    ver = arith.execute(recs, rings, arith.GradSvmDense(seed, X, y, B, lam), eta)
    got = arith.final_params(rings, ver).astype(np.float64)

    # the recurrence, in fp64 with numpy only
    Xk = np.tile(p0.astype(np.float64), (N, 1))
    W64 = W.astype(np.float64)
    for k in range(K):
        G = np.zeros_like(Xk)
        for i in range(N):
            rows = [rng.mix(seed, rng.STREAM_BATCH, i, k, m) % 64 for m in range(B)]
            Xb, yb = X[i][rows].astype(np.float64), y[i][rows].astype(np.float64)
            act = (yb * (Xb @ Xk[i])) < 1.0
            G[i] = lam * Xk[i] - (Xb * (yb * act)[:, None]).sum(0) / B
        Xk = W64.T @ Xk - float(np.float32(eta)) * G
    # fp32 storage per step on one side only: K steps of 2^-24 relative rounding
    assert np.max(np.abs(got - Xk)) <= 2e-6 * np.max(np.abs(Xk))


# ---- doubly stochastic W, zero gradient: mean preserved, X_k = (W^T)^k X_0 --------
@pytest.mark.parametrize("nb", [inputs.ring(4), inputs.torus(4, 4), inputs.ring_with_chords(12, 1, 2)])
def test_zero_gradient_is_matrix_power_and_keeps_the_mean(nb):
    N, d, K = len(nb), 16, 9
    W = inputs.metropolis_weights(nb)
    assert np.allclose(W.sum(0), 1, atol=1e-6) and np.allclose(W.sum(1), 1, atol=1e-6)
    X0 = np.random.default_rng(0).normal(size=(N, d)).astype(np.float32)
    h, recs = _run(nb, W, 0, 0, K)
    rings = arith.init_rings(X0, N, h.D)
    means = []
    arith.execute(recs, rings, arith.GradZero(), 0.1,
                  on_record=lambda r, out: means.append(None))
    got = arith.final_params(rings, [K] * N).astype(np.float64)
    want = np.linalg.matrix_power(W.astype(np.float64).T, K) @ X0.astype(np.float64)
    assert np.allclose(got, want, atol=2e-6)
    assert np.allclose(got.mean(0), X0.astype(np.float64).mean(0), atol=1e-6)


# ---- consensus contracts at the rate of the second eigenvalue -----------------------
@pytest.mark.parametrize("shape,rho", [(("ring", 4), 1 / 3), (("ring", 16), 0.94925),
                                       (("torus", 4), 0.6), (("torus", 8), 0.88284)])
def test_consensus_contraction(shape, rho):
    nb = inputs.ring(shape[1]) if shape[0] == "ring" else inputs.torus(shape[1], shape[1])
    N = len(nb)
    W = inputs.uniform_weights(nb)
    # closed forms: ring (1 + 2 cos(2 pi / N)) / 3, torus (1 + 2 + 2 cos(2 pi / n)) / 5
    n = shape[1]
    closed = (1 + 2 * np.cos(2 * np.pi / n)) / 3 if shape[0] == "ring" else (3 + 2 * np.cos(2 * np.pi / n)) / 5
    assert abs(closed - rho) < 1e-5
    ev = np.sort(np.abs(np.linalg.eigvalsh(W.astype(np.float64))))
    assert abs(ev[-2] - rho) < 1e-5 and abs(ev[-1] - 1) < 1e-6
    K, d = 10, 8
    X0 = np.random.default_rng(1).normal(size=(N, d)).astype(np.float32)
    s = 1                                                  # lock-step: staleness mode == standard
    h, recs = _run(nb, W, s, 0, K)
    rings = arith.init_rings(X0, N, h.D)
    dev = [np.linalg.norm(X0 - X0.mean(0))]
    done = [0]

    def watch(r, out):
        done[0] += 1
        if done[0] % N == 0:
            k = done[0] // N
            cur = np.stack([rings[i, k % h.D] for i in range(N)]).astype(np.float64)
            dev.append(np.linalg.norm(cur - cur.mean(0)))
    arith.execute(recs, rings, arith.GradZero(), 0.0, on_record=watch)
    for k in range(1, K + 1):
        assert dev[k] <= rho ** k * dev[0] * (1 + 1e-5) + 1e-6


# ---- identical replicas stay fixed in every mode -------------------------------------
@pytest.mark.parametrize("cfgn", [2, 3, 4, 5])
def test_identical_replicas_are_a_fixed_point(cfgn):
    c = inputs.config(cfgn)
    h, recs = _run(c["in_nbrs"], c["W"], c["s"], c["b"], 25, skip_on=c["skip_on"],
                   seed=c["seed"], delay_kind=c["delay_kind"], mult=c["mult"])
    p0 = inputs.initial_params(3, 32).numpy()
    rings = arith.init_rings(p0, h.N, h.D)
    ver = arith.execute(recs, rings, arith.GradZero(), 0.01)
    got = arith.final_params(rings, ver)
    # weights sum to 1 up to their fp32 rounding: a few ulp per step at most
    assert np.max(np.abs(got - p0)) <= 25 * 4 * 2.0 ** -24 * np.max(np.abs(p0))
    for r in recs:
        assert abs(float(np.sum(r.w32.astype(np.float64))) - 1.0) < 3e-7 * len(r.w32)


# ---- the SVM subgradient -----------------------------------------------------------------
def test_svm_subgradient_matches_matmul_and_finite_differences():
    rs = np.random.default_rng(5)
    rows_n, d, B, lam = 50, 30, 16, 0.05
    X = rs.normal(size=(rows_n, d)).astype(np.float32)
    y = np.sign(rs.normal(size=rows_n)).astype(np.float32)
    w = (0.2 * rs.normal(size=d)).astype(np.float32)
    rows = rs.integers(0, rows_n, size=B)
    g, margins, act = arith.svm_subgradient_dense(X, y, w, rows, lam)
    Xb, yb = X[rows].astype(np.float64), y[rows].astype(np.float64)
    want = lam * w.astype(np.float64) - Xb.T @ (yb * ((yb * (Xb @ w.astype(np.float64))) < 1)) / B
    assert np.allclose(g, want, rtol=1e-12, atol=1e-14)
    assert act.any() and (~act).any()

    def loss(v):
        return 0.5 * lam * v @ v + np.maximum(0.0, 1.0 - yb * (Xb @ v)).sum() / B
    assert np.min(np.abs(1 - margins)) > 1e-3              # away from the kink
    w64 = w.astype(np.float64)
    for c in range(d):
        e = np.zeros(d)
        e[c] = 1e-6
        fd = (loss(w64 + e) - loss(w64 - e)) / 2e-6
        assert abs(fd - g[c]) < 1e-6


def test_csr_subgradient_equals_dense_on_the_same_matrix():
    seed, rows_n, d, nnz, B, lam = 8, 64, 200, 7, 24, 1e-3
    wstar = inputs.hidden_w(seed, d)
    rowptr, col, val, y = [t.numpy() for t in inputs.csr_svm_data(seed, 0, rows_n, d, nnz, 1.1, wstar)]
    assert rowptr[-1] == rows_n * nnz and col.dtype == np.int32
    for r in range(rows_n):
        c = col[rowptr[r]:rowptr[r + 1]]
        assert np.all(np.diff(c) > 0)                      # distinct, ascending
    dense = np.zeros((rows_n, d), dtype=np.float32)
    for r in range(rows_n):
        dense[r, col[rowptr[r]:rowptr[r + 1]]] = val[rowptr[r]:rowptr[r + 1]]
    w = inputs.initial_params(seed, d, 0.5).numpy()
    rows = rng.batch_rows(seed, 0, 3, B, rows_n)
    g1, m1, a1 = arith.svm_subgradient_csr(rowptr, col, val, y, w, rows, lam)
    g2, m2, a2 = arith.svm_subgradient_dense(dense, y, w, rows, lam)
    assert np.allclose(m1, m2, rtol=1e-12) and (a1 == a2).all()
    assert np.allclose(g1, g2, rtol=1e-12, atol=1e-15)


# ---- inputs that the method relies on ---------------------------------------------------------
def test_metropolis_weights_are_doubly_stochastic():
    c = inputs.config(4)
    W = c["W"].astype(np.float64)
    assert np.allclose(W, W.T) and (W >= 0).all()
    assert np.allclose(W.sum(0), 1, atol=1e-6) and np.allclose(W.sum(1), 1, atol=1e-6)
    nb = c["in_nbrs"]
    assert all(i in nb[j] for i in range(32) for j in nb[i])
    assert min(len(l) for l in nb) >= 4 and sum(len(l) for l in nb) == 32 * 2 + 2 * 64
    for i in range(32):
        assert all(W[j][i] > 0 for j in nb[i]) and W[i][i] > 0
        assert np.count_nonzero(W[:, i]) == len(nb[i]) + 1


def test_synthetic_gradient_statistics_and_reproducibility():
    cols = np.arange(200_000)
    g = rng.synth_grad(5, 3, 17, cols, 1e-3)
    assert g.dtype == np.float32
    assert abs(g.mean()) < 3e-4 and abs(g.var() / 1e-3 - 1) < 0.02
    kurt = np.mean((g / g.std()) ** 4)
    assert abs(kurt - 3.0) < 0.15                           # close to normal (sum of 12 uniforms: 2.9)
    assert np.array_equal(g[1234:1300], rng.synth_grad(5, 3, 17, cols[1234:1300], 1e-3))
    g2 = rng.synth_grad(5, 3, 18, cols, 1e-3)
    assert abs(np.corrcoef(g, g2)[0, 1]) < 0.01
    assert abs(np.corrcoef(g[:-1], g[1:])[0, 1]) < 0.01


def test_batch_rows_are_uniform_and_keyed_by_iteration():
    r = np.concatenate([rng.batch_rows(1, 2, k, 64, 100) for k in range(200)])
    assert r.min() >= 0 and r.max() < 100
    assert np.abs(np.bincount(r, minlength=100) / len(r) - 0.01).max() < 0.004
    assert not np.array_equal(rng.batch_rows(1, 2, 5, 64, 100), rng.batch_rows(1, 2, 6, 64, 100))


# ---- log loss (Section 7.2: "We use log loss for SVM instead of hinge loss") -------------------------
def test_log_loss_gradient_matches_finite_differences_and_limits():
    rs = np.random.default_rng(9)
    rows_n, d, B, lam = 40, 25, 12, 0.03
    X = rs.normal(size=(rows_n, d)).astype(np.float32)
    y = np.sign(rs.normal(size=rows_n)).astype(np.float32)
    w = (0.3 * rs.normal(size=d)).astype(np.float32)
    rows = rs.integers(0, rows_n, size=B)
    g, margins, _ = arith.svm_subgradient_dense(X, y, w, rows, lam, loss="log")
    Xb, yb = X[rows].astype(np.float64), y[rows].astype(np.float64)

    def loss(v):
        return 0.5 * lam * v @ v + np.log1p(np.exp(-yb * (Xb @ v))).sum() / B
    w64 = w.astype(np.float64)
    for c in range(d):
        e = np.zeros(d)
        e[c] = 1e-6
        assert abs((loss(w64 + e) - loss(w64 - e)) / 2e-6 - g[c]) < 1e-7
    # far on the wrong side of the margin the log loss pulls like an active hinge sample, far on the
    # right side not at all
    c_neg, _ = arith.loss_coefficients(np.array([1.0, -1.0]), np.array([-50.0, -50.0]), 4, "log")
    c_pos, _ = arith.loss_coefficients(np.array([1.0, -1.0]), np.array([800.0, 50.0]), 4, "log")
    assert np.allclose(c_neg, [0.25, -0.25], rtol=1e-12) and np.all(np.abs(c_pos) < 1e-20)
    # csr agrees with dense on the same matrix
    wstar = inputs.hidden_w(3, 200)
    rowptr, col, val, yy = [t.numpy() for t in inputs.csr_svm_data(3, 0, 64, 200, 7, 1.1, wstar)]
    dense = np.zeros((64, 200), dtype=np.float32)
    for r in range(64):
        dense[r, col[rowptr[r]:rowptr[r + 1]]] = val[rowptr[r]:rowptr[r + 1]]
    wv = inputs.initial_params(3, 200, 0.5).numpy()
    rr = rng.batch_rows(3, 0, 1, 20, 64)
    g1, _, _ = arith.svm_subgradient_csr(rowptr, col, val, yy, wv, rr, 1e-3, loss="log")
    g2, _, _ = arith.svm_subgradient_dense(dense, yy, wv, rr, 1e-3, loss="log")
    assert np.allclose(g1, g2, rtol=1e-12, atol=1e-15)


# ---- momentum (Section 7.2: momentum 0.9) ------------------------------------------------------------
def test_momentum_closed_forms():
    nb = inputs.ring(4)
    W = inputs.uniform_weights(nb)
    N, d, K, eta, mu = 4, 6, 9, 0.05, 0.9
    h, recs = _run(nb, W, 1, 0, K)
    p0 = np.linspace(-1, 1, d).astype(np.float32)
    gconst = np.linspace(0.5, -0.5, d)

    class Const:
        def __call__(self, i, k, w):
            return gconst
    # identical replicas + the same constant gradient everywhere: averaging is the identity, so
    # x_K = x_0 - eta g sum_{t=1..K} (1 - mu^t) / (1 - mu)
    rings = arith.init_rings(p0, N, h.D)
    vel = np.zeros((N, d), dtype=np.float32)
    ver = arith.execute(recs, rings, Const(), eta, vel=vel, mu=mu)
    got = arith.final_params(rings, ver).astype(np.float64)
    mu32, eta32 = float(np.float32(mu)), float(np.float32(eta))
    geo = sum((1 - mu32 ** t) / (1 - mu32) for t in range(1, K + 1))
    want = p0.astype(np.float64) - eta32 * gconst * geo
    assert np.allclose(got, np.tile(want, (N, 1)), atol=2e-6)
    assert np.allclose(vel, np.tile(gconst * (1 - mu32 ** K) / (1 - mu32), (N, 1)), atol=1e-6)
    # mu = 0 is the plain update, bit for bit
    r1 = arith.init_rings(p0, N, h.D)
    r2 = arith.init_rings(p0, N, h.D)
    arith.execute(recs, r1, Const(), eta)
    arith.execute(recs, r2, Const(), eta, vel=np.zeros((N, d), dtype=np.float32), mu=0.0)
    assert np.array_equal(r1, r2)


def test_momentum_standard_mode_equals_dense_recurrence():
    """V_{k+1} = mu V_k + G_k, X_{k+1} = W^T X_k - eta V_{k+1} with numpy, under random delays."""
    nb = inputs.ring_with_chords(6, 1, 4)
    W = inputs.metropolis_weights(nb)
    N, d, K, B, lam, eta, mu, seed = 6, 30, 10, 8, 1e-2, 0.05, 0.9, 5
    X, y, p0 = _svm_problem(N, 64, d, seed)
    h, recs = _run(nb, W, 0, 0, K, seed=seed, delay_kind=rng.DELAY_EXP1, mult=[1, 2, 1, 1, 3, 1])
    rings = arith.init_rings(p0, N, h.D)
    vel = np.zeros((N, d), dtype=np.float32)
    ver = arith.execute(recs, rings, arith.GradSvmDense(seed, X, y, B, lam, loss="log"), eta, vel=vel, mu=mu)
    got = arith.final_params(rings, ver).astype(np.float64)
    Xk = np.tile(p0.astype(np.float64), (N, 1))
    Vk = np.zeros_like(Xk)
    W64, mu32, eta32 = W.astype(np.float64), float(np.float32(mu)), float(np.float32(eta))
    for k in range(K):
        G = np.zeros_like(Xk)
        for i in range(N):
            rows = [rng.mix(seed, rng.STREAM_BATCH, i, k, m) % 64 for m in range(B)]
            Xb, yb = X[i][rows].astype(np.float64), y[i][rows].astype(np.float64)
            G[i] = lam * Xk[i] - (Xb * (yb / (1 + np.exp(yb * (Xb @ Xk[i]))))[:, None]).sum(0) / B
        Vk = mu32 * Vk + G
        Xk = W64.T @ Xk - eta32 * Vk
    assert np.max(np.abs(got - Xk)) <= 3e-6 * np.max(np.abs(Xk))
