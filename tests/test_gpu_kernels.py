"""GPU parity of the single kernels, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import arith, rng
from paper_1902_01064_amd import hop, inputs
from parity import rel_err, strict_rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda:0"



def stream():
    return torch.cuda.current_stream().cuda_stream


def aligned(n, dtype=torch.float32):
    """Device tensor whose storage starts on a 16-byte boundary (torch gives 256+)."""
    t = torch.empty(n, dtype=dtype, device=DEV)
    assert t.data_ptr() % 16 == 0
    return t


# ------------------------------------------------------------------ Reduce + Apply ----
@pytest.mark.parametrize("d", [1, 3, 4, 5, 1023, 4096, 4097, 4096 * 3 + 2, (1 << 16) + 3, 1 << 20])
def test_mix_matches_oracle_over_sizes(d):
    print("mix d=%d" % d, flush=True)
    rs = np.random.default_rng(d)
    n_src, jobs, keep, want = 14, [], [], []
    pool = [aligned(d) for _ in range(n_src)]
    # replicas of one model: a common vector plus a few per cent of disagreement (what the rings
    # hold in a run); the last four sources are unrelated vectors, judged by the rounding bound
    base = rs.normal(size=d)
    host = [(base + 0.05 * rs.normal(size=d)).astype(np.float32) for _ in range(n_src - 4)]
    host += [rs.normal(size=d).astype(np.float32) for _ in range(4)]
    for t, h in zip(pool, host):
        t.copy_(torch.from_numpy(h))
    for A in (1, 2, 3, 5, 9, 12, 13, 14):
        for use_g in (True, False):
            related = A <= n_src - 4
            pick = rs.choice(n_src - 4 if related else n_src, size=A, replace=False)
            w = rs.dirichlet(np.ones(A)).astype(np.float32)
            g = aligned(d)
            gh = (0.03 * rs.normal(size=d)).astype(np.float32)
            g.copy_(torch.from_numpy(gh))
            out = aligned(d)
            out.fill_(float("nan"))
            keep += [g, out]
            jobs.append(dict(out=out.data_ptr(), g=g.data_ptr() if use_g else None, eta=0.05,
                             src=[pool[p].data_ptr() for p in pick], w=list(w)))
            mag = sum(abs(float(wa)) * np.abs(host[p].astype(np.float64)) for wa, p in zip(w, pick))
            mag = mag + (0.05 * np.abs(gh.astype(np.float64)) if use_g else 0.0)
            want.append((out, arith.reduce_apply([host[p] for p in pick], w, gh if use_g else None, 0.05),
                         related, (A + 2) * 2.0 ** -24 * mag))
    hop.hop_mix(jobs, d, stream())
    torch.cuda.synchronize()
    for out, ref, related, bound in want:
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        # an fp32 chain of A + 1 fused multiply-adds is within (A + 2) 2^-24 sum |terms| of the exact
        # sum (plus the oracle's own final rounding)
        assert np.all(np.abs(got.astype(np.float64) - ref) <= bound + 2.0 ** -24 * np.abs(ref))
        if related:
            assert rel_err(got, ref) <= 1e-5


def test_mix_many_jobs_full_width():
    """32 sources (the descriptor's limit) and more jobs than XCDs, ragged tail."""
    d = 50_001
    rs = np.random.default_rng(7)
    host = (rs.normal(size=d) + 0.05 * rs.normal(size=(40, d))).astype(np.float32)
    pool = torch.from_numpy(host).to(DEV)
    rows = [pool[i] for i in range(40)]
    # rows of a 2-D tensor with odd d are not 16-byte aligned: the library must refuse them
    with pytest.raises(hop.HopError) as e:
        hop.hop_mix([dict(out=rows[1].data_ptr(), g=None, eta=0.0, src=[rows[3].data_ptr()], w=[1.0])], d, stream())
    assert e.value.code == hop.HOP_ERR_INVALID_ARG
    src = [aligned(d) for _ in range(40)]
    for t, h in zip(src, host):
        t.copy_(torch.from_numpy(h))
    outs, jobs, want = [], [], []
    for j in range(21):
        A = 32 if j % 2 == 0 else 1 + j % 7
        pick = rs.choice(40, size=A, replace=False)
        w = rs.dirichlet(np.ones(A)).astype(np.float32)
        out = aligned(d)
        outs.append(out)
        jobs.append(dict(out=out.data_ptr(), g=None, eta=0.0, src=[src[p].data_ptr() for p in pick], w=list(w)))
        want.append(arith.reduce_apply([host[p] for p in pick], w, None, 0.0))
    hop.hop_mix(jobs, d, stream())
    torch.cuda.synchronize()
    for out, ref in zip(outs, want):
        assert rel_err(out.cpu().numpy(), ref) <= 1e-5
    hop.hop_mix([], d, stream())                              # empty launch is a no-op


# ----------------------------------------------------------------- synthetic gradient ----
@pytest.mark.parametrize("d", [1, 7, 512, 2049, (1 << 18) + 1])
def test_synth_grad_is_bit_exact(d):
    print("synth d=%d" % d, flush=True)
    g = aligned(d + 8)
    g.fill_(123.0)
    hop.hop_synth_grad(190201064, 5, 42, 1e-3, g.data_ptr(), d, stream())
    torch.cuda.synchronize()
    got = g.cpu().numpy()
    ref = rng.synth_grad(190201064, 5, 42, np.arange(d), 1e-3)
    assert np.array_equal(got[:d].view(np.uint32), ref.view(np.uint32))
    assert (got[d:] == 123.0).all()                           # nothing written past d


# ------------------------------------------------------------------- dense SVM gradient ----
def _check_gradient(got, ref, w, n_terms, mag):
    """A minibatch subgradient is a sum of +-x rows that largely cancel, so it is judged (a) by the
    rounding bound of an fp32 sum of n_terms + 1 products, (n + 3) 2^-24 sum |terms|, and (b) by
    what it does to the parameters: w - eta g at the 1e-5 bar of a single update (eta = 0.01)."""
    got64 = got.astype(np.float64)
    assert np.isfinite(got64).all()
    assert np.all(np.abs(got64 - ref) <= (n_terms + 3) * 2.0 ** -24 * mag + 1e-30)
    assert rel_err(w.astype(np.float64) - 0.01 * got64, w.astype(np.float64) - 0.01 * ref) <= 1e-5


def _near_tie_ok(margins, act_ref, act_gpu, scale):
    diff = act_ref != act_gpu
    return bool(np.all(np.abs(1.0 - margins[diff]) <= 1e-5 * (1.0 + scale[diff])))


@pytest.mark.parametrize("d,B,rows", [(1024, 64, 300), (1000, 1, 5), (1022, 37, 64), (65536 + 4, 128, 200),
                                      (16384 * 2, 1000, 1100), (6, 8, 8)])
def test_svm_grad_dense_matches_oracle(d, B, rows):
    print("dense d=%d B=%d" % (d, B), flush=True)
    seed = d + B
    ws = inputs.hidden_w(seed, d)
    X, y = inputs.dense_svm_data(seed, 0, rows, d, ws)
    w = (inputs.initial_params(seed, d, 0.01) + 0.02 * ws / np.sqrt(d)).contiguous()
    ridx = rng.batch_rows(seed, 0, 3, B, rows)
    lam = 1e-3
    Xd, yd, wd = X.to(DEV), y.to(DEV), w.to(DEV)
    rd = torch.from_numpy(ridx.astype(np.int32)).to(DEV)
    g, coef = aligned(d), aligned(B)
    scratch = aligned(hop.hop_grad_scratch_floats(d, B))
    hop.hop_svm_grad_dense(Xd.data_ptr(), yd.data_ptr(), wd.data_ptr(), rd.data_ptr(), B, d, lam,
                           g.data_ptr(), coef.data_ptr(), scratch.data_ptr(), stream())
    torch.cuda.synchronize()
    Xn, yn, wn = X.numpy(), y.numpy(), w.numpy()
    _, margins, act = arith.svm_subgradient_dense(Xn, yn, wn, ridx, lam)
    cg = coef.cpu().numpy()
    act_gpu = cg != 0
    scale = np.abs(Xn[ridx].astype(np.float64) * wn.astype(np.float64)).sum(1)
    assert _near_tie_ok(margins, act, act_gpu, scale)
    assert np.allclose(cg[act_gpu], yn[ridx][act_gpu] / B, rtol=1e-6)
    ref, _, _ = arith.svm_subgradient_dense(Xn, yn, wn, ridx, lam, active=act_gpu)
    mag = lam * np.abs(wn.astype(np.float64)) + np.abs(Xn[ridx][act_gpu].astype(np.float64)).sum(0) / B
    _check_gradient(g.cpu().numpy(), ref, wn, int(act_gpu.sum()), mag)


# --------------------------------------------------------------------- CSR SVM gradient ----
@pytest.mark.parametrize("d,nnz,B,rows,a", [(1 << 14, 64, 256, 1024, 1.1), (5000, 7, 33, 100, 1.05),
                                            (1 << 18, 128, 512, 2048, 1.05), (300, 130, 16, 40, 1.1)])
def test_svm_grad_csr_matches_oracle(d, nnz, B, rows, a):
    print("csr d=%d nnz=%d B=%d" % (d, nnz, B), flush=True)
    seed = d + nnz
    ws = inputs.hidden_w(seed, d)
    rowptr, col, val, y = inputs.csr_svm_data(seed, 0, rows, d, nnz, a, ws)
    w = (inputs.initial_params(seed, d, 0.01) + 0.05 * ws).contiguous()
    ridx = rng.batch_rows(seed, 0, 9, B, rows)
    lam = 1e-3
    dv = [t.to(DEV) for t in (rowptr, col, val, y, w)]
    rd = torch.from_numpy(ridx.astype(np.int32)).to(DEV)
    g, coef = aligned(d), aligned(B)
    hop.hop_svm_grad_csr(dv[0].data_ptr(), dv[1].data_ptr(), dv[2].data_ptr(), dv[3].data_ptr(),
                         dv[4].data_ptr(), rd.data_ptr(), B, d, lam, g.data_ptr(), coef.data_ptr(), stream())
    torch.cuda.synchronize()
    rp, cn, vn, yn, wn = rowptr.numpy(), col.numpy(), val.numpy(), y.numpy(), w.numpy()
    _, margins, act = arith.svm_subgradient_csr(rp, cn, vn, yn, wn, ridx, lam)
    cg = coef.cpu().numpy()
    act_gpu = cg != 0
    scale = np.array([np.abs(vn[rp[r]:rp[r + 1]].astype(np.float64) * wn[cn[rp[r]:rp[r + 1]]]).sum() for r in ridx])
    assert _near_tie_ok(margins, act, act_gpu, scale)
    ref, _, _ = arith.svm_subgradient_csr(rp, cn, vn, yn, wn, ridx, lam, active=act_gpu)
    mag = lam * np.abs(wn.astype(np.float64))
    for m, r in enumerate(ridx):
        if act_gpu[m]:
            np.add.at(mag, cn[rp[r]:rp[r + 1]], np.abs(vn[rp[r]:rp[r + 1]].astype(np.float64)) / B)
    _check_gradient(g.cpu().numpy(), ref, wn, int(act_gpu.sum()), mag)


def test_copy_and_download():
    a = torch.arange(4096, dtype=torch.float32, device=DEV)
    b = torch.zeros_like(a)
    hop.hop_copy(b.data_ptr(), a.data_ptr(), a.numel() * 4, stream())
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert np.array_equal(hop.hop_download(a.data_ptr() + 40, 10, stream()), np.arange(10, 20, dtype=np.float32))


def test_mix_with_velocity_for_every_width():
    """Momentum inside the fused kernel (v <- mu v + g in place, Apply with the new v) for the unrolled
    widths, the looped ones (A > 12) and the ragged tail, with and without a gradient."""
    d = 4099
    rs = np.random.default_rng(11)
    base = rs.normal(size=d)
    host = [(base + 0.05 * rs.normal(size=d)).astype(np.float32) for _ in range(24)]
    pool = [aligned(d) for _ in host]
    for t, h in zip(pool, host):
        t.copy_(torch.from_numpy(h))
    jobs, keep, want = [], [], []
    for A in (1, 2, 4, 7, 12, 13, 20):
        for use_g in (True, False):
            pick = rs.choice(len(host), size=A, replace=False)
            w = rs.dirichlet(np.ones(A)).astype(np.float32)
            gh = (0.03 * rs.normal(size=d)).astype(np.float32)
            vh = (0.1 * rs.normal(size=d)).astype(np.float32)
            g, vel, out = aligned(d), aligned(d), aligned(d)
            g.copy_(torch.from_numpy(gh))
            vel.copy_(torch.from_numpy(vh))
            out.fill_(float("nan"))
            keep += [g, vel, out]
            jobs.append(dict(out=out.data_ptr(), g=g.data_ptr() if use_g else None, eta=0.05, vel=vel.data_ptr(), mu=0.9,
                             src=[pool[p].data_ptr() for p in pick], w=list(w)))
            v64, v32 = arith.momentum_step(vh, gh if use_g else None, 0.9)
            want.append((out, vel, arith.reduce_apply([host[p] for p in pick], w, v64, 0.05), v32))
    hop.hop_mix(jobs, d, stream())
    torch.cuda.synchronize()
    for out, vel, ref, vref in want:
        assert rel_err(out.cpu().numpy(), ref) <= 1e-5
        assert rel_err(vel.cpu().numpy(), vref) <= 1e-6
