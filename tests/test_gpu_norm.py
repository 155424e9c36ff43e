"""Parity of the fused RMSNorm + AbsMax quantiser (forward and backward) against the CPU oracle.

Bars: rstd, the stored normalised activations, gamma, the INT8 codes and q / gamma bit-exact (every
decision is taken in fp32 on both sides; the mean of squares is an fp64 sum on both sides, whose order can
move rstd only when the fp64 value sits within 1e-16 of an fp32 rounding boundary); the backward within
max|a-b| / max|b| <= 1e-5 (fp32 I/O) or 2e-2 (bf16 I/O).
"""
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {False: 1e-5, True: 2e-2}


def dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def relerr(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def say(msg):
    print(msg, flush=True)


def _inputs(seed, T, K, bf16):
    rng = np.random.default_rng(seed)
    X = wl.activations(rng, T, K, outlier_frac=0.01, outlier_scale=20.0, bf16=bf16)
    g = wl.normal(rng, (K,), 0.1, bf16) + np.float32(1.0)
    if bf16:
        g = torch.from_numpy(g).to(torch.bfloat16).float().numpy()
    return X, g


@pytest.mark.parametrize("T,K,bf16", [(64, 256, False), (300, 2048, True), (37, 5504, True), (9, 4096, False),
                                     (5, 8192, True), (3, 32, True), (130, 4096, True), (0, 64, True), (257, 2048, False)])
def test_rmsnorm_quant_fwd_bit_exact(T, K, bf16):
    say(f"rmsnorm_quant_fwd T={T} K={K} bf16={bf16}")
    X, g = _inputs(700 + T, T, K, bf16)
    if T > 2:
        X[1] = 0.0                                   # a zero row: eps decides rstd, the codes are zero
        X[2, 5] = np.abs(X[2]).max() * 4             # a dominant channel
    eps = 1e-6
    Xn, Xq, gamma, Xt, rstd = pq.rmsnorm_quant_fwd(dev(X, bf16), dev(g, bf16), eps)
    torch.cuda.synchronize()
    ref = po.rmsnorm_quant_fwd(X, g, eps, bf16=bf16)
    assert np.array_equal(host(rstd), ref["rstd"])
    assert np.array_equal(host(Xn), ref["Xn"])
    assert np.array_equal(host(gamma), ref["gamma"])
    assert np.array_equal(host(Xq), ref["q"])
    xt_ref = torch.from_numpy(ref["Xt"]).to(torch.bfloat16).float().numpy()
    assert np.array_equal(host(Xt), xt_ref)


def test_rmsnorm_quant_fwd_equals_unfused_quantiser_and_optional_outputs():
    say("rmsnorm_quant_fwd vs quant_act of the stored normalised rows")
    T, K = 192, 2048
    X, g = _inputs(5, T, K, True)
    Xn, Xq, gamma, Xt, rstd = pq.rmsnorm_quant_fwd(dev(X, True), dev(g, True), 1e-6)
    Xq2, gamma2 = pq.quant_act(Xn)
    assert torch.equal(Xq, Xq2) and torch.equal(gamma, gamma2)
    _, Xq3, gamma3, xt3, r3 = pq.rmsnorm_quant_fwd(dev(X, True), dev(g, True), 1e-6, want_xn=False, want_xt=False, want_rstd=False)
    torch.cuda.synchronize()
    assert xt3 is None and r3 is None and torch.equal(Xq, Xq3) and torch.equal(gamma, gamma3)


@pytest.mark.parametrize("T,K,bf16", [(64, 256, False), (300, 2048, True), (37, 4096, True), (9, 2048, False), (3, 32, True),
                                     (1, 64, False), (1029, 1024, True)])
def test_rmsnorm_bwd_parity(T, K, bf16):
    say(f"rmsnorm_bwd T={T} K={K} bf16={bf16}")
    X, g = _inputs(900 + T, T, K, bf16)
    dXn = wl.normal(np.random.default_rng(33 + T), (T, K), 1.0, bf16)
    eps = 1e-6
    _, rstd_ref = po.rmsnorm(X, g, eps)
    dx_ref, dg_ref = po.rmsnorm_bwd(dXn, X, g, rstd_ref)
    dX, dg = pq.rmsnorm_bwd(dev(dXn, bf16), dev(X, bf16), dev(g, bf16), dev(rstd_ref))
    torch.cuda.synchronize()
    assert relerr(host(dX), dx_ref) <= TOL[bf16]
    assert relerr(host(dg), dg_ref) <= 1e-5          # dgain is fp32 whatever the I/O type


def test_rmsnorm_full_size_sampled_tokens():
    """Config-2 size (T=8192, K=2048, bf16), the launch the bench times: forward bit-exact and backward
    within tolerance on sampled tokens; dgain against the oracle on all tokens."""
    say("rmsnorm config-2 size")
    T, K = 8192, 2048
    X, g = _inputs(2, T, K, True)
    dXn = wl.normal(np.random.default_rng(8), (T, K), 1.0, True)
    Xn, Xq, gamma, Xt, rstd = pq.rmsnorm_quant_fwd(dev(X, True), dev(g, True), 1e-6)
    dX, dg = pq.rmsnorm_bwd(dev(dXn, True), dev(X, True), dev(g, True), rstd)
    torch.cuda.synchronize()
    rows = np.random.default_rng(0).choice(T, 64, replace=False)
    ref = po.rmsnorm_quant_fwd(X[rows], g, 1e-6, bf16=True)
    assert np.array_equal(host(Xq)[rows], ref["q"]) and np.array_equal(host(gamma)[rows], ref["gamma"])
    assert np.array_equal(host(Xn)[rows], ref["Xn"]) and np.array_equal(host(rstd)[rows], ref["rstd"])
    _, rstd_all = po.rmsnorm(X, g, 1e-6)
    dx_ref, dg_ref = po.rmsnorm_bwd(dXn, X, g, rstd_all)
    assert relerr(host(dX)[rows], dx_ref[rows]) <= 2e-2
    assert relerr(host(dg), dg_ref) <= 1e-5


# ---------------------------------------------------------------------------- the linear with its normalisation
def _run_linear_norm(c, gain, eps, bf16, alpha, beta):
    T, K, N, r = c["tokens"], c["d_in"], c["d_out"], c["hp_rank"]
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_BF16 if bf16 else pq.PQ_F32, alpha=alpha, beta=beta)
    bufs = pq.LinearNormBuffers(desc)
    X, W, dY, g = dev(c["X"], bf16), dev(c["W"], bf16), dev(c["dY"], bf16), dev(gain, bf16)
    A = dev(c["A"], bf16) if r else None
    B = dev(c["B"], bf16) if r else None
    io = torch.bfloat16 if bf16 else torch.float32
    Y = torch.empty((T, N), dtype=io, device="cuda")
    dX = torch.empty((T, K), dtype=io, device="cuda")
    dg = torch.empty((K,), dtype=torch.float32, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda") if r else None
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda") if r else None
    dab = torch.empty((2,), dtype=torch.float32, device="cuda")
    pq.linear_norm_fwd(desc, X, g, eps, W, Y, bufs, A=A, B=B)
    pq.linear_norm_bwd(desc, dY, X, g, W, bufs, dX, dg, dW, dab, A=A, B=B, dA=dA, dB=dB)
    torch.cuda.synchronize()
    out = dict(Y=host(Y), dX=host(dX), dg=host(dg), dW=host(dW), dab=host(dab))
    if r:
        out.update(dA=host(dA), dB=host(dB))
    return out


def _oracle_linear_norm(c, gain, eps, bf16, alpha, beta):
    r = c["hp_rank"]
    kw = dict(A=c["A"], B=c["B"]) if r else {}
    f = po.rmsnorm_quant_fwd(c["X"], gain, eps, bf16=bf16)
    fw = po.linear_fwd(f["Xn"], c["W"], alpha, beta, **kw)
    gr = po.linear_bwd(c["dY"], f["Xn"], c["W"], alpha, beta, fw, **kw)
    dXn = po._round_io(gr["dX"], bf16)                     # the library hands dX of the linear over in the I/O type
    dx, dg = po.rmsnorm_bwd(dXn, c["X"], gain, f["rstd"])
    dY = c["dY"].astype(np.float64)           # natural scales of the two scalar gradients (root-sum-square of their terms)
    sb = max(abs(gr["dbeta"]), np.sqrt(((dY * fw["Y1_nobeta"]) ** 2).sum()))
    sa = max(abs(gr["dalpha"]), np.sqrt(((dY * fw["Yhp"]) ** 2).sum()), 1e-30)
    out = dict(Y=fw["Y"], dX=dx, dg=dg, dW=gr["dW"], dab=np.array([gr["dalpha"], gr["dbeta"]]), dab_scale=np.array([sa, sb]))
    if r:
        out.update(dA=gr["dA"], dB=gr["dB"])
    return out


@pytest.mark.parametrize("T,K,N,r,bf16", [(64, 256, 256, 16, False), (333, 544, 416, 24, True), (70, 96, 64, 0, True),
                                         (300, 2048, 512, 0, False), (513, 1024, 768, 64, True)])
def test_linear_norm_parity(T, K, N, r, bf16):
    say(f"linear with normalisation T={T} K={K} N={N} r={r} bf16={bf16}")
    c = wl.linear_case(1200 + T + r, T, K, N, hp_rank=r, bf16=bf16, outlier_frac=0.02, outlier_scale=10.0)
    # un-normalised inputs: rows of very different length
    scale = np.exp2(np.random.default_rng(T).integers(-3, 4, size=(T, 1))).astype(np.float32)
    c["X"] = (c["X"] * scale).astype(np.float32)
    rng = np.random.default_rng(77)
    gain = wl.normal(rng, (K,), 0.1, False) + np.float32(1.0)
    if bf16:
        gain = torch.from_numpy(gain).to(torch.bfloat16).float().numpy()
    got = _run_linear_norm(c, gain, 1e-6, bf16, 2.0, 0.2)
    ref = _oracle_linear_norm(c, gain, 1e-6, bf16, 2.0, 0.2)
    tol = TOL[bf16]
    for k in ref:
        if k == "dab_scale":
            continue
        e = float(np.max(np.abs(got[k] - ref[k]) / ref["dab_scale"])) if k == "dab" else relerr(got[k], ref[k])
        say(f"  {k}: {e:.2e}")
        assert e <= tol, k
