"""Parity of the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Bars: bit-exact for sign bits, packed words, INT8 codes, gamma, int32 accumulators and routing
indices; max|a-b| / max|b| <= 1e-5 for fp32 I/O and <= 2e-2 for bf16 I/O on outputs and gradients, the same bar
on the relative L2 error and, for gradients with an input-channel axis (dW, dA), on every input channel taken
by itself (tests/parity_metrics.py).  Gradients that need every token of a full-size workload are compared with
values the oracle wrote to tests/golden/full_size_*.npz (tests/golden/make_full_size_expected.py).
"""
import os
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl
from parity_metrics import relerr, report

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

TOL = {False: 1e-5, True: 2e-2}


def dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------- quantiser
@pytest.mark.parametrize("T,K,bf16", [(64, 256, False), (300, 2048, True), (37, 5504, True), (9, 4096, False),
                                     (5, 16384, True), (3, 32, True), (130, 4096, True), (0, 64, True),
                                     (8192, 2048, True), (8192, 5504, True)])   # full sizes of configs 2 and 3
def test_quant_act_bit_exact(T, K, bf16):
    say(f"quant_act T={T} K={K} bf16={bf16}")
    X = wl.activations(np.random.default_rng(100 + T), T, K, outlier_frac=0.01, outlier_scale=20.0, bf16=bf16)
    if T > 2:
        X[1] = 0.0                                   # a zero row
        X[2, 5] = np.abs(X[2]).max() * 2             # a positive extreme: saturates at 127
    Xq, g = pq.quant_act(dev(X, bf16))
    torch.cuda.synchronize()
    q_ref, g_ref = po.quant_act(X)
    assert np.array_equal(host(g), g_ref)
    assert np.array_equal(host(Xq), q_ref)


# ---------------------------------------------------------------------------- binariser / packer
@pytest.mark.parametrize("N,K,bf16,tr", [(256, 256, False, True), (2048, 2048, True, True), (72, 96, True, False),
                                        (160, 544, False, True), (96, 5504, True, True), (32, 32, True, True),
                                        (5504, 2048, True, True), (11008, 4096, True, False),   # configs 3 and 4
                                        # widths that are not whole words (Table 1: D_ff - r = 5076): padded with +1 bits
                                        (2048, 5076, True, True), (5076, 2048, True, True), (72, 44, False, True),
                                        (37, 96, True, True), (50, 20, True, True)])
def test_pack_sign_bit_exact(N, K, bf16, tr):
    say(f"pack_sign N={N} K={K} bf16={bf16} transposed={tr}")
    W = wl.normal(np.random.default_rng(200 + N), (N, K), 0.02, bf16)
    W[0, :7] = W[1, 3]                                # repeated values
    P, Pt, ml = pq.pack_sign(dev(W, bf16), transposed=tr)
    torch.cuda.synchronize()
    mu, lam = po.weight_stats(W)
    S = po.binarise(W, mu)
    assert host(ml)[0] == mu and host(ml)[1] == lam
    assert np.array_equal(host(P).view(np.uint32), po.pack_sign(S))
    if tr:
        assert np.array_equal(host(Pt).view(np.uint32), po.pack_sign(S.T.copy()))


def test_pack_sign_all_equal_weights_map_to_plus_one():
    W = np.full((64, 64), 0.125, np.float32)
    P, _, ml = pq.pack_sign(dev(W, True))
    torch.cuda.synchronize()
    assert host(ml).tolist() == [0.125, 0.125]
    assert np.all(host(P).view(np.uint32) == 0xFFFFFFFF)


# ---------------------------------------------------------------------------- int8 x 1-bit GEMM
@pytest.mark.parametrize("T,K,N", [(64, 256, 256), (333, 1056, 840), (1, 4096, 256), (130, 128, 136),
                                  (4101, 64, 4096), (257, 5504, 264)])
def test_onebit_acc_int32_bit_exact(T, K, N):
    say(f"onebit_acc T={T} K={K} N={N}")
    rng = np.random.default_rng(300 + T)
    q = rng.integers(-128, 128, size=(T, K)).astype(np.int8)
    S = np.where(rng.random((N, K)) < 0.5, 1, -1).astype(np.int8)
    P = po.pack_sign(S)
    acc = pq.onebit_acc(dev(q), dev(P.view(np.int32)), N)
    torch.cuda.synchronize()
    ref = po.onebit_acc(q, S)
    assert np.array_equal(host(acc).astype(np.int64), ref)


def test_onebit_acc_full_size_sampled_rows():
    """Config-2 size (8192 tokens, 2048 x 2048): every token's accumulator row depends on that token alone, so the
    oracle recomputes sampled rows; the comparison is bit-exact."""
    T, K, N = 8192, 2048, 2048
    say(f"onebit_acc full size T={T} K={K} N={N}, sampled rows")
    rng = np.random.default_rng(321)
    q = rng.integers(-128, 128, size=(T, K)).astype(np.int8)
    q[7] = -128                                       # the extreme accumulator magnitude 128 K stays below 2^24
    S = np.where(rng.random((N, K)) < 0.5, 1, -1).astype(np.int8)
    S[5] = -1
    acc = pq.onebit_acc(dev(q), dev(po.pack_sign(S).view(np.int32)), N)
    torch.cuda.synchronize()
    rows = np.array([0, 7, 255, 256, 4095, 4096, 8190, 8191] + list(rng.choice(T, 24, replace=False)))
    assert np.array_equal(host(acc)[rows].astype(np.int64), po.onebit_acc(q[rows], S))
    assert host(acc)[7, 5] == 128 * K


# ---------------------------------------------------------------------------- router
@pytest.mark.parametrize("T,K,E,k,bf16", [(200, 256, 8, 1, True), (77, 2048, 8, 2, True), (50, 96, 4, 2, False),
                                         (33, 64, 16, 3, True), (9, 64, 40, 2, False),
                                         (8192, 2048, 8, 1, True), (4096, 4096, 8, 2, True)])   # config 3; config-4 widths
def test_router_topk(T, K, E, k, bf16):
    say(f"router T={T} K={K} E={E} k={k} bf16={bf16}")
    rng = np.random.default_rng(400 + T)
    X = wl.activations(rng, T, K, bf16=bf16)
    Wr = wl.normal(rng, (E, K), 0.02, bf16)
    Wr[1] = Wr[0]                                    # exact ties between experts 0 and 1
    idx, gate, probs = pq.router_topk(dev(X, bf16), dev(Wr, bf16), k)
    torch.cuda.synchronize()
    i_ref, g_ref, p_ref, _ = po.router_topk(X, Wr, k)
    assert np.array_equal(host(idx), i_ref)
    assert relerr(host(gate), g_ref) < 1e-6 and relerr(host(probs), p_ref) < 1e-6


# ---------------------------------------------------------------------------- decoupled linear
def run_linear(c, bf16, alpha, beta, ste_tau=None, top_k=1):
    T, K, N, r, E = c["tokens"], c["d_in"], c["d_out"], c["hp_rank"], c.get("n_experts", 1)
    desc = pq.make_desc(T, K, N, hp_rank=r, n_experts=E, top_k=top_k, io_dtype=pq.PQ_BF16 if bf16 else pq.PQ_F32,
                        alpha=alpha, beta=beta, ste_mode=pq.PQ_STE_CLIP if ste_tau is not None else pq.PQ_STE_IDENTITY,
                        ste_tau=ste_tau or 0.0)
    bufs = pq.LinearBuffers(desc)
    dt = torch.bfloat16 if bf16 else torch.float32
    X, W, dY = dev(c["X"], bf16), dev(c["W"], bf16), dev(c["dY"], bf16)
    A = dev(c["A"], bf16) if r else None
    B = dev(c["B"], bf16) if r else None
    Wr = dev(c["Wr"], bf16) if (r and E > 1) else None
    Y = torch.empty((T, N), dtype=dt, device="cuda")
    pq.linear_fwd(desc, X, W, Y, bufs, A=A, B=B, Wr=Wr)
    dX = torch.empty((T, K), dtype=dt, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    dA = torch.empty(c["A"].shape, dtype=torch.float32, device="cuda") if r else None
    dB = torch.empty(c["B"].shape, dtype=torch.float32, device="cuda") if r else None
    dWr = torch.empty(c["Wr"].shape, dtype=torch.float32, device="cuda") if Wr is not None else None
    dab = torch.empty((2,), dtype=torch.float32, device="cuda")
    pq.linear_bwd(desc, dY, X, W, bufs, dX, dW, dab, A=A, B=B, Wr=Wr, dA=dA, dB=dB, dWr=dWr)
    torch.cuda.synchronize()
    return dict(Y=host(Y), dX=host(dX), dW=host(dW), dA=host(dA) if r else None, dB=host(dB) if r else None,
                dWr=host(dWr) if dWr is not None else None, dab=host(dab))


def scalar_errs(got_dab, dalpha, dbeta, sa, sb):
    """d alpha and d beta: error relative to the natural scale of the sum (the root-sum-square of its terms)."""
    return {"dalpha": abs(got_dab[0] - dalpha) / max(abs(dalpha), sa, 1e-30),
            "dbeta": abs(got_dab[1] - dbeta) / max(abs(dbeta), sb, 1e-30)}


def assert_errs(errs, tol):
    say("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert v <= tol, f"{k}: {v} > {tol}"


def check_linear(c, bf16, alpha=2.0, beta=0.2, ste_tau=None, top_k=1):
    r, E = c["hp_rank"], c.get("n_experts", 1)
    got = run_linear(c, bf16, alpha, beta, ste_tau, top_k)
    A, B = (c["A"], c["B"]) if r else (None, None)
    Wr = c["Wr"] if (r and E > 1) else None
    f = po.linear_fwd(c["X"], c["W"], alpha, beta, A=A, B=B, Wr=Wr, top_k=top_k)
    g = po.linear_bwd(c["dY"], c["X"], c["W"], alpha, beta, f, A=A, B=B, Wr=Wr,
                      ste_tau=np.inf if ste_tau is None else np.float32(ste_tau))
    errs = {}
    errs.update(report("Y", got["Y"], f["Y"]))
    errs.update(report("dX", got["dX"], g["dX"]))
    errs.update(report("dW", got["dW"], g["dW"], per_channel=True))
    if r:
        errs.update(report("dA", got["dA"], g["dA"], per_channel=True))
        errs.update(report("dB", got["dB"], g["dB"]))
    if Wr is not None:
        errs.update(report("dWr", got["dWr"], g["dWr"]))
    dY = c["dY"].astype(np.float64)
    errs.update(scalar_errs(got["dab"], g["dalpha"], g["dbeta"], np.sqrt(((dY * f["Yhp"]) ** 2).sum()),
                            np.sqrt(((dY * f["Y1_nobeta"]) ** 2).sum())))
    assert_errs(errs, TOL[bf16])
    return got


def test_linear_config1_fp32():
    say("linear config1 fp32 (T=64, 256x256, r=16)")
    check_linear(wl.config1(), False)


@pytest.mark.parametrize("T,K,N,r,bf16", [(333, 544, 416, 24, False), (333, 544, 416, 24, True),
                                         (70, 96, 64, 0, True), (70, 96, 64, 0, False),
                                         (1, 64, 32, 8, True), (600, 1056, 1312, 136, True),
                                         # rank 64 / 128 with ragged token and channel tiles: the streaming loop of the
                                         # fused GEMMs with a second contraction of one and of two whole steps
                                         (600, 1152, 1408, 64, True), (300, 640, 384, 128, True),
                                         # 7 and 5 contraction steps forward: the second contraction's tiles start in the
                                         # ring's last and second stage
                                         (300, 896, 384, 128, True), (280, 640, 896, 64, True),
                                         # many tokens at rank 128: the streaming rank-r kernel computes H (ragged last block)
                                         (1100, 640, 384, 128, True), (1024, 64, 256, 128, True),
                                         # 2048 tokens or more in whole 512-token ranges: dB and dA take the streaming pair kernel
                                         (2048, 192, 320, 128, True), (2560, 64, 64, 128, True)])
def test_linear_ragged_multi_tile(T, K, N, r, bf16):
    say(f"linear ragged T={T} K={K} N={N} r={r} bf16={bf16}")
    c = wl.linear_case(500 + T + r, T, K, N, hp_rank=r, bf16=bf16, outlier_frac=0.02, outlier_scale=10.0)
    check_linear(c, bf16)


@pytest.mark.parametrize("bf16", [False, True])
def test_linear_ste_clip_and_scale_edge_cases(bf16):
    say(f"linear STE clip mask / beta=0 / alpha=0, bf16={bf16}")
    c = wl.linear_case(600, 130, 160, 96, hp_rank=16, bf16=bf16)
    check_linear(c, bf16, ste_tau=0.02)
    check_linear(c, bf16, alpha=1.5, beta=0.0)
    check_linear(c, bf16, alpha=0.0, beta=0.7)


def test_linear_with_a_feature_scale_far_below_the_other():
    """alpha twelve orders of magnitude below beta: the fused forward (which carries beta / alpha through the tile) steps
    aside for the two separately scaled branches of the Sec. 3.2 sum; everything stays finite and on the oracle."""
    say("linear alpha=1e-12, beta=0.2, bf16, fused-path shape")
    c = wl.linear_case(610, 300, 640, 384, hp_rank=128, bf16=True)
    got = check_linear(c, True, alpha=1e-12, beta=0.2)
    assert np.isfinite(got["Y"]).all() and np.isfinite(got["dX"]).all()


def test_linear_config2_reduced_tokens_bf16():
    say("linear config2 shape at T=1024 (2048x2048, r=128), bf16")
    check_linear(wl.config2(tokens=1024), True)


def test_linear_backward_is_deterministic():
    c = wl.linear_case(700, 300, 256, 256, hp_rank=16, bf16=True)
    a = run_linear(c, True, 2.0, 0.2)
    b = run_linear(c, True, 2.0, 0.2)
    for k in ("Y", "dX", "dW", "dA", "dB", "dab"):
        assert np.array_equal(a[k], b[k]), k


def test_linear_config2_full_size_sampled():
    """Full bench shape (T=8192, 2048x2048, r=128, bf16) in the launch configuration bench.py times.  Rows of Y
    and dX depend on their token alone: the oracle recomputes sampled tokens here.  dW, dA, dB, d alpha and d beta
    sum over every token: they are compared with what oracle.linear_bwd gave on the whole workload
    (tests/golden/full_size_config2.npz; dW and dB on sampled output channels, dA whole)."""
    say("linear config2 full size, sampled rows")
    c = wl.config2()
    got = run_linear(c, True, 2.0, 0.2)
    rng = np.random.default_rng(0)
    tok = np.sort(rng.choice(c["tokens"], 48, replace=False))
    f = po.linear_fwd(c["X"][tok], c["W"], 2.0, 0.2, A=c["A"], B=c["B"])
    g = po.linear_bwd(c["dY"][tok], c["X"][tok], c["W"], 2.0, 0.2, f, A=c["A"], B=c["B"])
    errs = {}
    errs.update(report("Y", got["Y"][tok], f["Y"]))
    errs.update(report("dX", got["dX"][tok], g["dX"]))
    ref = np.load(os.path.join(GOLDEN, "full_size_config2.npz"))
    ch = ref["ch"]
    errs.update(report("dW", got["dW"][ch], ref["dW"], per_channel=True))
    errs.update(report("dB", got["dB"][ch], ref["dB"]))
    errs.update(report("dA", got["dA"], ref["dA"], per_channel=True))
    errs.update(scalar_errs(got["dab"], float(ref["dalpha"]), float(ref["dbeta"]), float(ref["dalpha_scale"]),
                            float(ref["dbeta_scale"])))
    assert_errs(errs, TOL[True])


# ---------------------------------------------------------------------------- packed weights, inference, no tokens
@pytest.mark.parametrize("T,K,N,r,bf16", [(1, 256, 72, 8, True), (64, 544, 416, 24, True), (1024, 2048, 2048, 128, True),
                                         (64, 96, 72, 0, False), (300, 256, 264, 16, False)])
@pytest.mark.parametrize("with_ctx", [False, True])
def test_linear_fwd_on_packed_weights(T, K, N, r, bf16, with_ctx):
    """PQ_W_PACKED: the bits and mu/lambda come from pq_pack_sign, the forward runs with ctx = NULL (inference: codes,
    gamma and H live in the workspace) and with a ctx; d_out only needs to be a multiple of 8 here."""
    say(f"linear fwd packed T={T} K={K} N={N} r={r} bf16={bf16} ctx={with_ctx}")
    c = wl.linear_case(900 + T + r, T, K, N, hp_rank=r, bf16=bf16, outlier_frac=0.02, outlier_scale=10.0)
    P, _, ml = pq.pack_sign(dev(c["W"], bf16))
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_BF16 if bf16 else pq.PQ_F32, w_kind=pq.PQ_W_PACKED)
    bufs = pq.LinearBuffers(desc)
    Y = torch.empty((T, N), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
    pq.linear_fwd(desc, dev(c["X"], bf16), P, Y, bufs, A=dev(c["A"], bf16) if r else None, B=dev(c["B"], bf16) if r else None,
                  mu_lambda=ml, save=with_ctx)
    torch.cuda.synchronize()
    mu, lam = po.weight_stats(c["W"])
    f = po.linear_fwd(c["X"], None, 2.0, 0.2, A=c["A"] if r else None, B=c["B"] if r else None,
                      packed=po.pack_sign(po.binarise(c["W"], mu)), mu_lambda=(mu, lam))
    assert_errs(report("Y", host(Y), f["Y"]), TOL[bf16])


@pytest.mark.parametrize("bf16", [True, False])
def test_linear_with_no_tokens(bf16):
    """T = 0: the forward still prepares the weight side, the backward writes zero weight gradients (an empty sum)
    and zero scalar gradients."""
    say(f"linear T=0 bf16={bf16}")
    c = wl.linear_case(950, 0, 96, 64, hp_rank=8, bf16=bf16)
    got = run_linear(c, bf16, 2.0, 0.2)
    for k in ("dW", "dA", "dB", "dab"):
        assert np.all(got[k] == 0.0) and np.isfinite(got[k]).all(), k
    if bf16:                                          # routed experts: empty expert segments
        c = wl.linear_case(951, 0, 96, 64, hp_rank=8, n_experts=4, bf16=True)
        got = run_linear(c, True, 2.0, 0.2, top_k=2)
        for k in ("dW", "dA", "dB", "dWr", "dab"):
            assert np.all(got[k] == 0.0) and np.isfinite(got[k]).all(), k


# ---------------------------------------------------------------------------- routed low-rank experts (Sec. 3.3)
@pytest.mark.parametrize("T,K,N,r,E,k", [(200, 96, 160, 8, 4, 1), (200, 96, 160, 8, 4, 2), (700, 256, 544, 32, 8, 1),
                                         (130, 64, 64, 16, 2, 2), (1, 32, 32, 8, 8, 1), (1500, 1024, 288, 32, 8, 2),
                                         (1100, 128, 96, 8, 40, 3), (3000, 64, 64, 8, 16, 1),   # many experts; slot ranges of several batches per wavefront
                                         (128, 4096, 11008, 64, 8, 2)])   # the decode layer's shape (config 4) in training
def test_linear_routed_experts(T, K, N, r, E, k):
    """E > 1 inside pq_linear_fwd / pq_linear_bwd: router, stable permutation, grouped expert GEMMs, gate-weighted
    combine, and the backward through experts, gates and router (dA, dB, dWr, dX, d alpha)."""
    say(f"linear routed T={T} K={K} N={N} r={r} E={E} k={k}")
    c = wl.linear_case(1200 + T + k, T, K, N, hp_rank=r, n_experts=E, bf16=True, outlier_frac=0.02, outlier_scale=10.0)
    check_linear(c, True, top_k=k)


def test_linear_routed_experts_with_router_ties_and_unused_experts():
    """Two identical router rows (ties go to the lower index, so the higher one is never first) and more experts than
    tokens (empty expert segments)."""
    c = wl.linear_case(1300, 5, 64, 96, hp_rank=8, n_experts=16, bf16=True)
    c["Wr"][3] = c["Wr"][2]
    check_linear(c, True, top_k=2)


def test_linear_routed_experts_reject_fp32():
    with pytest.raises(pq.PQError):
        pq.LinearBuffers(pq.make_desc(16, 64, 64, hp_rank=8, n_experts=4, io_dtype=pq.PQ_F32))


# ---------------------------------------------------------------------------- INT8 form of the dense branch via hp_kind
@pytest.mark.parametrize("T,K,N,r", [(64, 256, 256, 32), (300, 1024, 768, 64), (1100, 512, 384, 128), (0, 64, 64, 32)])
def test_linear_with_int8_high_precision_branch(T, K, N, r):
    """hp_kind = PQ_HP_LOWRANK_INT8 through pq_linear_fwd / pq_linear_bwd (Sec. 3.2): the branch consumes the codes of
    the 1-bit branch; expected values are oracle.linear_fwd without a branch plus oracle.hp_int8_fwd / hp_int8_bwd."""
    say(f"linear hp_kind=INT8 T={T} K={K} N={N} r={r}")
    c = wl.linear_case(1400 + T + r, T, K, N, hp_rank=r, bf16=True, outlier_frac=0.02, outlier_scale=10.0)
    alpha, beta = 1.5, 0.3
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_BF16, alpha=alpha, beta=beta, hp_kind=pq.PQ_HP_LOWRANK_INT8)
    bufs = pq.LinearBuffers(desc)
    X, W, dY, A, B = (dev(c[n], True) for n in ("X", "W", "dY", "A", "B"))
    Y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    pq.linear_fwd(desc, X, W, Y, bufs, A=A, B=B)
    dX = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
    dab = torch.empty((2,), dtype=torch.float32, device="cuda")
    pq.linear_bwd(desc, dY, X, W, bufs, dX, dW, dab, A=A, B=B, dA=dA, dB=dB)
    torch.cuda.synchronize()
    if T == 0:
        assert not host(dW).any() and not host(dA).any() and not host(dB).any() and not host(dab).any()
        return
    f = po.linear_fwd(c["X"], c["W"], 0.0, beta)
    h = po.hp_int8_fwd(None, c["A"], c["B"], bf16=True, q_gamma=(f["q"], f["gamma"]))
    g = po.linear_bwd(c["dY"], c["X"], c["W"], 0.0, beta, f)
    dY64 = c["dY"].astype(np.float64)
    gh = po.hp_int8_bwd(alpha * dY64, h)
    errs = {}
    errs.update(report("Y", host(Y), f["Y1"].astype(np.float64) + alpha * h["Yhp"].astype(np.float64)))
    errs.update(report("dX", host(dX), g["dX"] + gh["dX"]))
    errs.update(report("dW", host(dW), g["dW"], per_channel=True))
    errs.update(report("dA", host(dA), gh["dA"], per_channel=True))
    errs.update(report("dB", host(dB), gh["dB"]))
    Yhp = h["Yhp"].astype(np.float64)
    errs.update(scalar_errs(host(dab), float((dY64 * Yhp).sum()), g["dbeta"], np.sqrt(((dY64 * Yhp) ** 2).sum()),
                            np.sqrt(((dY64 * f["Y1_nobeta"]) ** 2).sum())))
    assert_errs(errs, TOL[True])
