"""Parity of the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Bars: bit-exact for sign bits, packed words, INT8 codes, gamma, int32 accumulators and routing
indices; max|a-b| / max|b| <= 1e-5 for fp32 I/O and <= 2e-2 for bf16 I/O on outputs and gradients.
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
                                        (5504, 2048, True, True), (11008, 4096, True, False)])   # configs 3 and 4
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
def run_linear(c, bf16, alpha, beta, ste_tau=None):
    T, K, N, r = c["tokens"], c["d_in"], c["d_out"], c["hp_rank"]
    desc = pq.make_desc(T, K, N, hp_rank=r, io_dtype=pq.PQ_BF16 if bf16 else pq.PQ_F32, alpha=alpha, beta=beta,
                        ste_mode=pq.PQ_STE_CLIP if ste_tau is not None else pq.PQ_STE_IDENTITY,
                        ste_tau=ste_tau or 0.0)
    bufs = pq.LinearBuffers(desc)
    dt = torch.bfloat16 if bf16 else torch.float32
    X, W, dY = dev(c["X"], bf16), dev(c["W"], bf16), dev(c["dY"], bf16)
    A = dev(c["A"], bf16) if r else None
    B = dev(c["B"], bf16) if r else None
    Y = torch.empty((T, N), dtype=dt, device="cuda")
    pq.linear_fwd(desc, X, W, Y, bufs, A=A, B=B)
    dX = torch.empty((T, K), dtype=dt, device="cuda")
    dW = torch.empty((N, K), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda") if r else None
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda") if r else None
    dab = torch.empty((2,), dtype=torch.float32, device="cuda")
    pq.linear_bwd(desc, dY, X, W, bufs, dX, dW, dab, A=A, B=B, dA=dA, dB=dB)
    torch.cuda.synchronize()
    return dict(Y=host(Y), dX=host(dX), dW=host(dW), dA=host(dA) if r else None, dB=host(dB) if r else None,
                dab=host(dab))


def check_linear(c, bf16, alpha=2.0, beta=0.2, ste_tau=None):
    r = c["hp_rank"]
    got = run_linear(c, bf16, alpha, beta, ste_tau)
    A, B = (c["A"], c["B"]) if r else (None, None)
    f = po.linear_fwd(c["X"], c["W"], alpha, beta, A=A, B=B)
    g = po.linear_bwd(c["dY"], c["X"], c["W"], alpha, beta, f, A=A, B=B,
                      ste_tau=np.inf if ste_tau is None else np.float32(ste_tau))
    tol = TOL[bf16]
    errs = dict(Y=relerr(got["Y"], f["Y"]), dX=relerr(got["dX"], g["dX"]), dW=relerr(got["dW"], g["dW"]))
    if r:
        errs.update(dA=relerr(got["dA"], g["dA"]), dB=relerr(got["dB"], g["dB"]))
    # scalar gradients: error relative to the natural scale of the sum (its root-sum-square of terms)
    dY = c["dY"].astype(np.float64)
    sb = max(abs(g["dbeta"]), np.sqrt(((dY * f["Y1_nobeta"]) ** 2).sum()))
    sa = max(abs(g["dalpha"]), np.sqrt(((dY * f["Yhp"]) ** 2).sum()), 1e-30)
    errs["dbeta"] = abs(got["dab"][1] - g["dbeta"]) / sb
    errs["dalpha"] = abs(got["dab"][0] - g["dalpha"]) / sa
    say("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert v <= tol, f"{k}: {v} > {tol}"
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
    """Full bench shape (T=8192, 2048x2048, r=128, bf16) in the launch configuration bench.py times;
    the oracle recomputes sampled tokens (rows of Y, dX) and sampled output channels (rows of dW, dB)."""
    say("linear config2 full size, sampled rows")
    c = wl.config2()
    got = run_linear(c, True, 2.0, 0.2)
    rng = np.random.default_rng(0)
    tok = np.sort(rng.choice(c["tokens"], 48, replace=False))
    f = po.linear_fwd(c["X"][tok], c["W"], 2.0, 0.2, A=c["A"], B=c["B"])
    g = po.linear_bwd(c["dY"][tok], c["X"][tok], c["W"], 2.0, 0.2, f, A=c["A"], B=c["B"])
    eY, eX = relerr(got["Y"][tok], f["Y"]), relerr(got["dX"][tok], g["dX"])
    # weight-side gradients need every token: recompute sampled output channels from the definitions
    q, gamma = po.quant_act(c["X"])
    ch = np.sort(rng.choice(c["d_out"], 32, replace=False))
    dY64 = c["dY"].astype(np.float64)
    dW_rows = 0.2 * ((dY64[:, ch] / gamma.astype(np.float64)[:, None]).T @ q.astype(np.float64))
    H = c["X"].astype(np.float64) @ c["A"].astype(np.float64).T
    dB_rows = 2.0 * (dY64[:, ch].T @ H)
    eW, eB = relerr(got["dW"][ch], dW_rows), relerr(got["dB"][ch], dB_rows)
    say(f"  errors: Y={eY:.2e} dX={eX:.2e} dW={eW:.2e} dB={eB:.2e}")
    assert max(eY, eX, eW, eB) <= TOL[True]
