"""Parity of the INT8 form of the high-precision branch (Sec. 3.2) against the CPU oracle.

Bars: the codes and gammas of A, B and of the hidden state, the stored hidden state and (with alpha = 1, no
accumulation) the bf16 output bit-exact: both integer products are exact and the two scales come off in the
same fp32 order on both sides.  With alpha != 1 or accumulation, and for the STE backward (bf16 GEMMs on the
de-quantised factors), max|a-b| / max|b| <= 2e-2.
"""
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 2e-2


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


def _case(seed, T, K, N, r):
    rng = np.random.default_rng(seed)
    X = wl.activations(rng, T, K, outlier_frac=0.01, outlier_scale=20.0, bf16=True)
    A = wl.normal(rng, (r, K), 0.02, True)
    B = wl.normal(rng, (N, r), 0.02, True)
    dY = wl.normal(rng, (T, N), 1.0, True)
    return X, A, B, dY


def _run_fwd(X, A, B, alpha, Y0=None):
    T, K = X.shape
    N, r = B.shape
    Xq, gx = pq.quant_act(dev(X, True))
    bufs = pq.HpInt8Buffers(T, K, N, r)
    Y = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda") if Y0 is None else dev(Y0, True)
    pq.hp_int8_fwd(Xq, gx, dev(A, True), dev(B, True), alpha, Y, bufs, accumulate=Y0 is not None)
    torch.cuda.synchronize()
    return Xq, gx, Y, bufs


SHAPES = [(64, 256, 256, 32), (300, 2048, 1024, 64), (37, 512, 5504, 96), (513, 4096, 4096, 128), (1, 64, 32, 32),
          (0, 64, 64, 32), (260, 1024, 288, 160),
          (1100, 512, 384, 128), (2048, 2048, 256, 128)]   # rank 128, 1024 tokens or more: the streaming rank-r kernel computes H


@pytest.mark.parametrize("T,K,N,r", SHAPES)
def test_hp_int8_fwd_bit_exact(T, K, N, r):
    say(f"hp_int8_fwd T={T} K={K} N={N} r={r}")
    X, A, B, _ = _case(900 + T + r, T, K, N, r)
    if T > 2:
        X[1] = 0.0
    A[0] = 0.0                                        # a zero weight row: gamma from the 1e-5 floor, codes zero
    Xq, gx, Y, bufs = _run_fwd(X, A, B, 1.0)
    ref = po.hp_int8_fwd(X, A, B, bf16=True)
    q_a, g_a, q_b, g_b, H, q_h, g_h = bufs.views()
    assert np.array_equal(host(q_a), ref["q_a"]) and np.array_equal(host(g_a), ref["g_a"])
    assert np.array_equal(host(q_b), ref["q_b"]) and np.array_equal(host(g_b), ref["g_b"])
    if T == 0:
        return
    assert np.array_equal(host(Xq), ref["q_x"]) and np.array_equal(host(gx), ref["g_x"])
    assert np.array_equal(host(H), ref["H"])
    assert np.array_equal(host(q_h), ref["q_h"]) and np.array_equal(host(g_h), ref["g_h"])
    assert np.array_equal(host(Y), po._round_io(ref["Yhp"], True))


def test_hp_int8_fwd_alpha_accumulate():
    T, K, N, r = 200, 1024, 768, 64
    say(f"hp_int8_fwd alpha/accumulate T={T} K={K} N={N} r={r}")
    X, A, B, Y0 = _case(77, T, K, N, r)
    Y0 = (Y0 * np.float32(0.01)).astype(np.float32)
    Y0 = host(dev(Y0, True))
    alpha = 0.37
    ref = po.hp_int8_fwd(X, A, B, bf16=True)
    _, _, Y, _ = _run_fwd(X, A, B, alpha)
    assert relerr(host(Y), alpha * ref["Yhp"]) <= TOL
    _, _, Y, _ = _run_fwd(X, A, B, alpha, Y0=Y0)
    assert relerr(host(Y), Y0 + alpha * ref["Yhp"]) <= TOL


@pytest.mark.parametrize("T,K,N,r", [(64, 256, 256, 32), (300, 2048, 1024, 64), (37, 512, 5504, 96),
                                     (513, 4096, 4096, 128), (0, 64, 64, 32), (1100, 512, 384, 128),
                                     (2048, 192, 320, 128)])   # dB and dA in the streaming pair kernel
def test_hp_int8_bwd_parity(T, K, N, r):
    say(f"hp_int8_bwd T={T} K={K} N={N} r={r}")
    X, A, B, dY = _case(1900 + T + r, T, K, N, r)
    alpha = 0.5
    Xd = dev(X, True)
    Xq = torch.empty((T, K), dtype=torch.int8, device="cuda")
    gx = torch.empty((T,), dtype=torch.float32, device="cuda")
    Xt = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    if T > 0:
        # the quantiser of the fused norm kernel's family writes q / gamma in bf16 next to the codes
        g1 = torch.ones((K,), dtype=torch.bfloat16, device="cuda")
        _, Xq, gx, Xt, _ = pq.rmsnorm_quant_fwd(Xd, g1, 1e-6, want_xn=True, want_xt=True)
    bufs = pq.HpInt8Buffers(T, K, N, r)
    Y = torch.zeros((T, N), dtype=torch.bfloat16, device="cuda")
    pq.hp_int8_fwd(Xq, gx, dev(A, True), dev(B, True), alpha, Y, bufs)
    dX = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
    pq.hp_int8_bwd(dev(dY, True), Xt, alpha, bufs, dX, dA, dB)
    torch.cuda.synchronize()
    if T == 0:
        assert not host(dA).any() and not host(dB).any()
        return
    q_gamma = (host(Xq), host(gx))
    ref = po.hp_int8_fwd(None, A, B, bf16=True, q_gamma=q_gamma)
    g = po.hp_int8_bwd(alpha * dY.astype(np.float64), ref)
    assert relerr(host(dX), g["dX"]) <= TOL
    assert relerr(host(dA), g["dA"]) <= TOL
    assert relerr(host(dB), g["dB"]) <= TOL
    # accumulation into an existing dX
    dX0 = host(dX).copy()
    pq.hp_int8_bwd(dev(dY, True), Xt, alpha, bufs, dX, dA, dB, accumulate_dX=True)
    torch.cuda.synchronize()
    assert relerr(host(dX), 2.0 * dX0) <= TOL


def test_hp_int8_full_size_sampled():
    """Config-2 shape (8192 tokens, 4096 -> 4096, r = 128): sampled token rows against the oracle (every row of
    the forward depends on its own token only)."""
    T, K, N, r = 8192, 4096, 4096, 128
    say(f"hp_int8 full size T={T} K={K} N={N} r={r}")
    X, A, B, _ = _case(4242, T, K, N, r)
    Xq, gx, Y, bufs = _run_fwd(X, A, B, 1.0)
    rows = np.array([0, 1, 255, 256, 4095, 4097, 8190, 8191])
    ref = po.hp_int8_fwd(X[rows], A, B, bf16=True)
    q_a, g_a, q_b, g_b, H, q_h, g_h = bufs.views()
    assert np.array_equal(host(q_a), ref["q_a"]) and np.array_equal(host(q_b), ref["q_b"])
    assert np.array_equal(host(H)[rows], ref["H"])
    assert np.array_equal(host(q_h)[rows], ref["q_h"])
    assert np.array_equal(host(Y)[rows], po._round_io(ref["Yhp"], True))


def test_hp_int8_rejects_bad_arguments():
    bufs = pq.HpInt8Buffers(8, 64, 64, 32)
    Xq = torch.zeros((8, 64), dtype=torch.int8, device="cuda")
    gx = torch.ones(8, device="cuda")
    with pytest.raises(pq.PQError):                   # fp32 factors: the branch is bf16 only
        pq.hp_int8_fwd(Xq, gx, torch.zeros((32, 64), device="cuda"), torch.zeros((64, 32), device="cuda"), 1.0,
                       torch.zeros((8, 64), device="cuda"), bufs)
    small = pq.HpInt8Buffers(8, 64, 64, 32)
    small.shape = (64, 64, 64, 32)                    # ctx sized for 8 tokens, call made for 64
    with pytest.raises(pq.PQError):
        pq.hp_int8_fwd(torch.zeros((64, 64), dtype=torch.int8, device="cuda"), torch.ones(64, device="cuda"),
                       torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda"),
                       torch.zeros((64, 32), dtype=torch.bfloat16, device="cuda"), 1.0,
                       torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda"), small)
    assert pq.lib().pq_hp_int8_ctx_bytes(8, 60, 64, 32) == 0
    assert pq.lib().pq_hp_int8_ctx_bytes(8, 64, 64, 24) == 0
