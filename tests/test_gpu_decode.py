"""Parity of the packed-1-bit decode product (App. A) against the CPU oracle: int32 accumulators
bit-exact, bf16 outputs within 2e-2 (max-norm relative)."""
import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(x, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def relerr(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def run_decode(c, top_k, alpha, beta, tiled=False):
    L, B, K, N, E, r = c["n_layers"], c["batch"], c["d_in"], c["d_out"], c["n_experts"], c["hp_rank"]
    Ps, scales, mls = [], [], []
    for l in range(L):                                   # offline: binarise + pack + fold beta*lambda to fp16
        P, _, ml = pq.pack_sign(dev(c["W"][l], True))
        Ps.append(P); mls.append(ml.cpu().numpy())
        scales.append(np.float16(np.float32(beta) * mls[-1][1]))
    P = torch.stack(Ps).contiguous()
    Pin = torch.stack([pq.pack_retile64(p_, K) for p_ in Ps]).contiguous() if tiled else P
    scale = dev(np.array(scales, np.float16).view(np.int16))
    desc = pq.DecodeDesc(B, K, N, r, E if r else 1, top_k if r else 1, L,
                         pq.PQ_PACKED_TILED64 if tiled else pq.PQ_PACKED_ROWMAJOR, alpha)
    ws = pq.decode_workspace(desc)
    X = dev(c["X"], True)
    A = dev(c["A"], True) if r else None
    Bm = dev(c["B"], True) if r else None
    Wr = dev(c["Wr"], True) if r else None
    Y = torch.empty((L, B, N), dtype=torch.bfloat16, device="cuda")
    acc = torch.empty((L, B, N), dtype=torch.int32, device="cuda")
    pq.decode_gemv(desc, X, Pin, scale, Y, ws, A=A, B=Bm, Wr=Wr, acc_out=acc)
    torch.cuda.synchronize()
    return Y.float().cpu().numpy(), acc.cpu().numpy(), P.cpu().numpy().view(np.uint32), mls


def check_decode(c, top_k=2, alpha=2.0, beta=0.2, tiled=False):
    Y, acc, P, mls = run_decode(c, top_k, alpha, beta, tiled)
    r = c["hp_rank"]
    worst = 0.0
    for l in range(c["n_layers"]):
        mu, lam = po.weight_stats(c["W"][l])
        assert mls[l][0] == mu and mls[l][1] == lam
        Pref = po.pack_sign(po.binarise(c["W"][l], mu))
        assert np.array_equal(P[l], Pref)
        f = po.decode_gemv(c["X"][l], Pref, (mu, lam), alpha, beta, A=c["A"][l] if r else None,
                           B=c["B"][l] if r else None, Wr=c["Wr"][l] if r else None, top_k=top_k)
        assert np.array_equal(acc[l].astype(np.int64), f["acc"]), f"layer {l}: int32 accumulators differ"
        worst = max(worst, relerr(Y[l], f["Y"]))
    print(f"  decode max-norm relative error {worst:.2e}", flush=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("L,B,K,N,E,r,k", [(1, 1, 256, 136, 4, 16, 2), (2, 1, 4096, 1000, 8, 64, 2), (1, 1, 128, 64, 1, 0, 1),
                                           (3, 1, 640, 328, 8, 8, 1), (1, 1, 8192, 260, 4, 24, 3)])
@pytest.mark.parametrize("tiled", [False, True])
def test_decode_gemv_batch1(L, B, K, N, E, r, k, tiled):
    print(f"decode B=1: L={L} K={K} N={N} E={E} r={r} k={k} tiled={tiled}", flush=True)
    check_decode(wl.decode_case(40 + K + N, B, d_in=K, d_out=N, n_experts=E, hp_rank=r, n_layers=L), top_k=k,
                 tiled=tiled)


@pytest.mark.parametrize("L,B,K,N,E,r,k", [(1, 3, 512, 200, 4, 32, 2), (2, 8, 1024, 1028, 8, 64, 2), (1, 16, 512, 64, 2, 32, 1),
                                           # widths 2048 and 512 of the expert-by-expert hidden-state kernel; 128 slots per layer (per-slot kernel)
                                           (2, 5, 2048, 264, 8, 64, 2), (1, 16, 512, 64, 8, 32, 8),
                                           (1, 2, 4096, 300, 1, 0, 1), (1, 5, 1536, 520, 8, 32, 3)])
@pytest.mark.parametrize("tiled", [False, True])
def test_decode_small_batch(L, B, K, N, E, r, k, tiled):
    print(f"decode B={B}: L={L} K={K} N={N} E={E} r={r} k={k} tiled={tiled}", flush=True)
    check_decode(wl.decode_case(50 + K + N + B, B, d_in=K, d_out=N, n_experts=E, hp_rank=r, n_layers=L), top_k=k,
                 tiled=tiled)


@pytest.mark.parametrize("L,B,K,N,E,r,k", [(1, 4, 640, 132, 4, 32, 2), (2, 9, 1408, 260, 2, 64, 1),
                                           # the codes pass through LDS in blocks of 32 KB: three blocks, the last one ragged
                                           (1, 16, 4352, 132, 4, 32, 2), (1, 7, 8960, 200, 2, 32, 1)])
def test_decode_small_batch_tiled_ragged_k(L, B, K, N, E, r, k):
    """Row-interleaved packing takes any d_in that is a multiple of 128 (here not of 512) and a ragged last group."""
    print(f"decode tiled B={B}: L={L} K={K} N={N} E={E} r={r} k={k}", flush=True)
    check_decode(wl.decode_case(70 + K + N + B, B, d_in=K, d_out=N, n_experts=E, hp_rank=r, n_layers=L), top_k=k,
                 tiled=True)


@pytest.mark.parametrize("B,tiled", [(1, True), (8, True), (8, False)])
def test_decode_config4_full_size(B, tiled):
    """4096 -> 11008, E=8 top-2 experts of rank 64 (the bench shape), two layers."""
    print(f"decode config 4, B={B} tiled={tiled}", flush=True)
    check_decode(wl.decode_case(4, B, n_layers=2), top_k=2, tiled=tiled)


def test_decode_alpha_zero_and_beta_edge():
    c = wl.decode_case(60, 1, d_in=512, d_out=256, n_experts=4, hp_rank=16, n_layers=1)
    check_decode(c, alpha=0.0, beta=0.7)
    check_decode(c, alpha=1.5, beta=0.0)


# ------------------------------------------------------------------------------------------------
# Experts in their INT8 form (Sec. 3.2): accumulators and the bf16 hidden state bit-exact, outputs within 2e-2
# ------------------------------------------------------------------------------------------------
def check_decode_int8(c, top_k=2, alpha=2.0, beta=0.2, tiled=False):
    L, B, K, N, E, r = c["n_layers"], c["batch"], c["d_in"], c["d_out"], c["n_experts"], c["hp_rank"]
    Ps, scales, mls = [], [], []
    for l in range(L):
        P, _, ml = pq.pack_sign(dev(c["W"][l], True))
        Ps.append(P); mls.append(ml.cpu().numpy())
        scales.append(np.float16(np.float32(beta) * mls[-1][1]))
    Pin = torch.stack([pq.pack_retile64(p_, K) for p_ in Ps]).contiguous() if tiled else torch.stack(Ps).contiguous()
    scale = dev(np.array(scales, np.float16).view(np.int16))
    desc = pq.DecodeDesc(B, K, N, r, E, top_k, L, pq.PQ_PACKED_TILED64 if tiled else pq.PQ_PACKED_ROWMAJOR, alpha)
    ws = pq.decode_workspace(desc)
    Aq, gA = pq.quant_rows(dev(c["A"], True))            # offline: weight rows through the activation quantiser
    Bq, gB = pq.quant_rows(dev(c["B"], True))
    Y = torch.empty((L, B, N), dtype=torch.bfloat16, device="cuda")
    acc = torch.empty((L, B, N), dtype=torch.int32, device="cuda")
    pq.decode_gemv_int8(desc, dev(c["X"], True), Pin, scale, Y, ws, Aq, gA, Bq, gB, dev(c["Wr"], True), acc_out=acc)
    torch.cuda.synchronize()
    H = pq.decode_ws_hidden(desc, ws).cpu().numpy()
    Y = Y.float().cpu().numpy(); acc = acc.cpu().numpy()
    worst = 0.0
    for l in range(L):
        mu, lam = po.weight_stats(c["W"][l])
        Pref = po.pack_sign(po.binarise(c["W"][l], mu))
        f = po.decode_gemv_int8(c["X"][l], Pref, (mu, lam), alpha, beta, c["A"][l], c["B"][l], c["Wr"][l], top_k=top_k)
        qa, ga = po.quant_act(c["A"][l].reshape(E * r, K))
        assert np.array_equal(Aq[l].cpu().numpy().reshape(E * r, K), qa) and np.array_equal(gA[l].cpu().numpy().reshape(-1), ga)
        assert np.array_equal(acc[l].astype(np.int64), f["acc"]), f"layer {l}: int32 accumulators differ"
        assert np.array_equal(H[l], f["Hs"]), f"layer {l}: expert hidden states differ"
        worst = max(worst, relerr(Y[l], f["Y"]))
    print(f"  INT8-expert decode max-norm relative error {worst:.2e}", flush=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("L,K,N,E,r,k", [(1, 256, 136, 4, 32, 2), (2, 4096, 1000, 8, 64, 2), (3, 640, 328, 8, 32, 1),
                                         (1, 8192, 260, 4, 96, 3), (1, 128, 64, 1, 32, 1)])
@pytest.mark.parametrize("tiled", [False, True])
def test_decode_int8_experts_batch1(L, K, N, E, r, k, tiled):
    print(f"decode INT8 experts: L={L} K={K} N={N} E={E} r={r} k={k} tiled={tiled}", flush=True)
    check_decode_int8(wl.decode_case(80 + K + N, 1, d_in=K, d_out=N, n_experts=E, hp_rank=r, n_layers=L), top_k=k,
                      tiled=tiled)


def test_decode_int8_experts_config4_full_size():
    print("decode INT8 experts, config 4 shape, two layers", flush=True)
    check_decode_int8(wl.decode_case(4, 1, n_layers=2), top_k=2, tiled=True)


def test_decode_int8_experts_alone_and_limits():
    """beta = 0 leaves only the expert term, so the whole output tests the INT8 branch; unsupported shapes are errors."""
    c = wl.decode_case(61, 1, d_in=512, d_out=256, n_experts=4, hp_rank=32, n_layers=1)
    check_decode_int8(c, alpha=1.5, beta=0.0)
    z8 = torch.zeros(16, dtype=torch.int8, device="cuda")
    zf = torch.zeros(16, dtype=torch.float32, device="cuda")
    for desc in (pq.DecodeDesc(2, 512, 256, 32, 4, 2, 1, pq.PQ_PACKED_TILED64, 1.0),       # batch 2 with r % 64 != 0
                 pq.DecodeDesc(2, 512, 256, 64, 4, 2, 1, pq.PQ_PACKED_ROWMAJOR, 1.0)):     # batch 2 on the row-major packing
        ws = pq.decode_workspace(desc)
        with pytest.raises(pq.PQError):
            pq.decode_gemv_int8(desc, z8, z8, z8, z8, ws, z8, zf, z8, zf, z8)


@pytest.mark.parametrize("L,B,K,N,E,r,k", [(1, 3, 512, 200, 4, 64, 2), (2, 8, 1024, 1028, 8, 64, 2), (1, 16, 512, 64, 2, 64, 1),
                                           (1, 5, 1536, 520, 8, 128, 3), (1, 9, 640, 132, 4, 64, 2)])
def test_decode_int8_experts_small_batch(L, B, K, N, E, r, k):
    print(f"decode INT8 experts B={B}: L={L} K={K} N={N} E={E} r={r} k={k}", flush=True)
    check_decode_int8(wl.decode_case(90 + K + N + B, B, d_in=K, d_out=N, n_experts=E, hp_rank=r, n_layers=L), top_k=k,
                      tiled=True)


def test_decode_int8_experts_config4_batch8():
    print("decode INT8 experts, config 4 shape, batch 8, two layers", flush=True)
    check_decode_int8(wl.decode_case(4, 8, n_layers=2), top_k=2, tiled=True)


def test_decode_largest_d_in():
    """d_in = 16384 (bf16 experts) and 13056 (INT8 experts): a token's staging area in LDS exceeds 64 KB."""
    print("decode d_in = 16384", flush=True)
    check_decode(wl.decode_case(95, 1, d_in=16384, d_out=72, n_experts=2, hp_rank=16, n_layers=1), top_k=1, tiled=True)
    print("decode INT8 experts d_in = 13056", flush=True)
    check_decode_int8(wl.decode_case(96, 1, d_in=13056, d_out=72, n_experts=2, hp_rank=32, n_layers=1), top_k=1, tiled=True)


def test_decode_largest_d_in_small_batch():
    """d_in = 16384 with 16 and with 8 tokens on the row-interleaved packing: 256 KB resp. 128 KB of codes walk through
    32 KB of LDS in eight resp. four blocks; the INT8 experts at batch 8 likewise."""
    for B in (16, 8):
        print(f"decode d_in = 16384, B = {B}", flush=True)
        check_decode(wl.decode_case(97 + B, B, d_in=16384, d_out=136, n_experts=2, hp_rank=32, n_layers=1), top_k=1, tiled=True)
    print("decode INT8 experts d_in = 12800, B = 8", flush=True)
    check_decode_int8(wl.decode_case(99, 8, d_in=12800, d_out=136, n_experts=2, hp_rank=64, n_layers=1), top_k=1, tiled=True)
