"""Pins of the CPU oracle against things other than itself: hand-worked cases, brute force with
Python integers, exactly-rounded sums, library routines, the lookup-table route of App. A, closed
forms, error bounds and finite differences.  None of these need a GPU."""
import math
import os

import numpy as np
import pytest

from oracle import pquant_oracle as po
from paper_2602_22592_amd import workloads as wl

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")) as fh:
    for line in fh:
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            GOLD[k.strip()] = float(v)


# ---------------------------------------------------------------- weight statistics / binariser
def test_weight_stats_hand_case():
    W = np.array([[1.0, -3.0], [2.0, 4.0]], np.float32)
    mu, lam = po.weight_stats(W)
    assert mu == np.float32(1.0) and lam == np.float32(2.5)          # lambda on raw |W|, not |W - mu|


@pytest.mark.parametrize("seed,shape,bf16", [(0, (37, 64), False), (1, (256, 256), True), (2, (2048, 2048), True)])
def test_weight_stats_vs_exactly_rounded_sum(seed, shape, bf16):
    W = wl.normal(np.random.default_rng(seed), shape, 0.02, bf16)
    mu, lam = po.weight_stats(W)
    flat = [float(v) for v in W.ravel()]
    assert mu == np.float32(math.fsum(flat) / W.size)
    assert lam == np.float32(math.fsum(abs(v) for v in flat) / W.size)


def test_binarise_hand_cases():
    W = np.array([[1.0, -3.0], [2.0, 4.0]], np.float32)             # mu = 1 is an element: -> +1
    assert po.binarise(W, np.float32(1.0)).tolist() == [[1, -1], [1, 1]]
    C = np.full((3, 32), 0.125, np.float32)                          # all equal: W == mu everywhere
    mu, lam = po.weight_stats(C)
    assert mu == np.float32(0.125) and lam == np.float32(0.125)
    assert np.all(po.binarise(C, mu) == 1)


def test_binarise_is_sign_of_centred_weight():
    W = wl.normal(np.random.default_rng(3), (64, 96), 0.02)
    mu, _ = po.weight_stats(W)
    S = po.binarise(W, mu)
    d = W.astype(np.float64) - float(mu)
    assert np.all(S[d > 0] == 1) and np.all(S[d < 0] == -1)
    assert set(np.unique(S)) <= {-1, 1}
    # centring balances the code: about half the weights land on each side
    assert abs(S.astype(np.int64).sum()) < 0.1 * S.size


def test_pack_bruteforce_roundtrip_popcount_and_bytes():
    rng = np.random.default_rng(4)
    S = np.where(rng.random((16, 64)) < 0.4, 1, -1).astype(np.int8)
    P = po.pack_sign(S)
    assert P.dtype == np.uint32 and P.shape == (16, 2)
    for i in range(16):                                               # brute force, Python ints
        for w in range(2):
            word = 0
            for j in range(32):
                if S[i, 32 * w + j] == 1:
                    word |= 1 << j
            assert int(P[i, w]) == word
    assert np.array_equal(po.unpack_sign(P, 64), S)
    assert sum(bin(int(v)).count("1") for v in P.ravel()) == int((S == 1).sum())
    # library route: little-endian bit packing of the same booleans gives the same byte stream
    assert np.array_equal(np.packbits(S > 0, axis=1, bitorder="little"), P.view(np.uint8).reshape(16, -1))
    # App. A: 8 parameters per byte = 1/16 of FP16 storage
    assert P.nbytes / (S.size * 2) == GOLD["packed_vs_fp16"]


def test_bits_per_weight_matches_paper_tables():
    assert round(po.bits_per_weight(GOLD["frac_1bit_300m"], GOLD["frac_8bit_300m"]), 2) == GOLD["bits_300m"]
    assert round(po.bits_per_weight(GOLD["frac_1bit_1p3b"], GOLD["frac_8bit_1p3b"]), 2) == GOLD["bits_1p3b"]


# ---------------------------------------------------------------- activation quantiser
def test_quant_hand_cases():
    X = np.array([[2.0, -2.0, 1.0, 0.5],            # gamma = 64: +absmax saturates 128 -> 127
                  [0.0, 0.0, 0.0, 0.0],             # zero row -> gamma = 128 / 1e-5, codes 0
                  [128.0, 0.5, 1.5, 2.5],           # gamma = 1: ties go to even
                  [-4.0, 1.0, 3.0, 0.03125]],       # gamma = 32: -absmax -> -128, no clamp needed
                 np.float32)
    q, g = po.quant_act(X)
    assert q.tolist() == [[127, -128, 64, 32], [0, 0, 0, 0], [127, 0, 2, 2], [-128, 32, 96, 1]]
    assert g[0] == 64 and g[2] == 1 and g[3] == 32
    assert g[1] == np.float32(128.0) / np.float32(1e-5)
    assert 2 ** GOLD["act_range_log2"] == 128


def test_quant_bruteforce_and_invariants():
    X = wl.activations(np.random.default_rng(5), 33, 96, outlier_count=3, outlier_scale=10.0)
    q, g = po.quant_act(X)
    for t in range(X.shape[0]):
        a = max(abs(float(v)) for v in X[t])
        gt = np.float32(128.0) / np.float32(a)
        assert g[t] == gt
        for k in range(X.shape[1]):
            y = float(np.float32(X[t, k]) * gt)                       # fp32 product, then Python round (half-even)
            assert int(q[t, k]) == max(-128, min(127, round(y)))
    amax = np.abs(q.astype(np.int32)).max(axis=1)
    assert np.all((amax == 127) | (amax == 128))
    err = np.abs(X.astype(np.float64) - q / g.astype(np.float64)[:, None]) * g.astype(np.float64)[:, None]
    is_pos_max = X == np.abs(X).max(axis=1, keepdims=True)
    assert np.all(err[~is_pos_max] <= 0.5 + 1e-4) and np.all(err <= 1.0 + 1e-4)


def test_quant_idempotent_on_integer_rows():
    rng = np.random.default_rng(6)
    Z = rng.integers(-127, 128, size=(8, 64)).astype(np.float32)
    Z[:, 0] = -128.0                                                  # absmax = 128 -> gamma = 1
    q, g = po.quant_act(Z)
    assert np.all(g == 1) and np.array_equal(q.astype(np.float32), Z)


# ---------------------------------------------------------------- integer GEMM
def _lut_dot(qrow, Prow):
    """App. A lookup-table route: per group of 4 activations a 16-entry table of signed sums,
    indexed by the 4 weight bits; the dot product is a sum of looked-up entries."""
    total = 0
    for gidx in range(len(qrow) // 4):
        xs = [int(v) for v in qrow[4 * gidx:4 * gidx + 4]]
        table = [sum(x if (pat >> j) & 1 else -x for j, x in enumerate(xs)) for pat in range(16)]
        k = 4 * gidx
        pat = (int(Prow[k // 32]) >> (k % 32)) & 0xF
        total += table[pat]
    return total


def test_onebit_acc_bruteforce_and_lut_route():
    rng = np.random.default_rng(7)
    q = rng.integers(-128, 128, size=(5, 64)).astype(np.int8)
    S = np.where(rng.random((7, 64)) < 0.5, 1, -1).astype(np.int8)
    acc = po.onebit_acc(q, S)
    P = po.pack_sign(S)
    assert GOLD["lut_entries"] == 2 ** GOLD["lut_group"] == 16
    for t in range(5):
        for i in range(7):
            assert int(acc[t, i]) == sum(int(q[t, k]) * int(S[i, k]) for k in range(64))
            assert int(acc[t, i]) == _lut_dot(q[t], P[i])


def test_pack_sign_pads_partial_words_with_plus_one():
    """Row lengths that are not multiples of 32 (Table 1: 5076 = 158 words + 20 bits): the last word is filled with
    +1 bits.  Pins: brute force with Python integers, np.packbits on the padded signs, the round trip, and the fact
    the padding exists for -- codes extended by zeros against the padded signs give the unpadded accumulator."""
    rng = np.random.default_rng(44)
    for m, n in ((3, 44), (5, 5076), (2, 20), (4, 96)):
        S = np.where(rng.random((m, n)) < 0.5, 1, -1).astype(np.int8)
        P = po.pack_sign(S)
        nw = (n + 31) // 32
        assert P.shape == (m, nw) and P.dtype == np.uint32
        for i in range(m):
            for w in range(nw):
                word = 0
                for j in range(32):
                    k = 32 * w + j
                    if k >= n or S[i, k] > 0:
                        word |= 1 << j
                assert int(P[i, w]) == word
        padded = np.concatenate([S > 0, np.ones((m, 32 * nw - n), bool)], axis=1)
        assert np.array_equal(P.view(np.uint8), np.packbits(padded, axis=1, bitorder="little"))
        assert np.array_equal(po.unpack_sign(P, n), S)
        q = rng.integers(-128, 128, size=(6, n)).astype(np.int8)
        qp = np.concatenate([q, np.zeros((6, 32 * nw - n), np.int8)], axis=1)
        assert np.array_equal(po.onebit_acc(qp, po.unpack_sign(P, 32 * nw)), po.onebit_acc(q, S))


def test_ffn_paper_width_is_not_a_multiple_of_32():
    """The oracle's FFN takes the paper's own 1-bit width (Table 1: D_ff - r = 5076 at D_model = 2048 for 1.3B; here the
    same residues at a small size): no step of it needs whole words, and the hidden state has exactly F columns."""
    c = wl.ffn_case(46, 9, 32, 52, 2, 8)              # 52 = 32 + 20, like 5076 = 158 * 32 + 20
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2)
    assert f["Hd"].shape == (9, 52) and f["qh"].shape == (9, 52)
    S = f["st"]["down"]["S"]
    assert np.array_equal(f["acc_d"], po.onebit_acc(f["qh"], po.unpack_sign(po.pack_sign(S), 52)))


def test_onebit_acc_fp32_blas_is_an_exact_second_route():
    rng = np.random.default_rng(8)
    q = rng.integers(-128, 128, size=(64, 5504)).astype(np.int8)
    S = np.where(rng.random((96, 5504)) < 0.5, 1, -1).astype(np.int8)
    acc = po.onebit_acc(q, S)
    blas = q.astype(np.float32) @ S.astype(np.float32).T             # all partial sums are integers < 2^24
    assert np.array_equal(acc, blas.astype(np.int64))
    assert np.abs(acc).max() < 2 ** 24


# ---------------------------------------------------------------- forward
def test_forward_reduces_to_textbook_onebit_linear():
    c = wl.linear_case(9, 12, 64, 40)
    f = po.linear_fwd(c["X"], c["W"], 0.0, 1.0)
    mu = c["W"].astype(np.float64).mean()
    lam = np.abs(c["W"].astype(np.float64)).mean()
    S = np.sign(c["W"].astype(np.float64) - mu)
    a = np.abs(c["X"]).max(axis=1).astype(np.float64)
    q = np.clip(np.rint(c["X"].astype(np.float64) * (128.0 / a)[:, None]), -128, 127)
    ref = (lam * a / 128.0)[:, None] * (q @ S.T)                      # Y = lambda/gamma * W1 * Q(X)
    assert np.allclose(f["Y"], ref, rtol=1e-5, atol=1e-7)


def test_forward_within_quantisation_error_of_float_binary_linear():
    c = wl.linear_case(10, 20, 128, 48)
    beta = 0.7
    f = po.linear_fwd(c["X"], c["W"], 0.0, beta)
    ideal = beta * float(f["lam"]) * (c["X"].astype(np.float64) @ f["S"].astype(np.float64).T)
    bound = beta * float(f["lam"]) * c["X"].shape[1] * (1.0 / f["gamma"].astype(np.float64))  # |x - q/gamma| <= 1/gamma
    assert np.all(np.abs(f["Y"] - ideal) <= bound[:, None] * 1.0001)
    # and much closer on average: rounding errors are centred
    assert np.abs(f["Y"] - ideal).mean() < 0.1 * bound.mean()


def test_forward_beta_zero_is_plain_lowrank_matmul():
    c = wl.linear_case(11, 9, 64, 40, hp_rank=8)
    f = po.linear_fwd(c["X"], c["W"], 1.5, 0.0, A=c["A"], B=c["B"])
    ref = 1.5 * (c["X"].astype(np.float64) @ c["A"].astype(np.float64).T) @ c["B"].astype(np.float64).T
    assert np.allclose(f["Y"], ref, rtol=1e-12, atol=1e-15)


def test_forward_sums_the_two_branches_with_feature_scales():
    c = wl.linear_case(12, 9, 64, 40, hp_rank=8)
    a, b = 2.0, 0.2
    assert a == GOLD["alpha_init"] and b == GOLD["beta_init"]
    f = po.linear_fwd(c["X"], c["W"], a, b, A=c["A"], B=c["B"])
    one = po.linear_fwd(c["X"], c["W"], 0.0, 1.0)["Y"]
    hp = po.linear_fwd(c["X"], c["W"], 1.0, 0.0, A=c["A"], B=c["B"])["Y"]
    assert np.allclose(f["Y"], b * one + a * hp, rtol=1e-6, atol=1e-7)         # fp32 rounding of the 1-bit scale


def test_packed_forward_equals_master_forward():
    c = wl.linear_case(13, 6, 64, 40)
    f = po.linear_fwd(c["X"], c["W"], 0.0, 0.3)
    f2 = po.linear_fwd(c["X"], None, 0.0, 0.3, packed=f["P"], mu_lambda=(f["mu"], f["lam"]))
    assert np.array_equal(f["acc"], f2["acc"]) and np.array_equal(f["Y"], f2["Y"])
    f3 = po.decode_gemv(c["X"], f["P"], (f["mu"], f["lam"]), 0.0, 0.3)
    s16 = float(np.float16(np.float32(0.3) * f["lam"]))
    assert np.array_equal(f3["acc"], f["acc"])
    assert np.allclose(f3["Y"], (s16 / f["gamma"].astype(np.float64))[:, None] * f["acc"], rtol=1e-6)


# ---------------------------------------------------------------- router
def test_router_hand_case_ties_and_softmax():
    X = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]], np.float32)
    Wr = np.array([[1.0, 0.0], [1.0, 0.0], [0.0, 2.0], [0.0, -1.0]], np.float32)   # experts 0,1 identical
    idx, gate, p, logits = po.router_topk(X, Wr, 2)
    assert logits.tolist() == [[1, 1, 0, 0], [0, 0, 2, -1], [1, 1, 2, -1]]
    assert idx.tolist() == [[0, 1], [2, 0], [2, 0]]                    # ties -> lower index first
    e = np.exp(np.array([1.0, 1.0, 0.0, 0.0]))
    assert np.allclose(p[0], e / e.sum(), rtol=1e-12)
    assert np.allclose(gate[0], (e / e.sum())[[0, 1]], rtol=1e-12)


def test_router_invariants():
    c = wl.linear_case(14, 200, 64, 32, hp_rank=4, n_experts=8)
    for k in (1, 2):
        idx, gate, p, logits = po.router_topk(c["X"], c["Wr"], k)
        assert idx.shape == (200, k) and all(len(set(r)) == k for r in idx.tolist())
        assert np.bincount(idx.ravel(), minlength=8).sum() == 200 * k
        assert np.allclose(p.sum(axis=1), 1.0) and np.all(gate > 0) and np.all(gate <= 1)
        assert np.array_equal(idx[:, 0], np.argmax(logits, axis=1))
        if k == 2:
            assert np.all(gate[:, 0] >= gate[:, 1])


def test_routed_forward_bruteforce():
    c = wl.linear_case(15, 10, 32, 24, hp_rank=4, n_experts=4)
    f = po.linear_fwd(c["X"], c["W"], 1.0, 0.0, A=c["A"], B=c["B"], Wr=c["Wr"], top_k=2)
    X, A, B, Wr = (c[k].astype(np.float64) for k in ("X", "A", "B", "Wr"))
    for t in range(10):
        lg = np.float32(Wr @ X[t]).astype(np.float64)
        pr = np.exp(lg - lg.max()); pr /= pr.sum()
        order = sorted(range(4), key=lambda e: (-lg[e], e))[:2]
        y = sum(pr[e] * (B[e] @ (A[e] @ X[t])) for e in order)
        assert f["idx"][t].tolist() == order
        assert np.allclose(f["Y"][t], y, rtol=1e-10, atol=1e-14)


# ---------------------------------------------------------------- backward
def _fd(fun, x, eps):
    g = np.zeros_like(x, dtype=np.float64)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps; fp = fun()
        x[i] = old - eps; fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def test_ste_terms_equal_gradients_of_the_bilinear_surrogate():
    """With the STE the 1-bit branch is differentiated as beta * Xv Wv^T at Xv = q/gamma, Wv = lambda S."""
    c = wl.linear_case(16, 6, 32, 8)
    beta = 0.4
    f = po.linear_fwd(c["X"], c["W"], 0.0, beta)
    g = po.linear_bwd(c["dY"], c["X"], c["W"], 0.0, beta, f)
    dY = c["dY"].astype(np.float64)
    Xv = f["q"] / f["gamma"].astype(np.float64)[:, None]
    Wv = float(f["lam"]) * f["S"].astype(np.float64)
    loss = lambda: float((dY * (beta * Xv @ Wv.T)).sum())
    assert np.allclose(g["dX"], _fd(loss, Xv, 1e-3), rtol=1e-6, atol=1e-9)
    assert np.allclose(g["dW"], _fd(loss, Wv, 1e-4), rtol=1e-6, atol=1e-9)
    # brute-force loops of the same formula
    for n in range(8):
        for k in range(0, 32, 7):
            assert np.isclose(g["dW"][n, k], beta * sum(dY[t, n] * Xv[t, k] for t in range(6)), rtol=1e-10)
    bfn = lambda b: float((dY * po.linear_fwd(c["X"], c["W"], 0.0, b)["Y"]).sum())
    assert np.isclose(g["dbeta"], (bfn(beta + 1e-2) - bfn(beta - 1e-2)) / 2e-2, rtol=1e-4)


def test_dense_hp_and_scale_gradients_by_finite_differences():
    c = wl.linear_case(17, 7, 32, 12, hp_rank=4)
    al, be = 1.7, 0.3
    X, A, B = c["X"].astype(np.float64), c["A"].astype(np.float64), c["B"].astype(np.float64)
    dY = c["dY"].astype(np.float64)
    f = po.linear_fwd(X, c["W"], al, be, A=A, B=B)
    g = po.linear_bwd(dY, X, c["W"], al, be, f, A=A, B=B)
    loss = lambda: float((dY * po.linear_fwd(X, c["W"], al, be, A=A, B=B)["Yhp"]).sum()) * al
    assert np.allclose(g["dA"], _fd(loss, A, 1e-5), rtol=1e-5, atol=1e-8)
    assert np.allclose(g["dB"], _fd(loss, B, 1e-5), rtol=1e-5, atol=1e-8)
    # dX = STE part (bilinear surrogate) + true derivative of the hp branch
    ste = be * float(f["lam"]) * dY @ f["S"].astype(np.float64)
    # (X is rounded to fp32 inside the oracle; the hp branch is linear in X, so a coarse probe is exact)
    assert np.allclose(g["dX"] - ste, _fd(loss, X, 2.0 ** -6), rtol=1e-4, atol=1e-7)
    fa = lambda a: float((dY * po.linear_fwd(X, c["W"], a, be, A=A, B=B)["Y"]).sum())
    assert np.isclose(g["dalpha"], (fa(al + 1e-3) - fa(al - 1e-3)) / 2e-3, rtol=1e-6)


def test_gradient_scaling_invariants():
    """Sec. 3.2: alpha scales the hp-branch gradients, beta the 1-bit weight gradient."""
    c = wl.linear_case(18, 7, 32, 12, hp_rank=4)
    f1 = po.linear_fwd(c["X"], c["W"], 1.0, 1.0, A=c["A"], B=c["B"])
    g1 = po.linear_bwd(c["dY"], c["X"], c["W"], 1.0, 1.0, f1, A=c["A"], B=c["B"])
    f2 = po.linear_fwd(c["X"], c["W"], 2.0, 0.2, A=c["A"], B=c["B"])
    g2 = po.linear_bwd(c["dY"], c["X"], c["W"], 2.0, 0.2, f2, A=c["A"], B=c["B"])
    assert np.allclose(g2["dA"], 2.0 * g1["dA"]) and np.allclose(g2["dB"], 2.0 * g1["dB"])
    assert np.allclose(g2["dW"], 0.2 * g1["dW"])
    assert np.isclose(g2["dbeta"], g1["dbeta"]) and np.isclose(g2["dalpha"], g1["dalpha"])


def test_ste_clip_mask():
    c = wl.linear_case(19, 5, 32, 8)
    f = po.linear_fwd(c["X"], c["W"], 0.0, 1.0)
    g_inf = po.linear_bwd(c["dY"], c["X"], c["W"], 0.0, 1.0, f)
    g_tau = po.linear_bwd(c["dY"], c["X"], c["W"], 0.0, 1.0, f, ste_tau=0.02)
    keep = np.abs(c["W"].astype(np.float64) - float(f["mu"])) <= 0.02
    assert 0 < keep.sum() < keep.size
    assert np.array_equal(g_tau["dW"][keep], g_inf["dW"][keep]) and np.all(g_tau["dW"][~keep] == 0)


def test_routed_gradients_by_finite_differences():
    c = wl.linear_case(20, 9, 32, 10, hp_rank=3, n_experts=4, w_std=0.2)
    al, be, k = 1.3, 0.25, 2
    X, A, B, Wr = (c[n].astype(np.float64) for n in ("X", "A", "B", "Wr"))
    dY = c["dY"].astype(np.float64)
    f = po.linear_fwd(X, c["W"], al, be, A=A, B=B, Wr=Wr, top_k=k)
    g = po.linear_bwd(dY, X, c["W"], al, be, f, A=A, B=B, Wr=Wr)

    def loss():
        ff = po.linear_fwd(X, c["W"], al, be, A=A, B=B, Wr=Wr, top_k=k)
        assert np.array_equal(ff["idx"], f["idx"])                    # selection must not flip under the probe
        return al * float((dY * ff["Yhp"]).sum())
    # router logits are rounded to fp32 inside the oracle, so use a probe well above fp32 noise
    assert np.allclose(g["dA"], _fd(loss, A, 1e-3), rtol=2e-3, atol=1e-5)
    assert np.allclose(g["dB"], _fd(loss, B, 1e-3), rtol=2e-3, atol=1e-5)
    assert np.allclose(g["dWr"], _fd(loss, Wr, 1e-3), rtol=2e-3, atol=2e-5)
    ste = be * float(f["lam"]) * dY @ f["S"].astype(np.float64)
    assert np.allclose(g["dX"] - ste, _fd(loss, X, 1e-3), rtol=2e-3, atol=2e-5)


# ---------------------------------------------------------------- decoupled FFN
def test_ffn_forward_is_composition_of_pinned_pieces():
    c = wl.ffn_case(21, 11, 32, 64, 4, 4, bf16=True)
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"],
                   2.0, 0.2, top_k=1, bf16=True)
    up = po.linear_fwd(c["X"], c["W_up"], 0.0, 1.0)["Y"]
    gt = po.linear_fwd(c["X"], c["W_gate"], 0.0, 1.0)["Y"]
    U = wl.bf16_round(up.astype(np.float32)); G = wl.bf16_round(gt.astype(np.float32))
    assert np.array_equal(U, f["U"]) and np.array_equal(G, f["G"])
    hd = (G.astype(np.float64) / (1 + np.exp(-G.astype(np.float64))) * U).astype(np.float32)
    y1 = po.linear_fwd(hd, c["W_down"], 0.0, 1.0)["Y"]
    assert np.allclose(f["Y1"], y1, rtol=1e-6, atol=1e-9)
    X = c["X"].astype(np.float64)
    for t in range(11):
        lg = np.float32(c["Wr"].astype(np.float64) @ X[t]).astype(np.float64)
        e = int(np.argmax(lg)); pr = np.exp(lg - lg.max()); pr /= pr.sum()
        u = c["Up"][e].astype(np.float64) @ X[t]; gg = c["Gate"][e].astype(np.float64) @ X[t]
        y = pr[e] * (c["Down"][e].astype(np.float64) @ (gg / (1 + np.exp(-gg)) * u))
        assert f["idx"][t, 0] == e
        assert np.allclose(f["Y"][t], 0.2 * f["Y1"][t] + 2.0 * y, rtol=1e-9, atol=1e-12)


def test_ffn_expert_and_router_gradients_by_finite_differences():
    c = wl.ffn_case(22, 8, 32, 32, 4, 3, bf16=False, w_std=0.2, outlier_frac=0.0)
    al, be = 1.4, 0.3
    X, Up, Gate, Down, Wr = (c[n].astype(np.float64) for n in ("X", "Up", "Gate", "Down", "Wr"))
    dY = c["dY"].astype(np.float64)
    run = lambda: po.ffn_fwd(X, c["W_up"], c["W_gate"], c["W_down"], Up, Gate, Down, Wr, al, be, top_k=2, bf16=False)
    f = run()
    g = po.ffn_bwd(dY, X, Up, Gate, Down, Wr, al, be, f)

    def loss():
        ff = run()
        assert np.array_equal(ff["idx"], f["idx"])
        return al * float((dY * ff["Yhp"]).sum())
    assert np.allclose(g["dUp"], _fd(loss, Up, 1e-3), rtol=2e-3, atol=2e-5)
    assert np.allclose(g["dGate"], _fd(loss, Gate, 1e-3), rtol=2e-3, atol=2e-5)
    assert np.allclose(g["dDown"], _fd(loss, Down, 1e-3), rtol=2e-3, atol=2e-5)
    assert np.allclose(g["dWr"], _fd(loss, Wr, 1e-3), rtol=2e-3, atol=5e-5)
    fa = lambda a, b: float((dY * po.ffn_fwd(X, c["W_up"], c["W_gate"], c["W_down"], Up, Gate, Down, Wr, a, b,
                                             top_k=2, bf16=False)["Y"]).sum())
    assert np.isclose(g["dalpha"], (fa(al + 1e-3, be) - fa(al - 1e-3, be)) / 2e-3, rtol=1e-6)
    assert np.isclose(g["dbeta"], (fa(al, be + 1e-3) - fa(al, be - 1e-3)) / 2e-3, rtol=1e-6)


def test_ffn_ste_chain_equals_gradients_of_the_smooth_surrogate():
    """The 1-bit FFN differentiated with every quantiser replaced by identity, evaluated at the
    quantised operands: Y1 = (silu(Xv Wg^T) * (Xv Wu^T)) Wd^T with STE around the re-quantiser."""
    c = wl.ffn_case(23, 5, 32, 32, 2, 2, bf16=False, outlier_frac=0.0)
    be = 0.6
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"],
                   0.0, be, top_k=1, bf16=False)
    g = po.ffn_bwd(c["dY"], c["X"], c["Up"], c["Gate"], c["Down"], c["Wr"], 0.0, be, f)
    dY = c["dY"].astype(np.float64)
    st = f["st"]
    Wd = float(st["down"]["lam"]) * st["down"]["S"].astype(np.float64)
    # down projection: bilinear surrogate in (Hv, Wd) at Hv = qh/gamma_h
    Hv = f["qh"] / f["gamma_h"].astype(np.float64)[:, None]
    l_down = lambda: be * float((dY * (Hv @ Wd.T)).sum())
    assert np.allclose(g["dHd"], _fd(l_down, Hv, 1e-4), rtol=1e-6, atol=1e-9)
    assert np.allclose(g["dW_down"], _fd(l_down, Wd, 1e-4), rtol=1e-6, atol=1e-9)   # beta is upstream of the whole FFN
    # gated unit: true derivative of silu(G) * U given upstream dHd
    U, G = f["U"].astype(np.float64), f["G"].astype(np.float64)
    l_act = lambda: float((g["dHd"] * (G / (1 + np.exp(-G)) * U)).sum())
    assert np.allclose(g["dU"], _fd(l_act, U, 1e-6), rtol=1e-6, atol=1e-10)
    assert np.allclose(g["dG"], _fd(l_act, G, 1e-6), rtol=1e-5, atol=1e-10)
    # up / gate projections: bilinear surrogates at Xv = q/gamma
    Xv = f["q"] / f["gamma"].astype(np.float64)[:, None]
    Wu = float(st["up"]["lam"]) * st["up"]["S"].astype(np.float64)
    Wg = float(st["gate"]["lam"]) * st["gate"]["S"].astype(np.float64)
    l_in = lambda: float((g["dU"] * (Xv @ Wu.T)).sum() + (g["dG"] * (Xv @ Wg.T)).sum())
    assert np.allclose(g["dX"], _fd(l_in, Xv, 1e-4), rtol=1e-6, atol=1e-9)       # alpha = 0: no expert/router term
    assert np.allclose(g["dW_up"], _fd(l_in, Wu, 1e-5), rtol=1e-6, atol=1e-9)
    assert np.allclose(g["dW_gate"], _fd(l_in, Wg, 1e-5), rtol=1e-6, atol=1e-9)


def _grid_rows(rng, shape):
    """Rows whose entries already sit on their own AbsMax INT8 grid: integers in [-128, 127] with one -128 per row,
    times a power of two, so that gamma = 128 / absmax is a power of two and quantising changes nothing."""
    q = rng.integers(-127, 128, size=shape).astype(np.float64)
    q[..., 0] = -128.0
    return (q * 2.0 ** -9).astype(np.float32)


def test_ffn_int8_experts_on_grid_inputs_equal_the_float_experts():
    """Sec. 3.2, FFN^INT8: when x and the rows of Up_e, Gate_e, Down_e already lie on their INT8 grids, the quantisers
    of the first two products change nothing, so u and g equal the float experts' exactly (fp32 I/O, small integers), and
    the output differs from the float expert only by the re-quantisation of the hidden state: within a step of its grid
    per hidden unit, summed against Down."""
    rng = np.random.default_rng(61)
    T, d, F, E, r = 7, 32, 32, 3, 8
    c = wl.ffn_case(61, T, d, F, E, r, bf16=False)
    X = _grid_rows(rng, (T, d)); Up = _grid_rows(rng, (E, r, d)); Gate = _grid_rows(rng, (E, r, d)); Down = _grid_rows(rng, (E, d, r))
    args = (X, c["W_up"], c["W_gate"], c["W_down"], Up, Gate, Down, c["Wr"], 1.0, 0.0)
    f8 = po.ffn_fwd(*args, top_k=2, bf16=False, experts="int8")
    ff = po.ffn_fwd(*args, top_k=2, bf16=False)
    assert np.array_equal(f8["idx"], ff["idx"])
    assert np.allclose(f8["ue"], ff["ue"], rtol=1e-6, atol=0) and np.allclose(f8["ge"], ff["ge"], rtol=1e-6, atol=0)
    a = f8["ex8"]["a"].astype(np.float64)
    step = 1.0 / f8["ex8"]["ga"].astype(np.float64)                   # one code step of each (token, slot)
    # half a step, a whole one only where +absmax saturates at code 127 (Sec. 3.1 quantiser)
    dev = np.abs(f8["ex8"]["qa"] / f8["ex8"]["ga"][..., None] - a)
    sat = f8["ex8"]["qa"] == 127
    assert np.all(dev <= np.where(sat, 1.0, 0.5) * step[..., None] * (1 + 1e-4))
    bound = step[..., None] * np.abs(Down.astype(np.float64)).sum(axis=2)[f8["idx"]]     # [T, k, d]
    assert np.all(np.abs(f8["Ys"] - ff["Ys"]) <= bound * (1 + 1e-3) + 1e-9)
    assert np.abs(f8["Ys"] - ff["Ys"]).max() > 0                       # ... and the re-quantisation is really there


@pytest.mark.parametrize("bf16", [False, True])
def test_ffn_int8_experts_track_the_float_experts(bf16):
    """On ordinary inputs the INT8 experts stay within the quantisation error of the float experts: three quantised
    operands with relative step 1/128 each."""
    c = wl.ffn_case(62, 40, 64, 96, 4, 16, bf16=bf16, outlier_frac=0.0)
    args = (c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2)
    f8 = po.ffn_fwd(*args, top_k=2, bf16=bf16, experts="int8")
    ff = po.ffn_fwd(*args, top_k=2, bf16=bf16)
    assert np.array_equal(f8["idx"], ff["idx"]) and np.array_equal(f8["Y1"], ff["Y1"])
    err = np.abs(f8["Yhp"] - ff["Yhp"]).max() / np.abs(ff["Yhp"]).max()
    assert 1e-4 < err < 5e-2
    # codes of the weights are the activation quantiser applied to their rows
    q_u, g_u = f8["ex8"]["qw"]["up"][1]
    assert np.array_equal(q_u, po.quant_act(c["Up"][1])[0]) and np.array_equal(g_u, po.quant_act(c["Up"][1])[1])


def test_ffn_int8_experts_backward_is_the_gradient_of_the_dequantised_surrogate():
    """STE (App. B.1): with every quantiser read as the identity, the expert is Down~ a with a = silu(Gate~ x~) * (Up~ x~).
    Finite differences of that smooth function at the de-quantised factors reproduce dUp, dGate and the experts' share
    of dX; dDown is linear in Down~ with the quantised hidden state a~ held fixed.  The stored u, g (I/O rounding) and a~
    (re-quantised) differ from the surrogate's exact values by their rounding, hence the tolerances."""
    c = wl.ffn_case(63, 6, 32, 32, 2, 8, bf16=False, w_std=0.3, outlier_frac=0.0)
    al = 1.7
    args = (c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], al, 0.0)
    f = po.ffn_fwd(*args, top_k=1, bf16=False, experts="int8")
    dY = c["dY"].astype(np.float64)
    g = po.ffn_bwd(dY, c["X"], c["Up"], c["Gate"], c["Down"], c["Wr"], al, 0.0, f)
    E = 2
    deq = lambda qg: qg[0].astype(np.float64) / qg[1].astype(np.float64)[:, None]
    Upt = np.stack([deq(f["ex8"]["qw"]["up"][e]) for e in range(E)])
    Gtt = np.stack([deq(f["ex8"]["qw"]["gate"][e]) for e in range(E)])
    Dnt = np.stack([deq(f["ex8"]["qw"]["down"][e]) for e in range(E)])
    Xt = f["q"].astype(np.float64) / f["gamma"].astype(np.float64)[:, None]
    idx, gate = f["idx"][:, 0], f["gate"][:, 0].astype(np.float64)
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))

    def loss(Up_, Gt_, Dn_, X_):
        tot = 0.0
        for t in range(6):
            e = idx[t]
            gg = Gt_[e] @ X_[t]; u = Up_[e] @ X_[t]
            tot += al * gate[t] * float(dY[t] @ (Dn_[e] @ (gg * sig(gg) * u)))
        return tot
    fd_up = _fd(lambda: loss(Upt, Gtt, Dnt, Xt), Upt, 1e-5)
    fd_gt = _fd(lambda: loss(Upt, Gtt, Dnt, Xt), Gtt, 1e-5)
    fd_x = _fd(lambda: loss(Upt, Gtt, Dnt, Xt), Xt, 1e-5)
    scale = lambda a: np.abs(a).max()
    assert np.abs(g["dUp"] - fd_up).max() <= 2e-2 * scale(fd_up)
    assert np.abs(g["dGate"] - fd_gt).max() <= 2e-2 * scale(fd_gt)
    dX_router = po._router_bwd(g["dgate"] if "dgate" in g else np.einsum("ti,tji->tj", al * dY, f["Ys"]), f["idx"], f["probs"],
                               c["X"].astype(np.float64), c["Wr"].astype(np.float64))[1]
    assert np.abs((g["dX"] - dX_router) - fd_x).max() <= 2e-2 * scale(fd_x)
    # dDown: linear in Down~ with the quantised hidden state fixed -- compare with the explicit sum over tokens
    a_t = f["ex8"]["qa"][:, 0].astype(np.float64) / f["ex8"]["ga"][:, 0].astype(np.float64)[:, None]
    for e in range(E):
        ref = sum(al * gate[t] * np.outer(dY[t], a_t[t]) for t in range(6) if idx[t] == e)
        assert np.allclose(g["dDown"][e], ref, rtol=1e-12, atol=1e-15)


def test_workload_generators_are_seeded_and_bf16_exact():
    a, b = wl.config1(), wl.config1()
    assert all(np.array_equal(a[k], b[k]) for k in ("W", "X", "dY", "A", "B"))
    c = wl.linear_case(1, 8, 64, 32, hp_rank=8, bf16=True)
    for k in ("W", "X", "dY", "A", "B"):
        wl.bf16_bits(c[k])                                            # asserts representability
    col_energy = (a["X"].astype(np.float64) ** 2).mean(axis=0)
    assert (col_energy > 30).sum() == 4                               # the four x10 outlier channels


# ---------------------------------------------------------------------------------------------------
# Layer stack (config 5): wiring pins.  The pieces (linear, FFN) are pinned above; these cases fix the
# residual connections, the q/k/v average and the order of the backward chain.
# ---------------------------------------------------------------------------------------------------
def _tiny_stack(seed, n_layers=2, tokens=12, d=32, f=64, e=2, r=8):
    return wl.stack_case(seed, n_layers, tokens, d, f, e, r, vocab=50)


def test_stack_is_the_identity_when_the_output_projections_vanish():
    """An all-zero latent matrix has lambda = 0, so its 1-bit linear returns exactly 0.  With W_o = W_down = 0 and
    alpha = 0 both residual branches add nothing: the stack must hand its (bf16) input through unchanged, and the
    backward pass must hand the upstream gradient through unchanged."""
    c = _tiny_stack(5)
    for w in c["layers"]:
        w["Wo"] = np.zeros_like(w["Wo"]); w["W_down"] = np.zeros_like(w["W_down"]); w["alpha"] = 0.0
    h0 = c["table"][c["ids"]]
    out, saved = po.stack_fwd(h0, c["layers"])
    np.testing.assert_array_equal(np.asarray(out, np.float64), wl.bf16_round(h0).astype(np.float64))
    dY = c["dY"]
    d0, grads = po.stack_bwd(dY, c["layers"], saved)
    np.testing.assert_allclose(np.asarray(d0, np.float64), dY.astype(np.float64), rtol=0, atol=0)
    # W_o = 0 still receives a gradient (it depends on dY and the codes of m, not on lambda)
    assert np.abs(grads[0]["Wo"]).max() > 0


def test_stack_averages_q_k_v():
    """With W_q = W_k = W_v the stand-in for the attention core is (3 q) / 3 = q exactly, so the first half of a layer
    must equal h + L_o(L_q(h)) built by hand from the pinned linear."""
    c = _tiny_stack(6, n_layers=1)
    w = c["layers"][0]
    w["Wk"] = w["Wq"].copy(); w["Wv"] = w["Wq"].copy()
    h0 = wl.bf16_round(c["table"][c["ids"]])
    _, saved = po.stack_fwd(h0, c["layers"])
    q = wl.bf16_round(po.linear_fwd(h0, w["Wq"], 0.0, 1.0)["Y"].astype(np.float32))
    o = wl.bf16_round(po.linear_fwd(q, w["Wo"], 0.0, 1.0)["Y"].astype(np.float32))
    h1 = wl.bf16_round((h0.astype(np.float64) + o).astype(np.float32))
    np.testing.assert_array_equal(np.asarray(saved[0]["m"], np.float32), q)
    np.testing.assert_array_equal(np.asarray(saved[0]["h1"], np.float32), h1)


def test_stack_backward_carries_the_one_third_of_the_q_k_v_average():
    """With W_q = W_k = W_v, the FFN switched off (W_down = 0 gives lambda = 0, alpha = 0) and a non-zero W_o, the
    backward of one layer is d = dY + 3 * dX_q(dX_o(dY) / 3) = dY + dX_q(dX_o(dY)) by the linearity of the STE
    backward, built here by hand from the pinned linear_bwd; the weight gradient of W_q sees a third of dX_o(dY).
    A dropped or doubled 1/3 changes both."""
    c = _tiny_stack(8, n_layers=1)
    w = c["layers"][0]
    w["Wk"] = w["Wq"].copy(); w["Wv"] = w["Wq"].copy()
    w["W_down"] = np.zeros_like(w["W_down"]); w["alpha"] = 0.0
    h0 = wl.bf16_round(c["table"][c["ids"]])
    _, saved = po.stack_fwd(h0, c["layers"])
    dY = c["dY"].astype(np.float64)
    d0, grads = po.stack_bwd(dY, c["layers"], saved)
    fq = po.linear_fwd(h0, w["Wq"], 0.0, 1.0)
    m = wl.bf16_round(fq["Y"].astype(np.float32))
    fo = po.linear_fwd(m, w["Wo"], 0.0, 1.0)
    go = po.linear_bwd(dY, m, w["Wo"], 0.0, 1.0, fo)
    assert np.abs(go["dX"]).max() > 0
    gq = po.linear_bwd(go["dX"], h0, w["Wq"], 0.0, 1.0, fq)
    ref = dY + gq["dX"]
    assert np.abs(np.asarray(d0, np.float64) - ref).max() <= 1e-12 * np.abs(ref).max()
    for n in ("Wq", "Wk", "Wv"):
        assert np.abs(grads[0][n] - gq["dW"] / 3.0).max() <= 1e-12 * np.abs(gq["dW"]).max()
    np.testing.assert_array_equal(grads[0]["Wo"], go["dW"])


def test_stack_backward_is_linear_in_the_upstream_gradient():
    """The STE backward is a linear map of dY.  Scaling by 2 commutes with every rounding (exact), a sum of two
    upstream gradients gives the sum of the results up to the bf16 roundings of the stored gradients."""
    c = _tiny_stack(7)
    h0 = c["table"][c["ids"]]
    _, saved = po.stack_fwd(h0, c["layers"])
    rng = np.random.default_rng(70)
    dA = wl.bf16_round(rng.standard_normal(c["dY"].shape).astype(np.float32))
    dB = wl.bf16_round(rng.standard_normal(c["dY"].shape).astype(np.float32))
    xa, ga = po.stack_bwd(dA, c["layers"], saved)
    x2, g2 = po.stack_bwd(2.0 * dA, c["layers"], saved)
    np.testing.assert_array_equal(np.asarray(x2, np.float64), 2.0 * np.asarray(xa, np.float64))
    np.testing.assert_array_equal(np.asarray(g2[0]["Wq"], np.float64), 2.0 * np.asarray(ga[0]["Wq"], np.float64))
    xb, gb = po.stack_bwd(dB, c["layers"], saved)
    xs, gs = po.stack_bwd(dA + dB, c["layers"], saved)
    ref = np.asarray(xa, np.float64) + np.asarray(xb, np.float64)
    assert np.abs(np.asarray(xs, np.float64) - ref).max() <= 2e-2 * np.abs(ref).max()
    refw = np.asarray(ga[1]["W_up"], np.float64) + np.asarray(gb[1]["W_up"], np.float64)
    assert np.abs(np.asarray(gs[1]["W_up"], np.float64) - refw).max() <= 2e-2 * np.abs(refw).max()


# ------------------------------------------------------------------------------------------------
# Normalisation fused with the quantiser (Sec. 3.1 Q(Norm(X)); App. A; App. B)
# ------------------------------------------------------------------------------------------------
def test_rmsnorm_hand_cases():
    # x = (3, 4): mean square 12.5, so x_hat = (3, 4) / sqrt(12.5) times the gain
    xn, rstd = po.rmsnorm(np.array([[3.0, 4.0]], np.float32), np.array([1.0, 2.0], np.float32), 0.0)
    assert abs(float(rstd[0]) - 1.0 / math.sqrt(12.5)) < 1e-7
    assert np.allclose(xn[0], [3.0 / math.sqrt(12.5), 8.0 / math.sqrt(12.5)], rtol=3e-7, atol=0)
    # a constant row normalises to the sign of the constant times the gain
    g = np.array([0.5, -1.0, 2.0, 4.0], np.float32)
    xn, _ = po.rmsnorm(np.full((1, 4), -7.0, np.float32), g, 0.0)
    assert np.allclose(xn[0], -g, rtol=3e-7, atol=0)
    # eps dominates a zero row: the output is zero and rstd = eps^(-1/2)
    xn, rstd = po.rmsnorm(np.zeros((1, 8), np.float32), np.ones(8, np.float32), 1e-6)
    assert np.all(xn == 0) and abs(float(rstd[0]) - 1000.0) < 1e-3


@pytest.mark.parametrize("seed", [0, 1])
def test_rmsnorm_invariants(seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((9, 96)).astype(np.float32)
    X[:, 5] *= 30.0
    ones = np.ones(96, np.float32)
    xn, rstd = po.rmsnorm(X, ones, 0.0)
    # unit mean square per token
    assert np.allclose(np.mean(xn.astype(np.float64) ** 2, axis=1), 1.0, rtol=2e-6)
    # scaling a token by a power of two changes nothing, bit for bit (every operation scales exactly)
    xn4, rstd4 = po.rmsnorm(X * np.float32(4.0), ones, 0.0)
    assert np.array_equal(xn4, xn) and np.array_equal(rstd4 * np.float32(4.0), rstd)
    # any positive scale leaves the result unchanged up to rounding
    xn3, _ = po.rmsnorm(X * np.float32(3.0), ones, 0.0)
    assert np.allclose(xn3, xn, rtol=1e-6, atol=1e-7)
    # the gain multiplies channel-wise
    g = rng.standard_normal(96).astype(np.float32)
    xg, _ = po.rmsnorm(X, g, 0.0)
    assert np.allclose(xg, xn * g[None, :], rtol=2e-7, atol=0)


def test_rmsnorm_quant_is_the_quantiser_of_the_stored_normalised_rows():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((17, 64)).astype(np.float32) * 5.0
    g = (1.0 + 0.1 * rng.standard_normal(64)).astype(np.float32)
    for bf16 in (False, True):
        f = po.rmsnorm_quant_fwd(X, g, 1e-6, bf16=bf16)
        # codes: brute force from the definition of Q on the stored x_hat, element by element
        for t in range(X.shape[0]):
            row = f["Xn"][t]
            gam = np.float32(128.0) / max(np.float32(np.max(np.abs(row))), np.float32(1e-5))
            assert gam == f["gamma"][t]
            for k in range(X.shape[1]):
                code = int(min(127, max(-128, np.rint(np.float32(row[k] * gam)))))
                assert code == int(f["q"][t, k])
        # every token reaches the top code: |q| hits 127 or 128-clamped
        assert np.all(np.max(np.abs(f["q"].astype(np.int32)), axis=1) >= 127)
        # de-quantised activations stay within half a step of the stored ones (a full step where +absmax,
        # which maps to 128, was clamped to 127)
        step = 1.0 / f["gamma"][:, None].astype(np.float64)
        assert np.all(np.abs(f["Xt"].astype(np.float64) - f["Xn"]) <= step * (0.5 + 0.5 * (f["q"] == 127) + 1e-4))
        if bf16:   # stored rows are bf16 values
            import torch
            t32 = torch.from_numpy(f["Xn"])
            assert torch.equal(t32.to(torch.bfloat16).to(torch.float32), t32)


def test_rmsnorm_backward_by_finite_differences_and_orthogonality():
    rng = np.random.default_rng(11)
    T, K = 4, 12
    X = rng.standard_normal((T, K))
    g = 1.0 + 0.2 * rng.standard_normal(K)
    C = rng.standard_normal((T, K))            # L = sum(C * x_hat)
    eps = 1e-3

    def loss(Xv, gv):
        # fp64 evaluation of the forward definition through the oracle itself would round to fp32;
        # central differences need fp64, so the loss is the forward oracle applied to fp32-exact inputs
        # scaled up: use the identity x_hat(X) computed in fp64 from the printed formula
        ms = np.mean(Xv ** 2, axis=1, keepdims=True)
        return float(np.sum(C * (Xv / np.sqrt(ms + eps) * gv[None, :])))

    # the fp64 formula above and the oracle forward agree to fp32 rounding (ties the two together)
    xn, rstd = po.rmsnorm(X.astype(np.float32), g.astype(np.float32), eps)
    X32, g32 = X.astype(np.float32).astype(np.float64), g.astype(np.float32).astype(np.float64)
    ms = np.mean(X32 ** 2, axis=1, keepdims=True)
    assert np.allclose(xn, X32 / np.sqrt(ms + eps) * g32[None, :], rtol=3e-7, atol=1e-7)
    dx, dg = po.rmsnorm_bwd(C, X32, g32, (1.0 / np.sqrt(ms[:, 0] + eps)))
    h = 1e-6
    for (t, k) in [(0, 0), (1, 5), (3, 11), (2, 7)]:
        Xp, Xm = X32.copy(), X32.copy()
        Xp[t, k] += h
        Xm[t, k] -= h
        assert abs((loss(Xp, g32) - loss(Xm, g32)) / (2 * h) - dx[t, k]) < 1e-7
    for k in (0, 4, 11):
        gp, gm = g32.copy(), g32.copy()
        gp[k] += h
        gm[k] -= h
        assert abs((loss(X32, gp) - loss(X32, gm)) / (2 * h) - dg[k]) < 1e-7
    # without eps x_hat does not depend on the length of x, so the gradient is orthogonal to x
    ms0 = np.mean(X32 ** 2, axis=1)
    dx0, _ = po.rmsnorm_bwd(C, X32, g32, 1.0 / np.sqrt(ms0))
    assert np.all(np.abs(np.sum(dx0 * X32, axis=1)) < 1e-12)
    # linear in the upstream gradient
    dx2, dg2 = po.rmsnorm_bwd(2.0 * C, X32, g32, 1.0 / np.sqrt(ms[:, 0] + eps))
    assert np.allclose(dx2, 2.0 * dx, rtol=1e-14) and np.allclose(dg2, 2.0 * dg, rtol=1e-14)


# ------------------------------------------------------------------------------------------------
# INT8 form of the high-precision branch (Sec. 3.2)
# ------------------------------------------------------------------------------------------------
def test_hp_int8_integer_grid_inputs_give_the_exact_product():
    """Rows that already sit on the INT8 grid with gamma = 1 (most negative entry -128) are their own codes,
    so the first product must be the exact integer matrix product, entry by entry (Python integers)."""
    rng = np.random.default_rng(5)
    T, n, r, m = 5, 32, 8, 6
    X = rng.integers(-100, 100, size=(T, n)).astype(np.float32); X[:, 0] = -128
    A = rng.integers(-100, 100, size=(r, n)).astype(np.float32); A[:, 1] = -128
    B = rng.integers(-100, 100, size=(m, r)).astype(np.float32); B[:, 2] = -128
    f = po.hp_int8_fwd(X, A, B)
    assert np.all(f["g_x"] == 1.0) and np.all(f["g_a"] == 1.0) and np.all(f["g_b"] == 1.0)
    assert np.array_equal(f["q_x"], X.astype(np.int8)) and np.array_equal(f["q_a"], A.astype(np.int8))
    for t in range(T):
        for j in range(r):
            assert int(f["acc1"][t, j]) == sum(int(X[t, k]) * int(A[j, k]) for k in range(n))
            assert float(f["H"][t, j]) == float(f["acc1"][t, j])          # below 2^24: exact in fp32
    for t in range(T):
        for i in range(m):
            assert int(f["acc2"][t, i]) == sum(int(f["q_h"][t, j]) * int(f["q_b"][i, j]) for j in range(r))
    # the hidden state is re-quantised per token: its codes reach 127 or -128 in every row
    assert np.all(np.max(np.abs(f["q_h"].astype(np.int32)), axis=1) >= 127)


@pytest.mark.parametrize("bf16", [False, True])
def test_hp_int8_stays_within_the_quantisation_error_of_the_float_branch(bf16):
    rng = np.random.default_rng(9)
    T, n, r, m = 48, 256, 32, 64
    X = wl.activations(rng, T, n, bf16=bf16)
    A = wl.normal(rng, (r, n), 0.02, bf16)
    B = wl.normal(rng, (m, r), 0.02, bf16)
    f = po.hp_int8_fwd(X, A, B, bf16=bf16)
    ref = (X.astype(np.float64) @ A.astype(np.float64).T) @ B.astype(np.float64).T
    # three INT8 grids with uniform rounding error of 1/256 of each row maximum, averaged over 256- and 32-term sums
    err = np.abs(f["Yhp"] - ref).max() / np.abs(ref).max()
    assert err < 0.05
    # codes and gammas of X are the quantiser's; passing them in changes nothing
    q, g = po.quant_act(X)
    f2 = po.hp_int8_fwd(X, A, B, bf16=bf16, q_gamma=(q, g))
    assert np.array_equal(f2["Yhp"], f["Yhp"])
    # scaling a row of A by a power of two scales its gamma and leaves codes and result bits unchanged otherwise
    A2 = A.copy(); A2[3] *= 4.0
    f3 = po.hp_int8_fwd(X, A2, B, bf16=False)
    f1 = po.hp_int8_fwd(X, A, B, bf16=False)
    assert np.array_equal(f3["q_a"], f1["q_a"]) and f3["g_a"][3] * 4.0 == f1["g_a"][3]
    assert np.array_equal(f3["H"][:, 3], (f1["H"][:, 3] * np.float32(4.0)))


def test_hp_int8_backward_is_the_gradient_of_the_dequantised_bilinear_form():
    """STE: with the codes frozen, Y = (X~ A~^T -> H~) B~^T is bilinear in (H~, B~) and (X~, A~); the backward
    must equal the derivatives of <C, H' B'^T> and <dH, X' A'^T> at the de-quantised points (central
    differences are exact for bilinear forms up to rounding)."""
    rng = np.random.default_rng(13)
    T, n, r, m = 6, 32, 8, 5
    X = rng.standard_normal((T, n)).astype(np.float32)
    A = (0.1 * rng.standard_normal((r, n))).astype(np.float32)
    B = (0.1 * rng.standard_normal((m, r))).astype(np.float32)
    C = rng.standard_normal((T, m))
    f = po.hp_int8_fwd(X, A, B)
    g = po.hp_int8_bwd(C, f)
    Xt = f["q_x"].astype(np.float64) / f["g_x"].astype(np.float64)[:, None]
    At = f["q_a"].astype(np.float64) / f["g_a"].astype(np.float64)[:, None]
    Bt = f["q_b"].astype(np.float64) / f["g_b"].astype(np.float64)[:, None]
    Ht = f["q_h"].astype(np.float64) / f["g_h"].astype(np.float64)[:, None]
    h = 1e-3
    L2 = lambda Hm, Bm: float(np.sum(C * (Hm @ Bm.T)))
    L1 = lambda Xm, Am: float(np.sum(g["dH"] * (Xm @ Am.T)))
    for (i, j) in [(0, 0), (4, 7), (2, 3)]:
        E = np.zeros_like(Bt); E[i, j] = h
        assert abs((L2(Ht, Bt + E) - L2(Ht, Bt - E)) / (2 * h) - g["dB"][i, j]) < 1e-9
    for (t, j) in [(0, 0), (5, 7)]:
        E = np.zeros_like(Ht); E[t, j] = h
        assert abs((L2(Ht + E, Bt) - L2(Ht - E, Bt)) / (2 * h) - g["dH"][t, j]) < 1e-9
    for (j, k) in [(0, 0), (7, 31), (3, 10)]:
        E = np.zeros_like(At); E[j, k] = h
        assert abs((L1(Xt, At + E) - L1(Xt, At - E)) / (2 * h) - g["dA"][j, k]) < 1e-9
    for (t, k) in [(0, 0), (5, 31)]:
        E = np.zeros_like(Xt); E[t, k] = h
        assert abs((L1(Xt + E, At) - L1(Xt - E, At)) / (2 * h) - g["dX"][t, k]) < 1e-9
    # the de-quantised hidden state is within half a step of the stored one
    assert np.all(np.abs(Ht - f["H"]) <= (0.5 + 0.5 * (f["q_h"] == 127) + 1e-4) / f["g_h"].astype(np.float64)[:, None])


def test_decode_int8_experts_reduce_to_the_dense_int8_branch_and_track_the_float_experts():
    """One expert and top-1: the softmax gate over a single logit is exactly 1, so the routed INT8 decode must be
    the 1-bit product plus alpha times the dense INT8 branch, bit for bit.  With several experts the result stays
    within the INT8 quantisation error of the bf16-expert decode (same routing, same 1-bit branch)."""
    rng = np.random.default_rng(21)
    T, n, m, r, E = 3, 256, 64, 32, 4
    x = wl.activations(rng, T, n, bf16=True)
    W = wl.normal(rng, (m, n), 0.02, True)
    A = wl.normal(rng, (E, r, n), 0.02, True)
    B = wl.normal(rng, (E, m, r), 0.02, True)
    Wr = wl.normal(rng, (E, n), 0.05, True)
    mu, lam = po.weight_stats(W)
    P = po.pack_sign(po.binarise(W, mu))
    alpha, beta = 0.7, 0.9
    one = po.decode_gemv_int8(x, P, (mu, lam), alpha, beta, A[:1], B[:1], Wr[:1], top_k=1)
    assert np.all(one["gate"] == 1.0) and np.all(one["idx"] == 0)
    dense = po.hp_int8_fwd(x, A[0], B[0], bf16=True)
    plain = po.decode_gemv(x, P, (mu, lam), 0.0, beta)
    assert np.array_equal(one["acc"], plain["acc"])
    assert np.array_equal(one["Y"], plain["Y1"].astype(np.float64) + alpha * dense["Yhp"].astype(np.float64))
    assert np.array_equal(one["Hs"][:, 0], dense["H"])
    # several experts against the float experts
    f8 = po.decode_gemv_int8(x, P, (mu, lam), alpha, beta, A, B, Wr, top_k=2)
    ff = po.decode_gemv(x, P, (mu, lam), alpha, beta, A=A, B=B, Wr=Wr, top_k=2)
    assert np.array_equal(f8["idx"], ff["idx"]) and np.array_equal(f8["gate"], ff["gate"])
    assert np.abs(f8["Yhp"] - ff["Yhp"]).max() / np.abs(ff["Yhp"]).max() < 0.05
    # brute force of one output element from the stored codes (Python integers and one division chain)
    t, j, i = 1, 1, 5
    e = int(f8["idx"][t, j])
    qa, ga = po.quant_act(A[e]); qb, gb = po.quant_act(B[e]); qx, gx = po.quant_act(x)
    h = np.zeros(r, np.float32)
    for jj in range(r):
        a1 = sum(int(qx[t, k]) * int(qa[jj, k]) for k in range(n))
        h[jj] = np.float32(np.float32(np.float32(1.0) / gx[t]) * np.float32(a1)) / ga[jj]
    h = po._round_io(h, True)
    assert np.array_equal(h, f8["Hs"][t, j])
    qh, gh = po.quant_act(h[None, :])
    a2 = sum(int(qh[0, jj]) * int(qb[i, jj]) for jj in range(r))
    y = np.float32(np.float32(np.float32(1.0) / gh[0]) * np.float32(a2)) / gb[i]
    assert y == f8["Ys"][t, j, i]


def test_decode_ffn_agrees_with_the_training_forward_and_with_chained_decode_products():
    """decode_ffn is ffn_fwd read from packed bits with fp16-folded scales.  With weights whose lambda and
    beta * lambda are exactly representable in fp16 the two must agree to fp32 rounding; its three 1-bit products
    are those of decode_gemv (a different code path through linear_fwd), bit for bit; one expert output is
    recomputed with plain Python floats."""
    rng = np.random.default_rng(31)
    T, d, f, r, E = 3, 128, 256, 8, 4
    x = wl.activations(rng, T, d, bf16=True)
    def pm(shape, a):                                    # +/- a around a zero mean: mu = 0, lambda = a exactly
        W = np.where(rng.random(shape) < 0.5, -a, a).astype(np.float32)
        W.reshape(-1)[: W.size // 2] = a; W.reshape(-1)[W.size // 2:] = -a
        return rng.permuted(W.reshape(-1)).reshape(shape)
    Wu, Wg, Wd = pm((f, d), 0.03125), pm((f, d), 0.0625), pm((d, f), 0.015625)
    Up = wl.normal(rng, (E, r, d), 0.05, True); Gate = wl.normal(rng, (E, r, d), 0.05, True)
    Down = wl.normal(rng, (E, d, r), 0.05, True); Wr = wl.normal(rng, (E, d), 0.05, True)
    alpha, beta = 1.5, 0.5
    packs = []
    for W in (Wu, Wg, Wd):
        mu, lam = po.weight_stats(W)
        assert mu == 0.0
        packs.append((po.pack_sign(po.binarise(W, mu)), lam))
    (Pu, lu), (Pg, lg), (Pd, ld) = packs
    dec = po.decode_ffn(x, Pu, Pg, Pd, lu, lg, ld, Up, Gate, Down, Wr, alpha, beta, top_k=2)
    trn = po.ffn_fwd(x, Wu, Wg, Wd, Up, Gate, Down, Wr, alpha, beta, top_k=2, bf16=True)
    assert np.array_equal(dec["U"], trn["U"]) and np.array_equal(dec["G"], trn["G"])
    assert np.array_equal(dec["qh"], trn["qh"]) and np.array_equal(dec["acc_d"], trn["acc_d"])
    assert np.array_equal(dec["idx"], trn["idx"])
    assert np.abs(dec["Y"] - trn["Y"]).max() <= 1e-6 * np.abs(trn["Y"]).max()
    # the three products through decode_gemv
    up = po.decode_gemv(x, Pu, (0.0, lu), 0.0, 1.0)
    assert np.array_equal(up["acc"], dec["acc_u"]) and np.array_equal(po._round_io(up["Y1"], True), dec["U"])
    dn = po.decode_gemv(dec["Hd"], Pd, (0.0, ld), 0.0, beta)
    assert np.array_equal(dn["acc"], dec["acc_d"]) and np.array_equal(dn["Y1"], dec["Y1"])
    # one expert output element by hand
    t, j, i = 2, 1, 7
    e = int(dec["idx"][t, j])
    y = 0.0
    for k in range(r):
        u = sum(float(Up[e, k, c]) * float(x[t, c]) for c in range(d))
        g = sum(float(Gate[e, k, c]) * float(x[t, c]) for c in range(d))
        y += float(Down[e, i, k]) * (g / (1.0 + math.exp(-g))) * u
    want = float(dec["Y1"][t, i]) + alpha * sum(
        float(dec["gate"][t, jj]) * (y if jj == j else float((np.asarray(Down[int(dec["idx"][t, jj])], np.float64) @ dec["act"][t, jj])[i]))
        for jj in range(2))
    assert abs(want - dec["Y"][t, i]) <= 1e-9 * max(1.0, abs(want))


# ---------------------------------------------------------------------------- group-wise scales (Sec. 4.6 ablation)
def test_groupwise_scales_hand_case_and_sixteen_bit_rounding():
    """One row, two groups of four: means 2.5 and 0.1 (the latter is not an fp16 number: 0.0999755859375 is)."""
    W = np.array([[1.0, -2.0, 3.0, -4.0, 0.1, -0.1, 0.1, -0.1]], np.float64)
    lg = po.groupwise_scales(W, group=4)
    assert lg.shape == (1, 2) and lg.dtype == np.float32
    assert lg[0, 0] == np.float32(2.5)
    assert lg[0, 1] == np.float32(0.0999755859375)


def test_groupwise_forward_bruteforce():
    """Python-loop evaluation of the defining double sum on a tiny case (no matmul, no reshape)."""
    rng = np.random.default_rng(2301)
    T, n, m, group = 3, 8, 2, 4
    X = rng.standard_normal((T, n)).astype(np.float32)
    W = (0.05 * rng.standard_normal((m, n))).astype(np.float32)
    out = po.groupwise_fwd(X, W, beta=1.5, group=group)
    mu = np.float32(np.float64(W.astype(np.float64).sum()) / W.size)
    for t in range(T):
        amax = max(abs(float(v)) for v in X[t])
        gamma = np.float32(128.0) / np.float32(amax)
        q = [int(np.clip(np.rint(np.float32(X[t, j]) * gamma), -128, 127)) for j in range(n)]
        for i in range(m):
            y = 0.0
            for g in range(n // group):
                cols = range(g * group, (g + 1) * group)
                lam = float(np.float16(np.float32(sum(abs(float(W[i, j])) for j in cols) / group)))
                y += lam * sum((1 if W[i, j] >= mu else -1) * q[j] for j in cols)
            assert out["Y"][t, i] == pytest.approx(1.5 * y / float(gamma), rel=1e-12, abs=1e-300)


def test_groupwise_reduces_to_per_tensor_when_all_magnitudes_agree():
    """|W| constant (an fp16 number): every group scale equals lambda, so the group-wise product is the per-tensor one."""
    rng = np.random.default_rng(2302)
    T, n, m = 5, 128, 7
    c = np.float32(0.03125)
    W = (c * rng.choice([-1.0, 1.0], size=(m, n))).astype(np.float32)
    X = rng.standard_normal((T, n)).astype(np.float32)
    a = po.groupwise_fwd(X, W, beta=0.7, group=64)
    b = po.groupwise_fwd(X, W, beta=0.7, group=0)
    assert np.all(a["lam_group"] == c) and b["lam"] == c
    np.testing.assert_allclose(a["Y"], b["Y"], rtol=1e-13, atol=0)
    # and the per-tensor form is the 1-bit linear of the layer forward (alpha = 0, no branch), whose scale products are
    # rounded to fp32 once each
    ref = po.linear_fwd(X, W, alpha=0.0, beta=0.7)
    np.testing.assert_allclose(b["Y"], ref["Y"], rtol=1e-6, atol=1e-300)


def test_groupwise_one_group_per_row_is_the_channel_wise_closed_form():
    rng = np.random.default_rng(2303)
    T, n, m = 4, 64, 6
    W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    X = rng.standard_normal((T, n)).astype(np.float32)
    out = po.groupwise_fwd(X, W, beta=1.0, group=n)
    mu, _ = po.weight_stats(W)
    S = po.binarise(W, mu).astype(np.float64)
    q, gamma = po.quant_act(X)
    lam_row = np.abs(W.astype(np.float64)).mean(axis=1).astype(np.float32).astype(np.float16).astype(np.float64)
    ref = (q.astype(np.float64) @ S.T) * lam_row[None, :] / gamma.astype(np.float64)[:, None]
    np.testing.assert_allclose(out["Y"], ref, rtol=1e-13, atol=0)


def test_groupwise_tracks_the_weights_better_than_one_scale():
    """What the ablation is about: with per-group scales lambda_g Sign(W - mu) is closer to W than with one lambda
    whenever the magnitude varies along a row (here: by a factor of four between the halves of every row)."""
    rng = np.random.default_rng(2304)
    m, n = 16, 256
    W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    W[:, n // 2:] *= 4.0
    mu, lam = po.weight_stats(W)
    S = po.binarise(W, mu).astype(np.float64)
    lg = np.repeat(po.groupwise_scales(W, 64).astype(np.float64), 64, axis=1)
    err_group = np.linalg.norm(lg * S - W)
    err_tensor = np.linalg.norm(float(lam) * S - W)
    assert err_group < 0.9 * err_tensor
