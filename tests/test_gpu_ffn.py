"""Parity of the decoupled FFN (1-bit up/gate/down + routed bf16 experts; Sec. 3.2, 3.3) against the
CPU oracle: outputs and gradients within 2e-2 (bf16 I/O) in the max-norm relative error, the relative L2 error and,
for the weight gradients of the 1-bit projections, every input channel by itself (tests/parity_metrics.py)."""
import os

import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl
from parity_metrics import relerr, report

pytestmark = pytest.mark.gpu
TOL = 2e-2
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda().to(torch.bfloat16)


def run_ffn(c, top_k, alpha, beta, experts="bf16"):
    T, D, F, E, r = c["tokens"], c["d_model"], c["d_ffn"], c["n_experts"], c["hp_rank"]
    kind = pq.PQ_HP_LOWRANK_INT8 if experts == "int8" else pq.PQ_HP_LOWRANK_BF16
    desc = pq.FFNDesc(T, D, F, r, E, top_k, pq.PQ_BF16, alpha, beta, kind)
    bufs = pq.FFNBuffers(desc)
    t = {k: dev(c[k]) for k in ("X", "dY", "W_up", "W_gate", "W_down", "Up", "Gate", "Down", "Wr")}
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    out = dict(dW_up=f32(F, D), dW_gate=f32(F, D), dW_down=f32(D, F), dUp=f32(E, r, D), dGate=f32(E, r, D),
               dDown=f32(E, D, r), dWr=f32(E, D), dab=f32(2))
    pq.ffn_fwd(desc, t["X"], t["W_up"], t["W_gate"], t["W_down"], t["Up"], t["Gate"], t["Down"], t["Wr"], Y, bufs)
    pq.ffn_bwd(desc, t["dY"], t["X"], t["Up"], t["Gate"], t["Down"], t["Wr"], bufs, dX, out["dW_up"], out["dW_gate"],
               out["dW_down"], out["dUp"], out["dGate"], out["dDown"], out["dWr"], out["dab"])
    torch.cuda.synchronize()
    res = {k: v.cpu().numpy() for k, v in out.items()}
    res["Y"] = Y.float().cpu().numpy(); res["dX"] = dX.float().cpu().numpy()
    return res


def check_ffn(c, top_k=1, alpha=2.0, beta=0.2, experts="bf16"):
    got = run_ffn(c, top_k, alpha, beta, experts)
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], alpha, beta,
                   top_k=top_k, bf16=True, experts=experts)
    g = po.ffn_bwd(c["dY"], c["X"], c["Up"], c["Gate"], c["Down"], c["Wr"], alpha, beta, f)
    errs = report("Y", got["Y"], f["Y"])
    errs.update(report("dX", got["dX"], g["dX"]))
    for k in ("dW_up", "dW_gate", "dW_down"):
        errs.update(report(k, got[k], g[k], per_channel=True))
    for k in ("dUp", "dGate", "dDown", "dWr"):
        errs.update(report(k, got[k], g[k]))
    dY = c["dY"].astype(np.float64)
    sb = max(abs(g["dbeta"]), np.sqrt(((dY * f["Y1"]) ** 2).sum()), 1e-30)
    sa = max(abs(g["dalpha"]), np.sqrt(((dY * f["Yhp"]) ** 2).sum()), 1e-30)
    errs["dbeta"] = abs(got["dab"][1] - g["dbeta"]) / sb
    errs["dalpha"] = abs(got["dab"][0] - g["dalpha"]) / sa
    print("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    for k, v in errs.items():
        assert v <= TOL, f"{k}: {v} > {TOL}"


@pytest.mark.parametrize("T,D,F,E,r,k", [(200, 96, 160, 4, 8, 1), (200, 96, 160, 4, 8, 2), (700, 256, 544, 8, 32, 1),
                                         (130, 64, 64, 2, 16, 2), (1, 32, 32, 8, 8, 1),
                                         # hidden widths that are not whole packed words (like Table 1's 5076 = 158 * 32 + 20)
                                         (200, 96, 172, 4, 8, 1), (130, 64, 52, 2, 16, 2), (300, 256, 500, 1, 32, 1),
                                         # 1024 slots and more over ragged expert segments (one case with 64 experts, some of them empty)
                                         (1500, 128, 96, 4, 16, 2), (1100, 64, 64, 64, 8, 1), (1030, 192, 160, 3, 56, 1)])
def test_ffn_small(T, D, F, E, r, k):
    print(f"ffn T={T} d={D} F={F} E={E} r={r} k={k}", flush=True)
    check_ffn(wl.ffn_case(80 + T + k, T, D, F, E, r), top_k=k)


@pytest.mark.parametrize("T,D,F,E,r", [(300, 256, 544, 4, 32), (130, 256, 500, 2, 32)])
def test_ffn_stored_intermediates_at_code_level(T, D, F, E, r):
    """What pq_ffn_fwd stores for the backward, compared with the oracle piece by piece: the codes and gammas of x bit for
    bit; U and G to one bf16 rounding; the codes of the gated hidden state Hd = silu(G) U to one step (the kernel forms
    Hd in fp32 with the hardware exponential and reciprocal, the oracle in fp64, so a value next to a rounding boundary
    may land on the neighbouring code) on a small share of the entries, and its gammas to 1e-3; the padded columns of a
    width that is not a multiple of 32 hold zero codes."""
    print(f"ffn stored intermediates T={T} D={D} F={F} E={E} r={r}", flush=True)
    c = wl.ffn_case(2600 + F, T, D, F, E, r)
    desc = pq.FFNDesc(T, D, F, r, E, 1, pq.PQ_BF16, 2.0, 0.2, pq.PQ_HP_LOWRANK_BF16)
    bufs = pq.FFNBuffers(desc)
    t = {k: dev(c[k]) for k in ("X", "W_up", "W_gate", "W_down", "Up", "Gate", "Down", "Wr")}
    Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    pq.ffn_fwd(desc, t["X"], t["W_up"], t["W_gate"], t["W_down"], t["Up"], t["Gate"], t["Down"], t["Wr"], Y, bufs)
    torch.cuda.synchronize()
    f = po.ffn_fwd(c["X"], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2, top_k=1, bf16=True)
    Fp = (F + 31) // 32 * 32
    sec = lambda which: pq.ffn_ctx_section(desc, bufs, which)
    xq = sec(pq.FFN_CTX_XQ).view(torch.int8).view(T, D).cpu().numpy()
    gx = sec(pq.FFN_CTX_GAMMA_X).view(torch.float32).cpu().numpy()
    assert np.array_equal(xq, f["q"]) and np.array_equal(gx, f["gamma"])
    for name, which in (("U", pq.FFN_CTX_U), ("G", pq.FFN_CTX_G)):
        got = sec(which).view(torch.bfloat16).view(T, Fp)[:, :F].float().cpu().numpy().astype(np.float64)
        ref = np.asarray(f[name], np.float64)
        assert np.all(np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-30), name      # one bf16 rounding
        assert np.mean(got != ref) < 0.02, name
    hq = sec(pq.FFN_CTX_HQ).view(torch.int8).view(T, Fp).cpu().numpy().astype(np.int64)
    gh = sec(pq.FFN_CTX_GAMMA_H).view(torch.float32).cpu().numpy().astype(np.float64)
    assert np.all(hq[:, F:] == 0)
    d = np.abs(hq[:, :F] - f["qh"].astype(np.int64))
    share = float(np.mean(d != 0))
    print(f"  Hd codes: largest difference {d.max()}, share of entries that differ {share:.4f}", flush=True)
    assert d.max() <= 1 and share < 0.05
    assert np.abs(gh - f["gamma_h"].astype(np.float64)).max() <= 1e-3 * np.abs(f["gamma_h"]).max()


def test_ffn_scale_edge_cases():
    c = wl.ffn_case(90, 150, 64, 96, 4, 8)
    check_ffn(c, alpha=0.0, beta=0.7)
    check_ffn(c, alpha=1.5, beta=0.0)


def test_ffn_config3_reduced_tokens():
    print("ffn config 3 shape at T=384 (d=2048, F=5504, E=8, r=32, top-1)", flush=True)
    check_ffn(wl.config3(tokens=384), top_k=1)


@pytest.mark.parametrize("N", [1, 4])
def test_ffn_paper_1p3b_shape_reduced_tokens(N):
    """The paper's own 1.3B FFN (Table 1: D_model 2048, D_ff - r = 5076 one-bit hidden units, r = 384 per high-precision
    branch; Sec. 3.3 / Sec. 4.4: N branches, one active per token) at 384 tokens."""
    print(f"ffn paper-exact 1.3B shape, T=384, d=2048, F=5076, N={N} branches of r=384, top-1", flush=True)
    check_ffn(wl.ffn_case(700 + N, 384, 2048, 5076, N, 384), top_k=1)


@pytest.mark.parametrize("T,D,F,E,r,k", [(700, 256, 544, 8, 32, 1), (200, 96, 160, 4, 32, 2), (300, 256, 500, 1, 64, 1),
                                         (1, 32, 32, 8, 32, 1), (384, 2048, 5504, 8, 32, 1), (384, 2048, 5076, 4, 384, 1),
                                         # a single INT8 branch (the paper's default N = 1 in the form Sec. 3.2 prints): no routing
                                         (1100, 128, 96, 1, 32, 1), (384, 2048, 5076, 1, 384, 1)])
def test_ffn_int8_experts(T, D, F, E, r, k):
    """The experts in the INT8 form the FFN equation of Sec. 3.2 prints: weight rows and the expert's hidden state on the
    AbsMax grid, x's codes shared with the 1-bit branch, STE backward on the de-quantised factors.  The last two shapes
    are config 3 and the paper's 1.3B FFN (Table 1) at 384 tokens."""
    print(f"ffn int8 experts T={T} d={D} F={F} E={E} r={r} k={k}", flush=True)
    check_ffn(wl.ffn_case(180 + T + k + r, T, D, F, E, r), top_k=k, experts="int8")


def test_ffn_int8_experts_rejects_ranks_that_are_not_whole_words():
    with pytest.raises(pq.PQError):
        pq.FFNBuffers(pq.FFNDesc(64, 64, 64, 8, 2, 1, pq.PQ_BF16, 1.0, 1.0, pq.PQ_HP_LOWRANK_INT8))
    with pytest.raises(pq.PQError):
        pq.FFNBuffers(pq.FFNDesc(64, 64, 64, 32, 2, 1, pq.PQ_BF16, 1.0, 1.0, 7))


def test_ffn_config3_full_size_sampled_tokens():
    """Config 3 at its full size (T=8192) in the launch configuration the bench times.  Every step of the path is
    per token except the sums behind the weight gradients, so the oracle run on a sample of the tokens must
    reproduce the GPU's Y and dX rows of those tokens.  The weight, expert, router and scalar gradients sum over
    every token: they are compared with what oracle.ffn_bwd gave on the whole workload
    (tests/golden/full_size_config3.npz: sampled output channels of the three 1-bit weight gradients, sampled rows
    of the expert gradients, dWr whole, d alpha, d beta)."""
    print("ffn config 3, full size, 48 sampled tokens + stored full-size gradients", flush=True)
    c = wl.config3()
    got = run_ffn(c, 1, 2.0, 0.2)
    rows = np.random.default_rng(33).choice(c["tokens"], size=48, replace=False)
    rows.sort()
    f = po.ffn_fwd(c["X"][rows], c["W_up"], c["W_gate"], c["W_down"], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2,
                   top_k=1, bf16=True)
    g = po.ffn_bwd(c["dY"][rows], c["X"][rows], c["Up"], c["Gate"], c["Down"], c["Wr"], 2.0, 0.2, f)
    errs = report("Y", got["Y"][rows], f["Y"])
    errs.update(report("dX", got["dX"][rows], g["dX"]))
    ref = np.load(os.path.join(GOLDEN, "full_size_config3.npz"))
    chF, chD, rr = ref["chF"], ref["chD"], ref["rr"]
    errs.update(report("dW_up", got["dW_up"][chF], ref["dW_up"], per_channel=True))
    errs.update(report("dW_gate", got["dW_gate"][chF], ref["dW_gate"], per_channel=True))
    errs.update(report("dW_down", got["dW_down"][chD], ref["dW_down"], per_channel=True))
    errs.update(report("dUp", got["dUp"][:, rr], ref["dUp"]))
    errs.update(report("dGate", got["dGate"][:, rr], ref["dGate"]))
    errs.update(report("dDown", got["dDown"][:, chD], ref["dDown"]))
    errs.update(report("dWr", got["dWr"], ref["dWr"]))
    errs["dalpha"] = abs(got["dab"][0] - float(ref["dalpha"])) / max(abs(float(ref["dalpha"])), float(ref["dalpha_scale"]))
    errs["dbeta"] = abs(got["dab"][1] - float(ref["dbeta"])) / max(abs(float(ref["dbeta"])), float(ref["dbeta_scale"]))
    print("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    for k, v in errs.items():
        assert v <= TOL, f"{k}: {v} > {TOL}"
