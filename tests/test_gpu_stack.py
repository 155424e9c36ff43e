"""The layer stack (q,k,v,o pure 1-bit linears + decoupled FFN per layer) chained on the GPU against
the same chain of oracle calls, at 2 layers and T=256 (bf16; 2e-2 max-norm relative), and at the full
per-layer shape of the 24-layer run against sampled tokens and stored full-size weight gradients."""
import os

import numpy as np
import pytest
import torch

from oracle import pquant_oracle as po
from paper_2602_22592_amd import binding as pq
from paper_2602_22592_amd import workloads as wl
from paper_2602_22592_amd.stack import Stack
from parity_metrics import relerr, report

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda().to(torch.bfloat16)


@pytest.mark.parametrize("L,T,D,F,E,r", [(2, 256, 128, 352, 8, 32), (3, 100, 64, 96, 4, 8)])
def test_stack_two_layers(L, T, D, F, E, r):
    print(f"stack L={L} T={T} d={D} F={F} E={E} r={r}", flush=True)
    c = wl.stack_case(7, L, T, D, F, E, r, vocab=1000)
    names = ("Wq", "Wk", "Wv", "Wo", "W_up", "W_gate", "W_down", "Up", "Gate", "Down", "Wr")
    weights = [{n: dev(w[n]) for n in names} for w in c["layers"]]
    grads = [dict({n: torch.empty(w[n].shape, dtype=torch.float32, device="cuda") for n in names},
                  dab=torch.empty(2, dtype=torch.float32, device="cuda")) for w in c["layers"]]
    st = Stack(L, T, D, F, E, r, 1, [w["alpha"] for w in c["layers"]], [w["beta"] for w in c["layers"]])
    h0 = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    pq.glue_gather_rows(dev(c["table"]), torch.from_numpy(c["ids"]).cuda(), h0)
    out = st.forward(h0, weights)
    d0 = st.backward(dev(c["dY"]), weights, grads)
    torch.cuda.synchronize()

    h0_ref = c["table"][c["ids"]]
    assert np.array_equal(h0.float().cpu().numpy(), h0_ref)
    y_ref, saved = po.stack_fwd(h0_ref, c["layers"], top_k=1)
    d_ref, g_ref = po.stack_bwd(c["dY"], c["layers"], saved)
    errs = {"out": relerr(out.float().cpu().numpy(), y_ref), "dh0": relerr(d0.float().cpu().numpy(), d_ref)}
    for l in (0, L - 1):
        for n in ("Wq", "Wo", "W_up", "W_down", "Up", "Down", "Wr"):
            errs[f"{n}[{l}]"] = relerr(grads[l][n].cpu().numpy(), g_ref[l][n])
    print("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    # A routing decision of a later layer can flip on a near-tie once bf16-level differences have propagated into its
    # router's input; the bar below holds when the decisions agree.  Name the tokens whose top-2 logit gap in the
    # oracle is below what such differences can move (1e-2 of the logit scale): a failure with such tokens present
    # is a routing flip, not an arithmetic error.
    for l in range(L):
        lg = np.sort(saved[l]["ff"]["logits"].astype(np.float64), axis=1)
        gap = lg[:, -1] - lg[:, -2]
        near = np.nonzero(gap < 1e-2 * max(np.abs(lg).max(), 1e-30))[0]
        print(f"  layer {l}: tokens with a near-tie between their two best experts: {near.tolist()}", flush=True)
    assert max(errs.values()) <= 2e-2, errs


def test_stack_config5_layer_shape_sampled_tokens():
    """Two layers at the bench's per-layer shape (T=16384, d=2048, d_ffn=5504, E=8 x r=32, top-1), i.e. the launch
    configuration of every kernel of the 24-layer run.  A token's path through the stack does not depend on the
    other tokens (the weight statistics depend on the weights only), so the oracle runs the same chain on sampled
    tokens alone: forward output and input gradient of those tokens."""
    L, T, D, F, E, r = 2, 16384, 2048, 5504, 8, 32
    print(f"stack full layer shape L={L} T={T} d={D} F={F} E={E} r={r}, sampled tokens", flush=True)
    c = wl.stack_case(11, L, T, D, F, E, r, vocab=4096)
    names = ("Wq", "Wk", "Wv", "Wo", "W_up", "W_gate", "W_down", "Up", "Gate", "Down", "Wr")
    weights = [{n: dev(w[n]) for n in names} for w in c["layers"]]
    grads = [dict({n: torch.empty(w[n].shape, dtype=torch.float32, device="cuda") for n in names},
                  dab=torch.empty(2, dtype=torch.float32, device="cuda")) for w in c["layers"]]
    st = Stack(L, T, D, F, E, r, 1, [w["alpha"] for w in c["layers"]], [w["beta"] for w in c["layers"]])
    h0 = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    pq.glue_gather_rows(dev(c["table"]), torch.from_numpy(c["ids"]).cuda(), h0)
    out = st.forward(h0, weights)
    d0 = st.backward(dev(c["dY"]), weights, grads)
    torch.cuda.synchronize()

    tok = np.sort(np.random.default_rng(3).choice(T, 24, replace=False))
    tok[0], tok[-1] = 0, T - 1
    h0_ref = c["table"][c["ids"][tok]]
    assert np.array_equal(h0[torch.from_numpy(tok).cuda()].float().cpu().numpy(), h0_ref)
    y_ref, saved = po.stack_fwd(h0_ref, c["layers"], top_k=1)
    d_ref, _ = po.stack_bwd(c["dY"][tok], c["layers"], saved)
    tk = torch.from_numpy(tok).cuda()
    errs = {"out": relerr(out[tk].float().cpu().numpy(), y_ref), "dh0": relerr(d0[tk].float().cpu().numpy(), d_ref)}
    print("  errors: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert max(errs.values()) <= 2e-2, errs
    # Weight gradients of the two-layer chain against the oracle's full-size run (tests/golden/full_size_stack.npz).  The
    # single-layer bar does not carry over to a chain: the second layer's quantisers see inputs that already differ at the
    # level of one bf16 rounding, which moves a share of its INT8 codes by one step (1/128 .. 1/1 of a code's value) and,
    # for a handful of tokens with two nearly equal router logits, the selected expert; both sides are valid evaluations
    # of the same chain.  The figures are printed; the assertion is a sanity bound on the 1-bit weight gradients (the bar of
    # a single layer at this shape is test_stack_config5_single_layer_weight_gradients below).
    ref = np.load(os.path.join(GOLDEN, "full_size_stack.npz"))
    ch = ref["ch"]
    chain = {}
    chain.update(report("dWq[0]", grads[0]["Wq"].cpu().numpy()[ch], ref["Wq0"], per_channel=True))
    chain.update(report("dWo[1]", grads[L - 1]["Wo"].cpu().numpy()[ch], ref["Wo1"], per_channel=True))
    chain.update(report("dW_down[1]", grads[L - 1]["W_down"].cpu().numpy()[ch], ref["W_down1"], per_channel=True))
    chain.update(report("dWr[0]", grads[0]["Wr"].cpu().numpy(), ref["Wr0"]))
    chain.update(report("dWr[1]", grads[L - 1]["Wr"].cpu().numpy(), ref["Wr1"]))
    print("  two-layer chain, weight gradients: " + ", ".join(f"{k}={v:.2e}" for k, v in chain.items()), flush=True)
    print(f"  tokens of the last layer whose two best router logits are closer than 1e-3: {int((ref['gap1'] < 1e-3).sum())} of {T}",
          flush=True)
    for k in ("dWq[0].l2", "dWo[1].l2", "dW_down[1].l2"):
        assert chain[k] <= 1e-1, (k, chain[k])


def test_stack_config5_single_layer_weight_gradients():
    """One layer at the bench's per-layer shape (T=16384: the launch configuration, split plans included, of every kernel
    of the 24-layer run).  Forward output and input gradient of sampled tokens against the oracle run on those tokens,
    and the weight gradients (sums over all 16384 tokens) against the oracle's full-size run stored in
    tests/golden/full_size_stack1.npz.  The bar of a single linear (2e-2 in every measure) is asserted for the gradients
    whose operands reach both sides through at most one quantised linear (the attention projections, W_up, W_gate).
    The FFN's second half sits behind two more quantisers and the router: W_down keeps the bar in the max-norm and L2
    measures (its per-channel figure is printed: channels whose hidden codes are 0 or +/-1 move by whole steps), and the
    expert and router gradients are bounded at 1e-1 in L2: a token whose two best logits nearly tie may go to the other
    expert on either side, which moves its whole contribution between two experts' sums (the exact-input comparison of
    these gradients at full size is tests/test_gpu_ffn.py::test_ffn_config3_full_size_sampled_tokens)."""
    L, T, D, F, E, r = 1, 16384, 2048, 5504, 8, 32
    print(f"stack single layer, full shape T={T} d={D} F={F} E={E} r={r}", flush=True)
    c = wl.stack_case(12, L, T, D, F, E, r, vocab=4096)
    names = ("Wq", "Wk", "Wv", "Wo", "W_up", "W_gate", "W_down", "Up", "Gate", "Down", "Wr")
    weights = [{n: dev(w[n]) for n in names} for w in c["layers"]]
    grads = [dict({n: torch.empty(w[n].shape, dtype=torch.float32, device="cuda") for n in names},
                  dab=torch.empty(2, dtype=torch.float32, device="cuda")) for w in c["layers"]]
    st = Stack(L, T, D, F, E, r, 1, [w["alpha"] for w in c["layers"]], [w["beta"] for w in c["layers"]])
    h0 = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    pq.glue_gather_rows(dev(c["table"]), torch.from_numpy(c["ids"]).cuda(), h0)
    out = st.forward(h0, weights)
    d0 = st.backward(dev(c["dY"]), weights, grads)
    torch.cuda.synchronize()
    tok = np.sort(np.random.default_rng(4).choice(T, 24, replace=False))
    y_ref, saved = po.stack_fwd(c["table"][c["ids"][tok]], c["layers"], top_k=1)
    d_ref, _ = po.stack_bwd(c["dY"][tok], c["layers"], saved)
    tk = torch.from_numpy(tok).cuda()
    strict = {"out": relerr(out[tk].float().cpu().numpy(), y_ref), "dh0": relerr(d0[tk].float().cpu().numpy(), d_ref)}
    ref = np.load(os.path.join(GOLDEN, "full_size_stack1.npz"))
    ch, chF = ref["ch"], ref["chF"]
    g = {n: grads[0][n].cpu().numpy() for n in names}
    for n in ("Wq", "Wk", "Wo"):
        strict.update(report("d" + n, g[n][ch], ref[n], per_channel=True))
    for n in ("W_up", "W_gate"):
        strict.update(report("d" + n, g[n][chF], ref[n], per_channel=True))
    down = report("dW_down", g["W_down"][ch], ref["W_down"], per_channel=True)
    loose = {}
    loose.update(report("dWr", g["Wr"], ref["Wr"]))
    loose.update(report("dUp", g["Up"][:, :8], ref["Up"]))
    loose.update(report("dDown", g["Down"][:, ch], ref["Down"]))
    for name, errs in (("2e-2 bar", strict), ("W_down", down), ("experts and router", loose)):
        print(f"  {name}: " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert max(strict.values()) <= 2e-2, strict
    assert down["dW_down"] <= 2e-2 and down["dW_down.l2"] <= 2e-2, down
    for k in ("dWr.l2", "dUp.l2", "dDown.l2"):
        assert loose[k] <= 1e-1, (k, loose[k])
