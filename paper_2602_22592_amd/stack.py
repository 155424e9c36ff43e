"""A stack of transformer-shaped layers made of pQuant linears only (no attention core, no norms):

    per layer:  q,k,v = L_q(h), L_k(h), L_v(h)      pure 1-bit linears (Sec. 3.1: the MHA projections)
                m = (q + k + v) / 3                 stand-in for the attention core (glue)
                h1 = h + L_o(m)                     residual (glue)
                h2 = h1 + FFN(h1)                   decoupled FFN with routed experts (Sec. 3.2, 3.3)

This module only sequences C-ABI calls (pq_linear_*, pq_ffn_*, pq_glue_*); PyTorch provides the
device buffers.  It exists to time the linears of a 24-layer 1.3B-shaped model end to end.
"""
from __future__ import annotations

import torch

from . import binding as pq


class Stack:
    def __init__(self, n_layers, tokens, d_model, d_ffn, n_experts, hp_rank, top_k, alphas, betas, device="cuda"):
        self.L, self.T, self.D, self.F = n_layers, tokens, d_model, d_ffn
        self.E, self.r, self.k = n_experts, hp_rank, top_k
        bf = torch.bfloat16
        self.lin_desc = pq.make_desc(tokens, d_model, d_model, hp_rank=0, io_dtype=pq.PQ_BF16, alpha=0.0, beta=1.0)
        self.layers = []
        lin_ws = ffn_ws = None                       # one scratch buffer per kind, shared by all layers
        for l in range(n_layers):
            ffn_desc = pq.FFNDesc(tokens, d_model, d_ffn, hp_rank, n_experts, top_k, pq.PQ_BF16, alphas[l], betas[l])
            buf = {}
            for n in ("q", "k", "v", "o"):
                buf[n] = pq.LinearBuffers(self.lin_desc, device, ws=lin_ws)
                lin_ws = buf[n].ws
            fb = pq.FFNBuffers(ffn_desc, device, ws=ffn_ws)
            ffn_ws = fb.ws
            st = {n: torch.empty((tokens, d_model), dtype=bf, device=device) for n in ("h", "m", "h1")}
            self.layers.append(dict(ffn_desc=ffn_desc, ffn_buf=fb, lin_buf=buf, **st))
        e = lambda: torch.empty((tokens, d_model), dtype=bf, device=device)
        self.t = [e() for _ in range(5)]              # scratch activations
        self.out = e()
        self.dh = [e(), e()]
        self.dab = torch.empty((2,), dtype=torch.float32, device=device)

    def forward(self, h0, weights):
        h = h0
        q, k, v, o, f = self.t
        for l, (ly, w) in enumerate(zip(self.layers, weights)):
            ly["h"].copy_(h)
            for n, y in (("q", q), ("k", k), ("v", v)):
                pq.linear_fwd(self.lin_desc, ly["h"], w["W" + n], y, ly["lin_buf"][n])
            pq.glue_lincomb(ly["m"], [q, k, v], [1 / 3, 1 / 3, 1 / 3])
            pq.linear_fwd(self.lin_desc, ly["m"], w["Wo"], o, ly["lin_buf"]["o"])
            pq.glue_lincomb(ly["h1"], [ly["h"], o], [1.0, 1.0])
            pq.ffn_fwd(ly["ffn_desc"], ly["h1"], w["W_up"], w["W_gate"], w["W_down"], w["Up"], w["Gate"], w["Down"], w["Wr"],
                       f, ly["ffn_buf"])
            pq.glue_lincomb(self.out, [ly["h1"], f], [1.0, 1.0])
            h = self.out
        return self.out

    def backward(self, dY, weights, grads):
        """grads: per-layer dict of fp32 tensors shaped like the weights (plus 'dab' [2])."""
        d_cur, d_tmp = self.dh
        d_cur.copy_(dY)
        dq, dk, dv, dm, dx = self.t
        for l in reversed(range(self.L)):
            ly, w, g = self.layers[l], weights[l], grads[l]
            # h2 = h1 + FFN(h1)
            pq.ffn_bwd(ly["ffn_desc"], d_cur, ly["h1"], w["Up"], w["Gate"], w["Down"], w["Wr"], ly["ffn_buf"], dx, g["W_up"],
                       g["W_gate"], g["W_down"], g["Up"], g["Gate"], g["Down"], g["Wr"], g["dab"])
            pq.glue_lincomb(d_tmp, [d_cur, dx], [1.0, 1.0])            # d h1
            # h1 = h + L_o(m)
            pq.linear_bwd(self.lin_desc, d_tmp, ly["m"], w["Wo"], ly["lin_buf"]["o"], dm, g["Wo"], self.dab)
            pq.glue_lincomb(dm, [dm], [1 / 3])                         # d q = d k = d v = d m / 3
            for n, dxn in (("q", dq), ("k", dk), ("v", dv)):
                pq.linear_bwd(self.lin_desc, dm, ly["h"], w["W" + n], ly["lin_buf"][n], dxn, g["W" + n], self.dab)
            pq.glue_lincomb(d_cur, [d_tmp, dq, dk, dv], [1.0, 1.0, 1.0, 1.0])
        return d_cur
