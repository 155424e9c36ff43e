"""CPU oracle for the pQuant decoupled linear layer.  TEST INFRASTRUCTURE ONLY.

A plain, slow, NumPy transcription of the paper's definitions: fp64 arithmetic everywhere a value
is accumulated, one rounding to fp32 where a value is later compared or thresholded (mu, gamma, the
quantiser product, router logits).  It shares no code with the HIP library and never calls it; only
tests, the smoke check and the bench's cpu_baseline leg may import it.  The product path must not.

Notation follows the paper: W latent weight [m=d_out, n=d_in] (Y = W X), mu/lambda the weight
statistics (Sec. 3.1, eq. for mu and lambda), gamma the per-token AbsMax scale, Q(.) the INT8
quantiser (Sec. 3.1), alpha/beta the feature scales (Sec. 3.2, FFN equation), N experts with a
linear softmax router and top-k selection (Sec. 3.3).

Pins (tests/test_oracle_*.py) cover every function below; none is "parity unpinned".

Readings taken where the paper is silent or garbled (each also listed in the design notes):
  * Sign(0): W >= mu maps to +1 (a two-valued code needs a choice).
  * lambda is the mean of |W| on the raw (un-centred) weights, as printed.
  * RoundClip bounds: gamma = 128/absmax, round half to even, clamp to [-128, 127].
  * one gamma per token (row of X); a zero row uses max(absmax, 1e-5).
  * the high-precision branch reads the raw X (not Q(X)) and keeps 16-bit weights (Sec. 4.6 FP16 variant);
    its INT8 form (Sec. 3.2) quantises the rows of both factors and the hidden state like activations.
  * router: logits on raw X, top-k on logits (ties -> lower index), gates = softmax over all experts,
    not renormalised.
  * STE: identity through Sign and Q; mu, lambda, gamma carry no gradient.
  * group-wise weight scales (Sec. 4.6 ablation, contrast only): groups of 64 consecutive input columns of an output row,
    one scale per group = mean |W| of the group, held in 16 bits (fp16, rounded from its fp32 value); mu and the signs are
    those of the per-tensor form.
  * the normalisation in front of the quantiser is RMSNorm with a per-channel gain g and an eps inside the
    square root (App. B names RMSNorm, Sec. 3.1 prints LayerNorm; neither gives gain or eps).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
F64 = np.float64


# ----------------------------------------------------------------------------------------------
# Sec. 3.1: weight statistics, binarisation, packing (App. A: offline packing)
# ----------------------------------------------------------------------------------------------
def weight_stats(W):
    """mu = mean(W), lambda = mean(|W|) over the whole matrix (Sec. 3.1, eq. mu/lambda); fp64 sums,
    one rounding to fp32."""
    W64 = np.asarray(W, dtype=F64)
    n = W64.size
    mu = F32(W64.sum() / n)
    lam = F32(np.abs(W64).sum() / n)
    return mu, lam


def binarise(W, mu):
    """W^INT1 = Sign(W - mu) (Sec. 3.1); the compare is done in fp32 without forming W - mu."""
    W32 = np.asarray(W, dtype=F32)
    return np.where(W32 >= F32(mu), np.int8(1), np.int8(-1)).astype(np.int8)


def pack_sign(S):
    """Pack +/-1 into uint32 words along d_in, bit j of word w <-> column 32 w + j, bit 1 <-> +1
    (App. A: packed 1-bit storage; the paper packs 8 per byte, which is the same byte stream).
    A row whose length is not a multiple of 32 (Table 1: D_ff - r = 5076 for the 1.3B model) is padded to whole
    words with +1 bits (a reading: the paper does not say how partial words are filled): a padded column only
    ever meets an activation code of zero, so the pad value cannot reach an accumulator."""
    S = np.asarray(S)
    m, n = S.shape
    npad = (-n) % 32
    bits = np.concatenate([(S > 0), np.ones((m, npad), bool)], axis=1) if npad else (S > 0)
    bits = bits.reshape(m, (n + npad) // 32, 32).astype(np.uint64)
    place = np.uint64(1) << np.arange(32, dtype=np.uint64)
    return (bits * place).sum(axis=2).astype(np.uint32)


def unpack_sign(P, n):
    P = np.asarray(P, dtype=np.uint32)
    m = P.shape[0]
    j = np.arange(32, dtype=np.uint32)
    bits = (P[:, :, None] >> j) & np.uint32(1)
    return np.where(bits.reshape(m, -1)[:, :n] == 1, np.int8(1), np.int8(-1)).astype(np.int8)


def ste_mask(W, mu, tau):
    """Optional weight-gradient clipping mask 1[|W - mu| <= tau]; tau = inf is the paper's plain STE."""
    W64 = np.asarray(W, dtype=F64)
    return (np.abs(W64 - F64(mu)) <= F64(tau))


# ----------------------------------------------------------------------------------------------
# Sec. 3.1: AbsMax INT8 activation quantiser
# ----------------------------------------------------------------------------------------------
def quant_act(X):
    """Q(X) = RoundClip(X * gamma), gamma = 2^7 / max_k |x_k| per token (Sec. 3.1). fp32 throughout:
    IEEE division, one fp32 product, round half to even, clamp to [-128, 127]."""
    X32 = np.asarray(X, dtype=F32)
    a = np.max(np.abs(X32), axis=1) if X32.shape[1] else np.zeros(X32.shape[0], F32)
    gamma = (F32(128.0) / np.maximum(a, F32(1e-5))).astype(F32)
    y = (X32 * gamma[:, None]).astype(F32)
    q = np.clip(np.rint(y), -128, 127).astype(np.int8)
    return q, gamma


def onebit_acc(q, S):
    """Integer accumulator acc[t, i] = sum_j q[t, j] * S[i, j] (the W1A8 product of Sec. 3.1)."""
    return np.asarray(q, dtype=np.int64) @ np.asarray(S, dtype=np.int64).T


# ----------------------------------------------------------------------------------------------
# Sec. 3.3: router
# ----------------------------------------------------------------------------------------------
def router_topk(X, Wr, k):
    """Linear router + softmax gate + top-k (Sec. 3.3).  logits are fp64 dot products rounded once to
    fp32; selection is on the logits, descending, ties to the lower expert index."""
    X64 = np.asarray(X, dtype=F64)
    Wr64 = np.asarray(Wr, dtype=F64)
    logits = (X64 @ Wr64.T).astype(F32)
    l64 = logits.astype(F64)
    z = l64 - l64.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    idx = np.argsort(-l64, axis=1, kind="stable")[:, :k].astype(np.int32)
    gate = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    return idx, gate, p, logits


def _router_bwd(dgate, idx, p, X64, Wr64):
    """Gradient of gate[t,j] = softmax(logits)[t, idx[t,j]] w.r.t. logits, then Wr and X."""
    T, E = p.shape
    dlogit = np.zeros((T, E), F64)
    for j in range(idx.shape[1]):
        pj = np.take_along_axis(p, idx[:, j:j + 1].astype(np.int64), axis=1)[:, 0]
        onehot = np.zeros((T, E), F64)
        onehot[np.arange(T), idx[:, j]] = 1.0
        dlogit += (dgate[:, j] * pj)[:, None] * (onehot - p)
    return dlogit.T @ X64, dlogit @ Wr64, dlogit


# ----------------------------------------------------------------------------------------------
# Sec. 3.1-3.3: the decoupled linear layer, forward
# ----------------------------------------------------------------------------------------------
def linear_fwd(X, W, alpha, beta, A=None, B=None, Wr=None, top_k=1, packed=None, mu_lambda=None,
               scale_fp16=False):
    """Y = beta * (lambda/gamma) W^INT1 Q(X)  +  alpha * HP(X)   (Sec. 3.1 last eq.; Sec. 3.2 FFN eq.)

    HP is absent (A is None: the pure 1-bit linear of the attention projections), a single
    two-factor branch B (A x), or E routed low-rank experts B_e (A_e x) weighted by their gates.
    With `packed` given the weight side is read back from packed bits and `mu_lambda` (inference).
    `scale_fp16` rounds beta*lambda to fp16 once (the stored inference scale).
    """
    X32 = np.asarray(X, dtype=F32)
    X64 = X32.astype(F64)
    T, n = X32.shape
    if packed is None:
        mu, lam = weight_stats(W)
        S = binarise(W, mu)
        P = pack_sign(S)
    else:
        mu, lam = F32(mu_lambda[0]), F32(mu_lambda[1])
        P = np.asarray(packed, dtype=np.uint32)
        S = unpack_sign(P, n)
    q, gamma = quant_act(X32)
    acc = onebit_acc(q, S)
    assert np.all(np.abs(acc) < 2 ** 24)
    bl = F32(F32(beta) * lam)
    if scale_fp16:
        bl = F32(np.float16(bl))
    s = (bl / gamma).astype(F32)
    Y1 = (s[:, None] * acc.astype(F32)).astype(F32)               # beta already inside
    Y1_nobeta = (F64(lam) / gamma.astype(F64))[:, None] * acc       # for d beta
    out = dict(mu=mu, lam=lam, S=S, P=P, q=q, gamma=gamma, acc=acc, Y1=Y1, Y1_nobeta=Y1_nobeta)

    m = S.shape[0]
    Yhp = np.zeros((T, m), F64)
    if A is not None:
        A64 = np.asarray(A, dtype=F64)
        B64 = np.asarray(B, dtype=F64)
        if A64.ndim == 2:                                           # one dense branch
            H = X64 @ A64.T
            Yhp = H @ B64.T
            out["H"] = H
        else:                                                       # routed experts
            idx, gate, p, logits = router_topk(X32, Wr, top_k)
            E = A64.shape[0]
            Hs = np.zeros((T, top_k, A64.shape[1]), F64)
            Ys = np.zeros((T, top_k, m), F64)
            for j in range(top_k):
                for e in range(E):
                    sel = np.nonzero(idx[:, j] == e)[0]
                    if sel.size:
                        h = X64[sel] @ A64[e].T
                        Hs[sel, j] = h
                        Ys[sel, j] = h @ B64[e].T
            Yhp = (gate[:, :, None] * Ys).sum(axis=1)
            out.update(idx=idx, gate=gate, probs=p, logits=logits, Hs=Hs, Ys=Ys)
    out["Yhp"] = Yhp
    out["Y"] = Y1.astype(F64) + F64(alpha) * Yhp
    return out


# ----------------------------------------------------------------------------------------------
# STE backward (Sec. 4 intro; App. B.1)
# ----------------------------------------------------------------------------------------------
def linear_bwd(dY, X, W, alpha, beta, fwd, A=None, B=None, Wr=None, ste_tau=np.inf):
    """Gradients of the decoupled linear with the straight-through estimator: the quantised
    activation q/gamma and the binarised weight lambda*S are treated as if they were X and W."""
    dY64 = np.asarray(dY, dtype=F64)
    X64 = np.asarray(X, dtype=F64)
    S64 = fwd["S"].astype(F64)
    q64 = fwd["q"].astype(F64)
    g64 = fwd["gamma"].astype(F64)
    lam = F64(fwd["lam"])
    al, be = F64(alpha), F64(beta)

    g = dict()
    g["dbeta"] = float((dY64 * fwd["Y1_nobeta"]).sum())
    g["dalpha"] = float((dY64 * fwd["Yhp"]).sum())
    dX = be * lam * (dY64 @ S64)
    dW = be * ((dY64 / g64[:, None]).T @ q64)
    if np.isfinite(ste_tau):
        dW = dW * ste_mask(W, fwd["mu"], ste_tau)
    g["dW"] = dW

    if A is not None:
        A64 = np.asarray(A, dtype=F64)
        B64 = np.asarray(B, dtype=F64)
        G = al * dY64
        if A64.ndim == 2:
            H = fwd["H"]
            dH = G @ B64
            g["dB"] = G.T @ H
            g["dA"] = dH.T @ X64
            dX = dX + dH @ A64
        else:
            idx, gate, p = fwd["idx"], fwd["gate"], fwd["probs"]
            E = A64.shape[0]
            dA = np.zeros_like(A64)
            dB = np.zeros_like(B64)
            dgate = np.einsum("ti,tji->tj", G, fwd["Ys"])
            for j in range(idx.shape[1]):
                for e in range(E):
                    sel = np.nonzero(idx[:, j] == e)[0]
                    if not sel.size:
                        continue
                    dy = gate[sel, j][:, None] * G[sel]
                    dB[e] += dy.T @ fwd["Hs"][sel, j]
                    dh = dy @ B64[e]
                    dA[e] += dh.T @ X64[sel]
                    dX[sel] += dh @ A64[e]
            dWr, dX_r, dlogit = _router_bwd(dgate, idx, p, X64, np.asarray(Wr, dtype=F64))
            dX = dX + dX_r
            g.update(dA=dA, dB=dB, dWr=dWr, dgate=dgate, dlogit=dlogit)
    g["dX"] = dX
    return g


# ----------------------------------------------------------------------------------------------
# Sec. 3.2 / 3.3: the decoupled FFN (1-bit up/gate/down + routed high-precision FFN experts)
# ----------------------------------------------------------------------------------------------
def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def _silu(x):
    return x * _sigmoid(x)


def _dsilu(x):
    s = _sigmoid(x)
    return s * (1.0 + x * (1.0 - s))


def _round_io(x, bf16):
    """Round to the storage format of saved activations (bf16 via the library cast, else fp32)."""
    if not bf16:
        return np.asarray(x, dtype=F32)
    import torch
    return torch.from_numpy(np.asarray(x, dtype=F32)).to(torch.bfloat16).to(torch.float32).numpy()


def ffn_fwd(X, W_up, W_gate, W_down, Up, Gate, Down, Wr, alpha, beta, top_k=1, bf16=True, experts="bf16"):
    """Y = alpha * sum_j gate_j FFN_e_j(X) + beta * FFN^INT1(X)   (Sec. 3.2 FFN equation, Sec. 3.3).

    FFN^INT1: three pure 1-bit linears around a gated unit, hidden state re-quantised before the
    down projection:  U = L_up(Q(X)), G = L_gate(Q(X)), Hd = silu(G) * U, Y1 = L_down(Q(Hd)).
    U and G are rounded to the storage format (they are saved for the backward pass); Hd is formed
    from the rounded values and quantised from fp32 (a reading: the paper states no storage precision; FP16
    latent activations are what its mixed-precision training keeps, App. B).  Experts are gated FFNs of hidden width r.

    experts="int8" is the form the FFN equation of Sec. 3.2 prints (FFN^INT8): "8-bit weights are quantized identically
    to 8-bit activations", read as the AbsMax quantiser of Sec. 3.1 per output channel, i.e. per row of Up_e, Gate_e
    [r, d] and of Down_e [d, r]; the expert reads the codes and gamma of x that the 1-bit branch has formed (x is
    quantised once); its hidden state a = silu(g) * u is stored in the I/O type and quantised again per token (an
    8-bit activation like any other); u, g and the expert's output are exact integer accumulations de-quantised in the
    order of _dequant_scale, u and g stored in the I/O type.
    """
    X32 = np.asarray(X, dtype=F32)
    X64 = X32.astype(F64)
    T, d = X32.shape
    q, gamma = quant_act(X32)
    st = {}
    for name, Wm in (("up", W_up), ("gate", W_gate), ("down", W_down)):
        mu, lam = weight_stats(Wm)
        st[name] = dict(mu=mu, lam=lam, S=binarise(Wm, mu))
    U = ((st["up"]["lam"] / gamma).astype(F32)[:, None] * onebit_acc(q, st["up"]["S"]).astype(F32)).astype(F32)
    G = ((st["gate"]["lam"] / gamma).astype(F32)[:, None] * onebit_acc(q, st["gate"]["S"]).astype(F32)).astype(F32)
    U = _round_io(U, bf16)
    G = _round_io(G, bf16)
    Hd = (_silu(G.astype(F64)) * U.astype(F64)).astype(F32)
    qh, gamma_h = quant_act(Hd)
    acc_d = onebit_acc(qh, st["down"]["S"])
    Y1 = (F64(st["down"]["lam"]) / gamma_h.astype(F64))[:, None] * acc_d     # before beta

    idx, gate, p, logits = router_topk(X32, Wr, top_k)
    E, r, _ = np.asarray(Up).shape
    Up64, Gate64, Down64 = (np.asarray(a, dtype=F64) for a in (Up, Gate, Down))
    ue = np.zeros((T, top_k, r), F64)
    ge = np.zeros((T, top_k, r), F64)
    Ys = np.zeros((T, top_k, d), F64)
    ex8 = None
    if experts == "int8":
        qw = {n: [quant_act(np.asarray(W[e], dtype=F32)) for e in range(E)] for n, W in (("up", Up), ("gate", Gate), ("down", Down))}
        qa = np.zeros((T, top_k, r), np.int8)
        ga = np.zeros((T, top_k), F32)
        a_st = np.zeros((T, top_k, r), F32)
    for j in range(top_k):
        for e in range(E):
            sel = np.nonzero(idx[:, j] == e)[0]
            if not sel.size:
                continue
            if experts == "int8":
                (q_u, g_u), (q_g, g_g), (q_d, g_d) = qw["up"][e], qw["gate"][e], qw["down"][e]
                qx = q[sel].astype(np.int64)
                u = _round_io(_dequant_scale(qx @ q_u.astype(np.int64).T, gamma[sel], g_u), bf16)
                g_ = _round_io(_dequant_scale(qx @ q_g.astype(np.int64).T, gamma[sel], g_g), bf16)
                a = _round_io((_silu(g_.astype(F64)) * u.astype(F64)).astype(F32), bf16)
                q_a, g_a = quant_act(a)
                ue[sel, j], ge[sel, j] = u, g_
                a_st[sel, j], qa[sel, j], ga[sel, j] = a, q_a, g_a
                Ys[sel, j] = _dequant_scale(q_a.astype(np.int64) @ q_d.astype(np.int64).T, g_a, g_d)
            else:
                ue[sel, j] = X64[sel] @ Up64[e].T
                ge[sel, j] = X64[sel] @ Gate64[e].T
                Ys[sel, j] = (_silu(ge[sel, j]) * ue[sel, j]) @ Down64[e].T
    if experts == "int8":
        ex8 = dict(qw=qw, a=a_st, qa=qa, ga=ga)
    Yhp = (gate[:, :, None] * Ys).sum(axis=1)
    Y = F64(beta) * Y1 + F64(alpha) * Yhp
    return dict(Y=Y, Y1=Y1, Yhp=Yhp, q=q, gamma=gamma, U=U, G=G, Hd=Hd, qh=qh, gamma_h=gamma_h,
                st=st, idx=idx, gate=gate, probs=p, logits=logits, ue=ue, ge=ge, Ys=Ys, acc_d=acc_d, ex8=ex8)


def ffn_bwd(dY, X, Up, Gate, Down, Wr, alpha, beta, fwd):
    """STE backward of ffn_fwd: identity through every quantiser, rounding and Sign.  For INT8 experts (fwd["ex8"]) that
    means (App. B.1) every product is differentiated with the de-quantised factors it multiplied: X~ = q_x / gamma_x,
    Up~, Gate~, Down~ (rows over their gammas) and the hidden state a~ = q_a / gamma_a; the gated unit is differentiated
    at the stored u and g.  The router still reads and is differentiated at the unquantised x."""
    dY64 = np.asarray(dY, dtype=F64)
    X64 = np.asarray(X, dtype=F64)
    al, be = F64(alpha), F64(beta)
    st = fwd["st"]
    g = dict(dbeta=float((dY64 * fwd["Y1"]).sum()), dalpha=float((dY64 * fwd["Yhp"]).sum()))

    dY1 = be * dY64
    Sd = st["down"]["S"].astype(F64)
    dHd = F64(st["down"]["lam"]) * (dY1 @ Sd)
    g["dW_down"] = (dY1 / fwd["gamma_h"].astype(F64)[:, None]).T @ fwd["qh"].astype(F64)
    U64, G64 = fwd["U"].astype(F64), fwd["G"].astype(F64)
    dU = dHd * _silu(G64)
    dG = dHd * U64 * _dsilu(G64)
    q64 = fwd["q"].astype(F64)
    gx = fwd["gamma"].astype(F64)[:, None]
    g["dW_up"] = (dU / gx).T @ q64
    g["dW_gate"] = (dG / gx).T @ q64
    dX = F64(st["up"]["lam"]) * (dU @ st["up"]["S"].astype(F64)) \
        + F64(st["gate"]["lam"]) * (dG @ st["gate"]["S"].astype(F64))

    Up64, Gate64, Down64 = (np.asarray(a, dtype=F64) for a in (Up, Gate, Down))
    idx, gate, p = fwd["idx"], fwd["gate"], fwd["probs"]
    E = Up64.shape[0]
    ex8 = fwd.get("ex8")
    Xe = X64
    if ex8 is not None:                                             # the experts' operands as they were multiplied
        deq = lambda qg: qg[0].astype(F64) / qg[1].astype(F64)[:, None]
        Up64 = np.stack([deq(ex8["qw"]["up"][e]) for e in range(E)])
        Gate64 = np.stack([deq(ex8["qw"]["gate"][e]) for e in range(E)])
        Down64 = np.stack([deq(ex8["qw"]["down"][e]) for e in range(E)])
        Xe = fwd["q"].astype(F64) / fwd["gamma"].astype(F64)[:, None]
    Gr = al * dY64
    dUp, dGate, dDown = np.zeros_like(Up64), np.zeros_like(Gate64), np.zeros_like(Down64)
    dgate = np.einsum("ti,tji->tj", Gr, fwd["Ys"])
    for j in range(idx.shape[1]):
        for e in range(E):
            sel = np.nonzero(idx[:, j] == e)[0]
            if not sel.size:
                continue
            u, gg = fwd["ue"][sel, j], fwd["ge"][sel, j]
            a = _silu(gg) * u if ex8 is None else ex8["qa"][sel, j].astype(F64) / ex8["ga"][sel, j].astype(F64)[:, None]
            dy = gate[sel, j][:, None] * Gr[sel]
            dDown[e] += dy.T @ a
            da = dy @ Down64[e]
            du = da * _silu(gg)
            dg = da * u * _dsilu(gg)
            dUp[e] += du.T @ Xe[sel]
            dGate[e] += dg.T @ Xe[sel]
            dX[sel] += du @ Up64[e] + dg @ Gate64[e]
    dWr, dX_r, dlogit = _router_bwd(dgate, idx, p, X64, np.asarray(Wr, dtype=F64))
    g.update(dX=dX + dX_r, dUp=dUp, dGate=dGate, dDown=dDown, dWr=dWr, dU=dU, dG=dG, dHd=dHd)
    return g


# ----------------------------------------------------------------------------------------------
# App. A: inference on packed weights (decode GEMV)
# ----------------------------------------------------------------------------------------------
def decode_gemv(x, P, mu_lambda, alpha, beta, A=None, B=None, Wr=None, top_k=2):
    """One decode step on packed 1-bit weights: linear_fwd read from packed bits, with beta*lambda
    folded into a single fp16 scale (App. A: scalars merged for inference)."""
    return linear_fwd(x, None, alpha, beta, A=A, B=B, Wr=Wr, top_k=top_k, packed=P,
                      mu_lambda=mu_lambda, scale_fp16=True)


# ----------------------------------------------------------------------------------------------
# A stack of layers made of the pieces above (used only to check the chaining of the GPU calls)
# ----------------------------------------------------------------------------------------------
def stack_fwd(h0, layers, top_k=1):
    """Per layer: q,k,v = pure 1-bit linears of h (Sec. 3.1); m = (q+k+v)/3 stands in for the attention
    core; h1 = h + L_o(m); h2 = h1 + FFN(h1) (Sec. 3.2/3.3).  Every stored activation is bf16."""
    h = _round_io(h0, True)
    saved = []
    for w in layers:
        fq, fk, fv = (linear_fwd(h, w[n], 0.0, 1.0) for n in ("Wq", "Wk", "Wv"))
        q, k, v = (_round_io(f["Y"], True).astype(F64) for f in (fq, fk, fv))
        m = _round_io((q + k + v) / 3.0, True)
        fo = linear_fwd(m, w["Wo"], 0.0, 1.0)
        h1 = _round_io(h.astype(F64) + _round_io(fo["Y"], True), True)
        ff = ffn_fwd(h1, w["W_up"], w["W_gate"], w["W_down"], w["Up"], w["Gate"], w["Down"], w["Wr"], w["alpha"], w["beta"],
                     top_k=top_k, bf16=True)
        h2 = _round_io(h1.astype(F64) + _round_io(ff["Y"], True), True)
        saved.append(dict(h=h, m=m, h1=h1, fq=fq, fk=fk, fv=fv, fo=fo, ff=ff))
        h = h2
    return h, saved


def stack_bwd(dY, layers, saved):
    d = np.asarray(dY, dtype=F64)
    grads = []
    for w, sv in zip(reversed(layers), reversed(saved)):
        gf = ffn_bwd(d, sv["h1"], w["Up"], w["Gate"], w["Down"], w["Wr"], w["alpha"], w["beta"], sv["ff"])
        dh1 = d + gf["dX"]
        go = linear_bwd(dh1, sv["m"], w["Wo"], 0.0, 1.0, sv["fo"])
        dm = go["dX"] / 3.0
        gq, gk, gv = (linear_bwd(dm, sv["h"], w[n], 0.0, 1.0, sv[f]) for n, f in (("Wq", "fq"), ("Wk", "fk"), ("Wv", "fv")))
        d = dh1 + gq["dX"] + gk["dX"] + gv["dX"]
        grads.append(dict(Wq=gq["dW"], Wk=gk["dW"], Wv=gv["dW"], Wo=go["dW"], W_up=gf["dW_up"], W_gate=gf["dW_gate"],
                          W_down=gf["dW_down"], Up=gf["dUp"], Gate=gf["dGate"], Down=gf["dDown"], Wr=gf["dWr"]))
    return d, grads[::-1]


# ----------------------------------------------------------------------------------------------
# Sec. 3.1 (Y = (lambda/gamma) W Q(Norm(X))), App. A (RMSNorm merged with activation quantisation),
# App. B (RMSNorm in front of the quantiser): normalisation fused with the AbsMax quantiser
# ----------------------------------------------------------------------------------------------
def rmsnorm(X, g, eps):
    """x_hat[t, k] = x[t, k] * rstd[t] * g[k], rstd[t] = (mean_k x[t, k]^2 + eps)^(-1/2).
    The mean of squares and rstd are formed in fp64 and rstd is rounded once to fp32; the two products
    are fp32, (x * rstd) first."""
    X32 = np.asarray(X, dtype=F32)
    g32 = np.asarray(g, dtype=F32)
    ms = np.mean(X32.astype(F64) ** 2, axis=1)
    rstd = (1.0 / np.sqrt(ms + F64(eps))).astype(F32)
    xn = ((X32 * rstd[:, None]).astype(F32) * g32[None, :]).astype(F32)
    return xn, rstd


def rmsnorm_quant_fwd(X, g, eps, bf16=False):
    """Q(Norm(X)) in one pass: the normalised activations are rounded to their storage format (what
    the high-precision branch and the backward read), and the AbsMax quantiser of Sec. 3.1 acts on
    those stored values.  Returns x_hat (stored), q, gamma, rstd and x_tilde = q / gamma."""
    xn, rstd = rmsnorm(X, g, eps)
    xn = _round_io(xn, bf16)
    q, gamma = quant_act(xn)
    xt = (q.astype(F32) / gamma[:, None]).astype(F32)
    return dict(Xn=xn, q=q, gamma=gamma, rstd=rstd, Xt=xt)


def rmsnorm_bwd(dXn, X, g, rstd):
    """Backward of rmsnorm for an upstream gradient dXn w.r.t. x_hat (the quantiser is passed straight
    through, App. B.1).  With u = x * rstd:  dg[k] = sum_t dXn[t, k] u[t, k];
    dx[t, :] = rstd[t] * (g * dXn[t, :] - u[t, :] * mean_k(g[k] dXn[t, k] u[t, k])).  fp64 throughout,
    rstd as stored by the forward (fp32)."""
    d = np.asarray(dXn, dtype=F64)
    x = np.asarray(X, dtype=F64)
    g64 = np.asarray(g, dtype=F64)
    s = np.asarray(rstd, dtype=F64)[:, None]
    u = x * s
    dg = np.sum(d * u, axis=0)
    gd = d * g64[None, :]
    c = np.mean(gd * u, axis=1, keepdims=True)
    dx = s * (gd - u * c)
    return dx, dg


# ----------------------------------------------------------------------------------------------
# Sec. 3.2: the high-precision branch in its INT8 form ("8-bit weights are quantized identically to 8-bit
# activations"), for the two-factor branch B (A x) of a single linear
# ----------------------------------------------------------------------------------------------
def _dequant_scale(acc, g_row, g_col):
    """De-quantisation of an integer accumulator whose two factors each carry a per-row AbsMax scale (Sec. 3.1:
    the product of quantised operands is divided by their scales; Sec. 3.2 applies the activation quantiser to
    the 8-bit weights as well).  The paper does not fix the order of the two fp32 operations; the reading taken is
    fl32(fl32(fl32(1 / g_row) * fl32(acc)) / g_col): the token (row) scale comes off first as a reciprocal formed
    once per row, the weight-row (column) scale second by division."""
    s = (F32(1.0) / g_row.astype(F32)).astype(F32)
    v = (s[:, None] * acc.astype(F32)).astype(F32)
    return (v / g_col.astype(F32)[None, :]).astype(F32)


def hp_int8_fwd(X, A, B, bf16=False, q_gamma=None):
    """Y_hp = B~ Q(A~ Q(x)) with every factor on the INT8 grid of Sec. 3.1: x per token, the rows of A [r, n]
    and of B [m, r] per row (their output channel), and the hidden state per token again.  Both products are
    exact integer accumulations; the hidden state is stored in the I/O type before it is re-quantised.
    `q_gamma` passes in codes and gamma of X that the caller already has (the 1-bit branch's)."""
    q_x, g_x = quant_act(X) if q_gamma is None else q_gamma
    q_a, g_a = quant_act(np.asarray(A, dtype=F32))
    q_b, g_b = quant_act(np.asarray(B, dtype=F32))
    acc1 = q_x.astype(np.int64) @ q_a.astype(np.int64).T
    H = _round_io(_dequant_scale(acc1, g_x, g_a), bf16)
    q_h, g_h = quant_act(H)
    acc2 = q_h.astype(np.int64) @ q_b.astype(np.int64).T
    Yhp = _dequant_scale(acc2, g_h, g_b)
    return dict(q_x=q_x, g_x=g_x, q_a=q_a, g_a=g_a, q_b=q_b, g_b=g_b, acc1=acc1, H=H, q_h=q_h, g_h=g_h, acc2=acc2,
                Yhp=Yhp)


def hp_int8_bwd(dYhp, fwd):
    """STE backward of hp_int8_fwd (App. B.1): every quantiser is differentiated as identity, so each product
    is differentiated with the de-quantised factors it actually multiplied: with X~ = q_x / g_x, A~, B~, H~
    likewise,  dH = dY B~,  dB = dY^T H~,  dA = dH^T X~,  dX = dH A~.  fp64."""
    d = np.asarray(dYhp, dtype=F64)
    Xt = fwd["q_x"].astype(F64) / fwd["g_x"].astype(F64)[:, None]
    At = fwd["q_a"].astype(F64) / fwd["g_a"].astype(F64)[:, None]
    Bt = fwd["q_b"].astype(F64) / fwd["g_b"].astype(F64)[:, None]
    Ht = fwd["q_h"].astype(F64) / fwd["g_h"].astype(F64)[:, None]
    dH = d @ Bt
    return dict(dH=dH, dB=d.T @ Ht, dA=dH.T @ Xt, dX=dH @ At)


def decode_gemv_int8(x, P, mu_lambda, alpha, beta, A, B, Wr, top_k=2):
    """decode_gemv with the routed experts in their INT8 form (Sec. 3.2: 8-bit weights quantised like the
    8-bit activations; Sec. 3.3 routing; App. A inference scales): the 1-bit branch and the router are those of
    decode_gemv (the router reads the unquantised x), every selected expert is hp_int8_fwd on the token's own
    codes with a bf16 hidden state, and Y = Y1 + alpha * sum_j gate_j Y_e_j.  A [E, r, n], B [E, m, r]."""
    X32 = np.asarray(x, dtype=F32)
    base = linear_fwd(X32, None, 0.0, beta, packed=P, mu_lambda=mu_lambda, scale_fp16=True)
    idx, gate, p, logits = router_topk(X32, Wr, top_k)
    T = X32.shape[0]
    E, r = np.asarray(A).shape[0], np.asarray(A).shape[1]
    m = np.asarray(B).shape[1]
    Hs = np.zeros((T, top_k, r), F32)
    Ys = np.zeros((T, top_k, m), F32)
    for t in range(T):
        for j in range(top_k):
            e = int(idx[t, j])
            f = hp_int8_fwd(None, A[e], B[e], bf16=True, q_gamma=(base["q"][t:t + 1], base["gamma"][t:t + 1]))
            Hs[t, j] = f["H"][0]
            Ys[t, j] = f["Yhp"][0]
    Yhp = (gate.astype(F64)[:, :, None] * Ys.astype(F64)).sum(axis=1)
    return dict(acc=base["acc"], gamma=base["gamma"], Y1=base["Y1"], idx=idx, gate=gate, Hs=Hs, Ys=Ys, Yhp=Yhp,
                Y=base["Y1"].astype(F64) + F64(alpha) * Yhp)


def decode_ffn(x, P_up, P_gate, P_down, lam_up, lam_gate, lam_down, Up, Gate, Down, Wr, alpha, beta, top_k=2):
    """The decoupled FFN at inference on packed weights (Sec. 3.2 FFN equation, Sec. 3.3, App. A): the forward of
    ffn_fwd with the weight side read from packed bits and every layer's scalars folded into one fp16 scale
    (lambda_up, lambda_gate, beta * lambda_down).  x is quantised once for the up and the gate projection; U and
    G are stored in bf16; Hd = silu(G) * U is quantised from fp32; the routed experts are gated FFNs of hidden
    width r evaluated on the unquantised x:  Y = Y1 + alpha * sum_j gate_j Down_e (silu(Gate_e x) * (Up_e x))."""
    X32 = np.asarray(x, dtype=F32)
    X64 = X32.astype(F64)
    T, d = X32.shape
    f = np.asarray(P_up).shape[0]
    q, gamma = quant_act(X32)
    acc_u = onebit_acc(q, unpack_sign(np.asarray(P_up, dtype=np.uint32), d))
    acc_g = onebit_acc(q, unpack_sign(np.asarray(P_gate, dtype=np.uint32), d))
    su = (F32(np.float16(F32(lam_up))) / gamma).astype(F32)
    sg = (F32(np.float16(F32(lam_gate))) / gamma).astype(F32)
    U = _round_io((su[:, None] * acc_u.astype(F32)).astype(F32), True)
    G = _round_io((sg[:, None] * acc_g.astype(F32)).astype(F32), True)
    Hd = (_silu(G.astype(F64)) * U.astype(F64)).astype(F32)
    qh, gamma_h = quant_act(Hd)
    acc_d = onebit_acc(qh, unpack_sign(np.asarray(P_down, dtype=np.uint32), f))
    sd = (F32(np.float16(F32(F32(beta) * F32(lam_down)))) / gamma_h).astype(F32)
    Y1 = (sd[:, None] * acc_d.astype(F32)).astype(F32)
    idx, gate, p, logits = router_topk(X32, Wr, top_k)
    Up64, Gate64, Down64 = (np.asarray(a, dtype=F64) for a in (Up, Gate, Down))
    r = Up64.shape[1]
    act = np.zeros((T, top_k, r), F64)
    Ys = np.zeros((T, top_k, d), F64)
    for t in range(T):
        for j in range(top_k):
            e = int(idx[t, j])
            act[t, j] = _silu(Gate64[e] @ X64[t]) * (Up64[e] @ X64[t])
            Ys[t, j] = Down64[e] @ act[t, j]
    Yhp = (gate.astype(F64)[:, :, None] * Ys).sum(axis=1)
    return dict(acc_u=acc_u, acc_g=acc_g, U=U, G=G, Hd=Hd, qh=qh, gamma_h=gamma_h, acc_d=acc_d, Y1=Y1, idx=idx,
                gate=gate, act=act, Yhp=Yhp, Y=Y1.astype(F64) + F64(alpha) * Yhp)


def bits_per_weight(frac_1bit, frac_8bit):
    """Average bit-width of a decoupled layer (Table 1 percentages -> the 'Bit' column of Table 2)."""
    return frac_1bit * 1.0 + frac_8bit * 8.0


# ----------------------------------------------------------------------------------------------
# Sec. 4.6 ablation (contrast only): group-wise scales of the 1-bit weights
# ----------------------------------------------------------------------------------------------
def groupwise_scales(W, group=64):
    """lambda[i, g] = mean_{j in group g} |W[i, j]| for groups of `group` consecutive input columns, as the 16-bit value the
    ablation stores per group: the exact mean rounded to fp32, then to fp16 (returned as fp32)."""
    W64 = np.abs(np.asarray(W, dtype=F64))
    m, n = W64.shape
    assert n % group == 0
    lam = W64.reshape(m, n // group, group).sum(axis=2) / F64(group)
    return lam.astype(F32).astype(np.float16).astype(F32)


def groupwise_fwd(X, W, beta, group=64):
    """1-bit linear with one scale per `group` weights instead of one per tensor (the group-wise variant the paper
    evaluates and rejects in Sec. 4.6): Y[t, i] = beta / gamma_t * sum_g lambda[i, g] * sum_{j in g} S[i, j] q[t, j],
    with mu, S = Sign(W - mu) and the activation quantiser of Sec. 3.1.  group = 0 gives the per-tensor form."""
    mu, lam = weight_stats(W)
    S = binarise(W, mu).astype(np.int64)
    q, gamma = quant_act(X)
    q64 = q.astype(np.int64)
    T, n = q64.shape
    m = S.shape[0]
    if group == 0:
        Y = F64(beta) * F64(lam) * (q64 @ S.T).astype(F64) / gamma.astype(F64)[:, None]
        return dict(Y=Y, q=q, gamma=gamma, mu=mu, lam=lam)
    lg = groupwise_scales(W, group).astype(F64)          # [m, n/group]
    G = n // group
    Y = np.zeros((T, m), F64)
    for g in range(G):
        part = q64[:, g * group:(g + 1) * group] @ S[:, g * group:(g + 1) * group].T   # exact integers
        Y += part.astype(F64) * lg[None, :, g]
    Y = F64(beta) * Y / gamma.astype(F64)[:, None]
    return dict(Y=Y, q=q, gamma=gamma, mu=mu, lam_group=lg.astype(F32))
