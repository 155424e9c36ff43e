"""Thin ctypes binding over libpquant.so: argument marshalling only.

Every computation runs in the HIP kernels behind the C ABI (include/pquant.h).  PyTorch is used for
device memory and the current stream.  There is no CPU fallback: if the library has not been
built, the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpquant.so")

PQ_F32, PQ_BF16 = 0, 1
PQ_W_MASTER, PQ_W_PACKED = 0, 1
PQ_STE_IDENTITY, PQ_STE_CLIP = 0, 1
PQ_HP_LOWRANK_BF16, PQ_HP_LOWRANK_INT8 = 0, 1
PQ_PACKED_ROWMAJOR, PQ_PACKED_TILED64 = 0, 1

EXPORTS = [
    "pq_version", "pq_last_error_string", "pq_quant_act", "pq_pack_workspace_bytes", "pq_pack_sign",
    "pq_router_topk", "pq_onebit_acc", "pq_linear_ctx_bytes", "pq_linear_workspace_bytes",
    "pq_linear_fwd", "pq_linear_bwd", "pq_prof_enable", "pq_prof_count", "pq_prof_label", "pq_prof_read",
    "pq_prof_reset", "pq_decode_workspace_bytes", "pq_decode_gemv", "pq_pack_tiled64_bytes", "pq_pack_retile64", "pq_ffn_ctx_bytes", "pq_ffn_workspace_bytes",
    "pq_ffn_fwd", "pq_ffn_bwd", "pq_glue_lincomb", "pq_glue_gather_rows",
    "pq_rmsnorm_quant_fwd", "pq_rmsnorm_bwd_workspace_bytes", "pq_rmsnorm_bwd",
    "pq_linear_norm_ctx_bytes", "pq_linear_norm_workspace_bytes", "pq_linear_norm_fwd", "pq_linear_norm_bwd",
    "pq_hp_int8_ctx_bytes", "pq_hp_int8_workspace_bytes", "pq_hp_int8_fwd", "pq_hp_int8_bwd", "pq_decode_gemv_int8",
    "pq_decode_ffn_workspace_bytes", "pq_decode_ffn", "pq_rmsnorm_bwd_static_max_bytes", "pq_rmsnorm_bwd_static",
    "pq_groupwise_workspace_bytes", "pq_groupwise_fwd", "pq_ffn_ctx_section",
]


class LinearDesc(C.Structure):
    _fields_ = [("tokens", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("hp_rank", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("io_dtype", C.c_int32), ("w_kind", C.c_int32),
                ("ste_mode", C.c_int32), ("ste_tau", C.c_float), ("alpha", C.c_float), ("beta", C.c_float),
                ("hp_kind", C.c_int32)]


class DecodeDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("d_in", C.c_int32), ("d_out", C.c_int32), ("hp_rank", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("n_layers", C.c_int32),
                ("packed_layout", C.c_int32), ("alpha", C.c_float)]


class FFNDesc(C.Structure):
    _fields_ = [("tokens", C.c_int32), ("d_model", C.c_int32), ("d_ffn", C.c_int32), ("hp_rank", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("io_dtype", C.c_int32), ("alpha", C.c_float),
                ("beta", C.c_float), ("hp_kind", C.c_int32)]


class DecodeFFNDesc(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("d_ffn", C.c_int32), ("hp_rank", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("n_layers", C.c_int32), ("alpha", C.c_float), ("batch", C.c_int32)]


class PQError(RuntimeError):
    pass


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_22592_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.pq_last_error_string.restype = C.c_char_p
        L.pq_prof_label.restype = C.c_char_p
        for name in ("pq_pack_workspace_bytes", "pq_linear_ctx_bytes", "pq_linear_workspace_bytes",
                     "pq_decode_workspace_bytes", "pq_pack_tiled64_bytes", "pq_ffn_ctx_bytes",
                     "pq_ffn_workspace_bytes", "pq_rmsnorm_bwd_workspace_bytes", "pq_linear_norm_ctx_bytes",
                     "pq_linear_norm_workspace_bytes", "pq_hp_int8_ctx_bytes", "pq_hp_int8_workspace_bytes",
                     "pq_decode_ffn_workspace_bytes", "pq_rmsnorm_bwd_static_max_bytes"):
            getattr(L, name).restype = C.c_size_t
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise PQError(f"libpquant error {rc}: {lib().pq_last_error_string().decode()}")


def _p(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t):
    if t.dtype == torch.float32:
        return PQ_F32
    if t.dtype == torch.bfloat16:
        return PQ_BF16
    raise PQError(f"unsupported dtype {t.dtype}")


def _bytes(n, device):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


def version():
    return lib().pq_version()


def quant_act(X):
    T, K = X.shape
    Xq = torch.empty((T, K), dtype=torch.int8, device=X.device)
    gamma = torch.empty((T,), dtype=torch.float32, device=X.device)
    _check(lib().pq_quant_act(_p(X), _dt(X), T, K, _p(Xq), _p(gamma), _stream()))
    return Xq, gamma


def quant_act_into(X, Xq, gamma):
    T, K = X.shape
    _check(lib().pq_quant_act(_p(X), _dt(X), T, K, _p(Xq), _p(gamma), _stream()))


def rmsnorm_quant_fwd_into(X, gain, eps, Xn, Xq, gamma, Xt, rstd):
    """Same call as rmsnorm_quant_fwd, writing into buffers the caller holds (any of Xn, Xt, rstd may be None)."""
    T, K = X.shape
    _check(lib().pq_rmsnorm_quant_fwd(_p(X), _p(gain), _dt(X), T, K, C.c_float(eps), _p(Xn), _p(Xq), _p(gamma), _p(Xt),
                                      _p(rstd), _stream()))


def rmsnorm_bwd_into(dXn, X, gain, rstd, dX, dgain, ws):
    T, K = X.shape
    _check(lib().pq_rmsnorm_bwd(_p(dXn), _p(X), _p(gain), _p(rstd), _dt(X), T, K, _p(dX), _p(dgain), _p(ws),
                                C.c_size_t(ws.numel()), _stream()))


def rmsnorm_bwd_static_into(dXn, X, gain, rstd, dX, dgain):
    """pq_rmsnorm_bwd_static: no workspace argument, nothing allocated by the call."""
    T, K = X.shape
    _check(lib().pq_rmsnorm_bwd_static(_p(dXn), _p(X), _p(gain), _p(rstd), _dt(X), T, K, _p(dX), _p(dgain), _stream()))


def rmsnorm_bwd_static_max_bytes():
    return lib().pq_rmsnorm_bwd_static_max_bytes()


def rmsnorm_quant_fwd(X, gain, eps, want_xn=True, want_xt=True, want_rstd=True):
    """Returns (Xn, Xq, gamma, Xt, rstd); entries not asked for are None."""
    T, K = X.shape
    Xq = torch.empty((T, K), dtype=torch.int8, device=X.device)
    gamma = torch.empty((T,), dtype=torch.float32, device=X.device)
    Xn = torch.empty_like(X) if want_xn else None
    Xt = torch.empty((T, K), dtype=torch.bfloat16, device=X.device) if want_xt else None
    rstd = torch.empty((T,), dtype=torch.float32, device=X.device) if want_rstd else None
    _check(lib().pq_rmsnorm_quant_fwd(_p(X), _p(gain), _dt(X), T, K, C.c_float(eps), _p(Xn), _p(Xq), _p(gamma), _p(Xt),
                                      _p(rstd), _stream()))
    return Xn, Xq, gamma, Xt, rstd


def rmsnorm_bwd(dXn, X, gain, rstd, ws=None):
    """Returns (dX, dgain)."""
    T, K = X.shape
    dX = torch.empty_like(X)
    dgain = torch.empty((K,), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = _bytes(lib().pq_rmsnorm_bwd_workspace_bytes(T, K), X.device)
    _check(lib().pq_rmsnorm_bwd(_p(dXn), _p(X), _p(gain), _p(rstd), _dt(X), T, K, _p(dX), _p(dgain), _p(ws),
                                C.c_size_t(ws.numel()), _stream()))
    return dX, dgain


def pack_sign(W, transposed=False):
    N, K = W.shape
    P = torch.empty((N, (K + 31) // 32), dtype=torch.int32, device=W.device)
    Pt = torch.empty((K, (N + 31) // 32), dtype=torch.int32, device=W.device) if transposed else None
    ml = torch.empty((2,), dtype=torch.float32, device=W.device)
    nws = lib().pq_pack_workspace_bytes(N, K)
    ws = _bytes(nws, W.device)
    _check(lib().pq_pack_sign(_p(W), _dt(W), N, K, _p(P), _p(Pt), _p(ml), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return P, Pt, ml


def router_topk(X, Wr, k, want_probs=True):
    T, K = X.shape
    E = Wr.shape[0]
    idx = torch.empty((T, k), dtype=torch.int32, device=X.device)
    gate = torch.empty((T, k), dtype=torch.float32, device=X.device)
    probs = torch.empty((T, E), dtype=torch.float32, device=X.device) if want_probs else None
    _check(lib().pq_router_topk(_p(X), _p(Wr), _dt(X), T, K, E, k, _p(idx), _p(gate), _p(probs), _stream()))
    return idx, gate, probs


def onebit_acc(Xq, P, N):
    T, K = Xq.shape
    acc = torch.empty((T, N), dtype=torch.int32, device=Xq.device)
    _check(lib().pq_onebit_acc(_p(Xq), _p(P), T, K, N, _p(acc), _stream()))
    return acc


def make_desc(tokens, d_in, d_out, hp_rank=0, n_experts=1, top_k=1, io_dtype=PQ_BF16, w_kind=PQ_W_MASTER,
              ste_mode=PQ_STE_IDENTITY, ste_tau=0.0, alpha=2.0, beta=0.2, hp_kind=PQ_HP_LOWRANK_BF16):
    return LinearDesc(tokens, d_in, d_out, hp_rank, n_experts, top_k, io_dtype, w_kind, ste_mode, ste_tau,
                      alpha, beta, hp_kind)


class LinearBuffers:
    """Caller-owned ctx / workspace for one descriptor (allocated once, reused across steps)."""

    def __init__(self, desc, device="cuda", ws=None):
        nctx = lib().pq_linear_ctx_bytes(C.byref(desc))
        nws = lib().pq_linear_workspace_bytes(C.byref(desc))
        if nctx == 0 or nws == 0:
            raise PQError(f"bad descriptor: {lib().pq_last_error_string().decode()}")
        self.ctx = _bytes(nctx, device)
        self.ws = ws if ws is not None else _bytes(nws, device)   # scratch may be shared between layers


def linear_fwd(desc, X, W, Y, bufs, A=None, B=None, Wr=None, mu_lambda=None, save=True):
    ctx = bufs.ctx if save else None
    _check(lib().pq_linear_fwd(C.byref(desc), _p(X), _p(W), _p(mu_lambda), _p(A), _p(B), _p(Wr), _p(Y),
                               _p(ctx), C.c_size_t(0 if ctx is None else ctx.numel()),
                               _p(bufs.ws), C.c_size_t(bufs.ws.numel()), _stream()))
    return Y


def linear_bwd(desc, dY, X, W, bufs, dX, dW, d_ab, A=None, B=None, Wr=None, dA=None, dB=None, dWr=None):
    _check(lib().pq_linear_bwd(C.byref(desc), _p(dY), _p(X), _p(W), _p(A), _p(B), _p(Wr),
                               _p(bufs.ctx), C.c_size_t(bufs.ctx.numel()), _p(dX), _p(dW), _p(dA), _p(dB),
                               _p(dWr), _p(d_ab), _p(bufs.ws), C.c_size_t(bufs.ws.numel()), _stream()))
    return dX, dW, d_ab


class LinearNormBuffers:
    """ctx / workspace of the linear with its normalisation in front."""

    def __init__(self, desc, device="cuda"):
        nctx = lib().pq_linear_norm_ctx_bytes(C.byref(desc))
        nws = lib().pq_linear_norm_workspace_bytes(C.byref(desc))
        if nctx == 0 or nws == 0:
            raise PQError(f"bad descriptor: {lib().pq_last_error_string().decode()}")
        self.ctx = _bytes(nctx, device)
        self.ws = _bytes(nws, device)


def linear_norm_fwd(desc, X, gain, eps, W, Y, bufs, A=None, B=None, Wr=None):
    _check(lib().pq_linear_norm_fwd(C.byref(desc), _p(X), _p(gain), C.c_float(eps), _p(W), _p(A), _p(B), _p(Wr), _p(Y),
                                    _p(bufs.ctx), C.c_size_t(bufs.ctx.numel()), _p(bufs.ws), C.c_size_t(bufs.ws.numel()),
                                    _stream()))
    return Y


def linear_norm_bwd(desc, dY, X, gain, W, bufs, dX, dgain, dW, d_ab, A=None, B=None, Wr=None, dA=None, dB=None, dWr=None):
    _check(lib().pq_linear_norm_bwd(C.byref(desc), _p(dY), _p(X), _p(gain), _p(W), _p(A), _p(B), _p(Wr), _p(bufs.ctx),
                                    C.c_size_t(bufs.ctx.numel()), _p(dX), _p(dgain), _p(dW), _p(dA), _p(dB), _p(dWr), _p(d_ab),
                                    _p(bufs.ws), C.c_size_t(bufs.ws.numel()), _stream()))
    return dX, dgain, dW, d_ab


class HpInt8Buffers:
    """ctx and workspace of the INT8 high-precision branch, with views of what the forward saved."""

    def __init__(self, T, K, N, r, device="cuda"):
        self.shape = (T, K, N, r)
        self.ctx = _bytes(lib().pq_hp_int8_ctx_bytes(T, K, N, r), device)
        self.ws = _bytes(lib().pq_hp_int8_workspace_bytes(T, K, N, r), device)

    def views(self):
        """(q_a, g_a, q_b, g_b, H, q_h, g_h) as tensors over ctx (same order and 256-byte rounding as the library)."""
        T, K, N, r = self.shape
        off = 0

        def take(nbytes, dtype, shape):
            nonlocal off
            v = self.ctx[off:off + nbytes].view(dtype).view(shape)
            off += (nbytes + 255) // 256 * 256
            return v
        q_a = take(r * K, torch.int8, (r, K)); g_a = take(r * 4, torch.float32, (r,)); take(r * K * 2, torch.bfloat16, (r, K))
        q_b = take(N * r, torch.int8, (N, r)); g_b = take(N * 4, torch.float32, (N,)); take(N * r * 2, torch.bfloat16, (N, r))
        H = take(T * r * 2, torch.bfloat16, (T, r)); q_h = take(T * r, torch.int8, (T, r)); g_h = take(T * 4, torch.float32, (T,))
        return q_a, g_a, q_b, g_b, H, q_h, g_h


def hp_int8_fwd(Xq, gamma_x, A, B, alpha, Y, bufs, accumulate=False):
    T, K, N, r = bufs.shape
    _check(lib().pq_hp_int8_fwd(_p(Xq), _p(gamma_x), _p(A), _p(B), _dt(A), T, K, N, r, C.c_float(alpha), _p(Y),
                                int(accumulate), _p(bufs.ctx), C.c_size_t(bufs.ctx.numel()), _p(bufs.ws),
                                C.c_size_t(bufs.ws.numel()), _stream()))


def hp_int8_bwd(dY, Xt, alpha, bufs, dX, dA, dB, accumulate_dX=False):
    T, K, N, r = bufs.shape
    _check(lib().pq_hp_int8_bwd(_p(dY), _p(Xt), _dt(dY), T, K, N, r, C.c_float(alpha), _p(bufs.ctx),
                                C.c_size_t(bufs.ctx.numel()), _p(dX), int(accumulate_dX), _p(dA), _p(dB), _p(bufs.ws),
                                C.c_size_t(bufs.ws.numel()), _stream()))


def groupwise_fwd(X, W, beta, group=64, Y=None, ws=None):
    """Sec. 4.6 contrast: the 1-bit forward with one fp16 scale per 64 weights (group=64) or the per-tensor scale in the
    same kernel (group=0).  X [T][K], W [N][K] bf16 on the device; returns Y [T][N] fp32."""
    import torch
    T, K = X.shape
    N = W.shape[0]
    lib().pq_groupwise_workspace_bytes.restype = C.c_size_t
    nbytes = lib().pq_groupwise_workspace_bytes(T, K, N)
    if ws is None:
        ws = torch.empty((max(int(nbytes), 256),), dtype=torch.uint8, device=X.device)
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=X.device)
    _check(lib().pq_groupwise_fwd(_p(X), _p(W), _dt(X), T, K, N, int(group), C.c_float(beta), _p(Y), _p(ws),
                                  C.c_size_t(ws.numel()), _stream()))
    return Y


def prof_enable(on=True):
    _check(lib().pq_prof_enable(1 if on else 0))


def prof_reset():
    _check(lib().pq_prof_reset())


def prof_read():
    """{label: (total_ms, launches)} for every kernel label with at least one recorded launch."""
    out = {}
    for i in range(lib().pq_prof_count()):
        ms, n = C.c_double(0), C.c_int(0)
        _check(lib().pq_prof_read(i, C.byref(ms), C.byref(n)))
        if n.value:
            out[lib().pq_prof_label(i).decode()] = (ms.value, n.value)
    return out


def decode_workspace(desc, device="cuda"):
    n = lib().pq_decode_workspace_bytes(C.byref(desc))
    if n == 0:
        raise PQError(f"bad decode descriptor: {lib().pq_last_error_string().decode()}")
    return _bytes(n, device)


def decode_gemv(desc, X, packed, scale_fp16, Y, ws, A=None, B=None, Wr=None, acc_out=None):
    """scale_fp16: int16/uint16 tensor [L] holding the fp16 bits of beta*lambda per layer."""
    _check(lib().pq_decode_gemv(C.byref(desc), _p(X), _p(packed), _p(scale_fp16), _p(A), _p(B), _p(Wr), _p(Y),
                                _p(acc_out), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return Y


def quant_rows(W):
    """AbsMax INT8 codes and gammas of the rows of the last axis of a bf16 / fp32 tensor (the activation quantiser
    applied to weight rows): returns (codes of W's shape, gammas of W's shape without the last axis)."""
    K = W.shape[-1]
    q, g = quant_act(W.reshape(-1, K).contiguous())
    return q.view(W.shape), g.view(W.shape[:-1])


def decode_gemv_int8(desc, X, packed, scale_fp16, Y, ws, Aq, gA, Bq, gB, Wr, acc_out=None):
    _check(lib().pq_decode_gemv_int8(C.byref(desc), _p(X), _p(packed), _p(scale_fp16), _p(Aq), _p(gA), _p(Bq), _p(gB),
                                     _p(Wr), _p(Y), _p(acc_out), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return Y


def decode_ws_hidden(desc, ws):
    """The expert hidden states [L][B][top_k][r] (fp32) inside a decode workspace (same section order and 256-byte
    rounding as the library: codes, bit planes, row sums, gammas, indices, gates, hidden states)."""
    L, B, K, k, r = desc.n_layers, desc.batch, desc.d_in, desc.top_k, desc.hp_rank
    off = 0
    for nbytes in (L * B * K, L * B * 8 * (K // 32) * 4, L * B * 4, L * B * 4, L * B * k * 4, L * B * k * 4):
        off = (off + nbytes + 255) // 256 * 256
    return ws[off:off + L * B * k * r * 4].view(torch.float32).view(L, B, k, r)


def decode_ws_idx(desc, ws):
    """The selected expert indices [L][B][top_k] (int32) inside a decode workspace (section order as in decode_ws_hidden)."""
    L, B, K, k = desc.n_layers, desc.batch, desc.d_in, desc.top_k
    off = 0
    for nbytes in (L * B * K, L * B * 8 * (K // 32) * 4, L * B * 4, L * B * 4):
        off = (off + nbytes + 255) // 256 * 256
    return ws[off:off + L * B * k * 4].view(torch.int32).view(L, B, k)


def decode_ffn_workspace(desc, device="cuda"):
    n = lib().pq_decode_ffn_workspace_bytes(C.byref(desc))
    if n == 0:
        raise PQError(f"bad decode FFN descriptor: {lib().pq_last_error_string().decode()}")
    return _bytes(n, device)


def decode_ffn(desc, X, packed_upgate, scale_upgate, packed_down, scale_down, UpGate, Down, Wr, Y, ws, acc_upgate=None):
    _check(lib().pq_decode_ffn(C.byref(desc), _p(X), _p(packed_upgate), _p(scale_upgate), _p(packed_down), _p(scale_down),
                               _p(UpGate), _p(Down), _p(Wr), _p(Y), _p(acc_upgate), _p(ws), C.c_size_t(ws.numel()), _stream()))
    return Y


def pack_retile64(P, K):
    """Row-major packed words [N][K/32] -> the row-interleaved order used by batch-1 decode."""
    N = P.shape[0]
    n = lib().pq_pack_tiled64_bytes(N, K)
    if n == 0:
        raise PQError("pq_pack_tiled64_bytes: bad shape")
    T = torch.empty((n // 4,), dtype=torch.int32, device=P.device)
    _check(lib().pq_pack_retile64(_p(P), N, K, _p(T), _stream()))
    return T


class FFNBuffers:
    def __init__(self, desc, device="cuda", ws=None):
        nctx = lib().pq_ffn_ctx_bytes(C.byref(desc))
        nws = lib().pq_ffn_workspace_bytes(C.byref(desc))
        if nctx == 0 or nws == 0:
            raise PQError(f"bad FFN descriptor: {lib().pq_last_error_string().decode()}")
        self.ctx = _bytes(nctx, device)
        self.ws = ws if ws is not None else _bytes(nws, device)


FFN_CTX_XQ, FFN_CTX_GAMMA_X, FFN_CTX_U, FFN_CTX_G, FFN_CTX_HQ, FFN_CTX_GAMMA_H = range(6)


def ffn_ctx_section(desc, bufs, section):
    """The bytes of one stored intermediate of pq_ffn_fwd inside bufs.ctx (a uint8 view)."""
    off, n = C.c_size_t(0), C.c_size_t(0)
    _check(lib().pq_ffn_ctx_section(C.byref(desc), int(section), C.byref(off), C.byref(n)))
    return bufs.ctx[off.value:off.value + n.value]


def ffn_fwd(desc, X, W_up, W_gate, W_down, Up, Gate, Down, Wr, Y, bufs):
    _check(lib().pq_ffn_fwd(C.byref(desc), _p(X), _p(W_up), _p(W_gate), _p(W_down), _p(Up), _p(Gate), _p(Down), _p(Wr),
                            _p(Y), _p(bufs.ctx), C.c_size_t(bufs.ctx.numel()), _p(bufs.ws), C.c_size_t(bufs.ws.numel()),
                            _stream()))
    return Y


def ffn_bwd(desc, dY, X, Up, Gate, Down, Wr, bufs, dX, dW_up, dW_gate, dW_down, dUp, dGate, dDown, dWr, d_ab):
    _check(lib().pq_ffn_bwd(C.byref(desc), _p(dY), _p(X), _p(Up), _p(Gate), _p(Down), _p(Wr), _p(bufs.ctx),
                            C.c_size_t(bufs.ctx.numel()), _p(dX), _p(dW_up), _p(dW_gate), _p(dW_down), _p(dUp),
                            _p(dGate), _p(dDown), _p(dWr), _p(d_ab), _p(bufs.ws), C.c_size_t(bufs.ws.numel()), _stream()))


def glue_lincomb(out, xs, cs):
    xs = list(xs) + [None] * (4 - len(xs))
    cs = list(cs) + [0.0] * (4 - len(cs))
    _check(lib().pq_glue_lincomb(_p(out), _p(xs[0]), _p(xs[1]), _p(xs[2]), _p(xs[3]), C.c_float(cs[0]), C.c_float(cs[1]),
                                 C.c_float(cs[2]), C.c_float(cs[3]), C.c_size_t(out.numel()), _stream()))
    return out


def glue_gather_rows(table, ids, out):
    _check(lib().pq_glue_gather_rows(_p(table), _p(ids), ids.numel(), table.shape[1], _p(out), _stream()))
    return out
