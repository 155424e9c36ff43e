// The decoupled FFN (Sec. 3.2 FFN equation, Sec. 3.3):
//     Y = beta * FFN_1bit(X) + alpha * sum_j gate_j * FFN_e_j(X)
// FFN_1bit: three pure 1-bit linears around a gated unit, hidden state re-quantised before the down
// projection; FFN_e: routed experts of hidden width r (permute -> grouped GEMMs -> combine), either on 16-bit
// weights and the unquantised x, or in the INT8 form of the FFN equation: weight rows and the expert's hidden
// state on the AbsMax grid, x's codes shared with the 1-bit branch, exact int32 products de-quantised in the
// GEMM epilogue, and the STE backward on the de-quantised factors.
// This file sequences the kernels; all arithmetic lives in pq_gemm.hip / pq_quant.hip / pq_moe.hip.
#include <string.h>
#include "pq_internal.h"

namespace {

#define PQ_REQUIRE(cond, code, ...) \
  do { if (!(cond)) return pq_set_error(code, __VA_ARGS__); } while (0)

inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

struct cursor {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off = pq_align_up(off + (bytes ? bytes : 1), 256);
    return o;
  }
};

struct ffn_layout {
  // ctx
  size_t ml_up, ml_gate, ml_down, P_up, Pt_up, P_gate, Pt_gate, P_down, Pt_down, Xq, gx, Xt, U, G, Hq, gh, Ht;
  size_t idx, gate, probs, counts, offsets, perm, inv, Xp, ue, ge, a, Ys;
  // Up and Gate of every expert as one [E][2 r][D] matrix (both projections are one product whose output [S][2 r] starts
  // at ue: the left half of a row is u, the right half g)
  size_t UG;
  // INT8 experts: codes, row scales and de-quantised bf16 copies of the expert weights (of the rows of UG, and of Down);
  // x's codes and gamma in slot order; the hidden state's codes, scales and de-quantised copy (Xp then holds the rows of
  // X~ instead of X)
  size_t UGQ, gUG, UGT, DownQ, gDown, DownT, XqP, gxP, aQ, gA, aT, ctx_total;
  // workspace
  size_t stat, red_a, red_b, splitk, dHd, dU, dG, dYp, rd, da, du, dg, as, dXs, dlogit, dwr, dUG, ws_total;
  int n_red_a, n_red_b;
};

ffn_layout make_layout(const pq_ffn_desc& d) {
  ffn_layout L;
  memset(&L, 0, sizeof(L));
  // F here is the padded width of the 1-bit FFN's hidden state: d_ffn rounded up to whole packed words (Table 1's
  // 5076 -> 5088); every internal buffer uses it as its row length, the padded columns hold zero codes / gradients
  const size_t T = d.tokens, D = d.d_model, F = ((size_t)d.d_ffn + 31) / 32 * 32, r = d.hp_rank, E = d.n_experts, S = T * (size_t)d.top_k;
  cursor c;
  L.ml_up = c.take(8); L.ml_gate = c.take(8); L.ml_down = c.take(8);
  L.P_up = c.take(F * D / 8); L.Pt_up = c.take(F * D / 8);
  L.P_gate = c.take(F * D / 8); L.Pt_gate = c.take(F * D / 8);
  L.P_down = c.take(F * D / 8); L.Pt_down = c.take(F * D / 8);
  L.Xq = c.take(T * D); L.gx = c.take(T * 4); L.Xt = c.take(T * D * 2);
  L.U = c.take(T * F * 2); L.G = c.take(T * F * 2);
  L.Hq = c.take(T * F); L.gh = c.take(T * 4); L.Ht = c.take(T * F * 2);
  L.idx = c.take(S * 4); L.gate = c.take(S * 4); L.probs = c.take(T * E * 4);
  L.counts = c.take(E * 4); L.offsets = c.take((E + 1) * 4); L.perm = c.take(S * 4); L.inv = c.take(S * 4);
  L.Xp = c.take(S * D * 2); L.ue = c.take(2 * S * r * 2); L.ge = L.ue + S * r * 2; L.a = c.take(S * r * 2);
  L.Ys = c.take(S * D * 2);
  if (d.hp_kind == PQ_HP_LOWRANK_INT8) {
    // rows of [Up_e; Gate_e] (one [2 r][D] matrix per expert, as in the bf16 form): codes, gammas, de-quantised copy
    L.UGQ = c.take(E * 2 * r * D); L.gUG = c.take(E * 2 * r * 4); L.UGT = c.take(E * 2 * r * D * 2);
    L.DownQ = c.take(E * D * r); L.gDown = c.take(E * D * 4); L.DownT = c.take(E * D * r * 2);
    L.XqP = c.take(S * D); L.gxP = c.take(S * 4);
    L.aQ = c.take(S * r); L.gA = c.take(S * 4); L.aT = c.take(S * r * 2);
  }
  L.UG = c.take(E * 2 * r * D * 2);
  L.ctx_total = c.off;
  cursor w;
  L.stat = w.take(2 * sizeof(double) * 1024);
  L.n_red_a = pq_rowdot_blocks((int)S);
  L.n_red_b = pq_plan_gemm(0, (int)D, (int)F, (int)T).red_blocks;      // dW_down GEMM
  L.red_a = w.take(sizeof(double) * (size_t)L.n_red_a);
  L.red_b = w.take(sizeof(double) * (size_t)L.n_red_b);
  size_t sk = 0;
  const int Ti = d.tokens, Di = d.d_model, Fi = (int)F;
  // (the last seven: the expert products of a single high-precision branch, which run as plain GEMMs over all slots)
  const int Si = (int)S, ri = (int)r;
  const int shapes[11][3] = {{Di, Fi, Ti}, {Ti, Fi, Di}, {Ti, Di, Fi}, {Fi, Di, Ti},
                             {Si, 2 * ri, Di}, {Si, ri, Di}, {Si, Di, 2 * ri}, {Si, Di, ri}, {Di, ri, Si}, {2 * ri, Di, Si}, {ri, Di, Si}};
  for (const auto& sh : shapes) {
    if (sh[0] <= 0 || sh[1] <= 0) continue;
    const size_t b = pq_plan_gemm(0, sh[0], sh[1], sh[2]).ws_bytes;
    if (b > sk) sk = b;
  }
  // the expert up/gate projections and their input gradients split the contraction up to 8 ways: [8][S][r] fp32
  if (8 * S * r * sizeof(float) > sk) sk = 8 * S * r * sizeof(float);
  // the per-expert weight gradients cut their slot ranges into pieces (slabs of all experts' outputs)
  if (pq_mode2_ws_bytes((int)D, (int)r, (int)E, (int)S) > sk) sk = pq_mode2_ws_bytes((int)D, (int)r, (int)E, (int)S);
  if (pq_mode2_ws_bytes((int)r, (int)D, (int)E, (int)S) > sk) sk = pq_mode2_ws_bytes((int)r, (int)D, (int)E, (int)S);
  if (pq_mode2_ws_bytes(2 * (int)r, (int)D, (int)E, (int)S) > sk) sk = pq_mode2_ws_bytes(2 * (int)r, (int)D, (int)E, (int)S);
  if (8 * S * 2 * r * sizeof(float) > sk) sk = 8 * S * 2 * r * sizeof(float);
  L.splitk = w.take(sk);
  L.dHd = w.take(T * F * 2); L.dU = w.take(T * F * 2); L.dG = w.take(T * F * 2);
  L.dYp = w.take(S * D * 2); L.rd = w.take(S * 4);
  L.da = w.take(S * r * 2); L.du = w.take(2 * S * r * 2); L.dg = L.du + S * r * 2; L.as = w.take(S * r * 2);
  L.dXs = w.take(S * D * 2); L.dlogit = w.take(T * E * 4);
  L.dwr = w.take(pq_dwr_scratch_bytes((int)T, (int)D, (int)E));
  L.dUG = w.take(E * 2 * r * D * 4);
  L.ws_total = w.off;
  return L;
}

int check_ffn(const pq_ffn_desc* d) {
  PQ_REQUIRE(d != nullptr, PQ_ERR_BAD_ARG, "desc is NULL");
  PQ_REQUIRE(d->tokens >= 0 && d->d_model > 0 && d->d_ffn > 0 && d->hp_rank > 0, PQ_ERR_BAD_ARG, "bad dimension");
  PQ_REQUIRE(d->io_dtype == PQ_BF16, PQ_ERR_DTYPE, "the FFN path runs on bf16 I/O only");
  PQ_REQUIRE(d->d_model % 32 == 0 && d->d_ffn % 4 == 0, PQ_ERR_SHAPE, "d_model=%d must be a multiple of 32 and d_ffn=%d of 4",
             d->d_model, d->d_ffn);
  PQ_REQUIRE(d->hp_rank % 8 == 0, PQ_ERR_SHAPE, "hp_rank=%d must be a multiple of 8", d->hp_rank);
  PQ_REQUIRE(d->n_experts >= 1 && d->n_experts <= 64, PQ_ERR_BAD_ARG, "n_experts=%d must be in 1..64", d->n_experts);
  PQ_REQUIRE(d->top_k >= 1 && d->top_k <= d->n_experts, PQ_ERR_BAD_ARG, "top_k=%d must be in 1..n_experts", d->top_k);
  PQ_REQUIRE(d->hp_kind == PQ_HP_LOWRANK_BF16 || d->hp_kind == PQ_HP_LOWRANK_INT8, PQ_ERR_BAD_ARG, "hp_kind=%d is not a pq_hp_kind",
             d->hp_kind);
  PQ_REQUIRE(d->hp_kind != PQ_HP_LOWRANK_INT8 || d->hp_rank % 32 == 0, PQ_ERR_SHAPE, "INT8 experts need hp_rank=%d to be a multiple of 32",
             d->hp_rank);
  return PQ_OK;
}

pq_epilogue epi0() {
  pq_epilogue e;
  memset(&e, 0, sizeof(e));
  e.scale = 1.0f;
  return e;
}

int pack_weight(const void* W, int N, int K, char* cx, size_t offP, size_t offPt, size_t offml, double* part, hipStream_t s) {
  const size_t n = (size_t)N * K;
  const int nb = pq_stats_blocks(n);
  if (int e = pq_launch_wstats_partial(W, PQ_BF16, n, part, nb, s)) return e;
  return pq_launch_pack(W, PQ_BF16, N, K, part, nb, (uint32_t*)(cx + offP), (uint32_t*)(cx + offPt), (float*)(cx + offml), s);
}

}  // namespace

extern "C" size_t pq_ffn_ctx_bytes(const pq_ffn_desc* d) {
  if (check_ffn(d) != PQ_OK) return 0;
  return make_layout(*d).ctx_total;
}
// Where pq_ffn_fwd leaves what it stores in ctx (for inspection: tests compare the stored codes with the oracle's).
extern "C" int pq_ffn_ctx_section(const pq_ffn_desc* d, int32_t section, size_t* offset, size_t* bytes) {
  if (int e = check_ffn(d)) return e;
  PQ_REQUIRE(offset && bytes, PQ_ERR_BAD_ARG, "NULL result pointer");
  const ffn_layout L = make_layout(*d);
  const size_t T = d->tokens, D = d->d_model, F = ((size_t)d->d_ffn + 31) / 32 * 32;
  switch (section) {
    case PQ_FFN_CTX_XQ: *offset = L.Xq; *bytes = T * D; break;
    case PQ_FFN_CTX_GAMMA_X: *offset = L.gx; *bytes = T * 4; break;
    case PQ_FFN_CTX_U: *offset = L.U; *bytes = T * F * 2; break;
    case PQ_FFN_CTX_G: *offset = L.G; *bytes = T * F * 2; break;
    case PQ_FFN_CTX_HQ: *offset = L.Hq; *bytes = T * F; break;
    case PQ_FFN_CTX_GAMMA_H: *offset = L.gh; *bytes = T * 4; break;
    default: return pq_set_error(PQ_ERR_BAD_ARG, "unknown ctx section %d", section);
  }
  return PQ_OK;
}

extern "C" size_t pq_ffn_workspace_bytes(const pq_ffn_desc* d) {
  if (check_ffn(d) != PQ_OK) return 0;
  return make_layout(*d).ws_total;
}

extern "C" int pq_ffn_fwd(const pq_ffn_desc* d, const void* X, const void* W_up, const void* W_gate, const void* W_down,
                          const void* Up, const void* Gate, const void* Down, const void* Wr, void* Y, void* ctx,
                          size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_ffn(d)) return e;
  const ffn_layout L = make_layout(*d);
  PQ_REQUIRE(X && W_up && W_gate && W_down && Up && Gate && Down && Wr && Y && ctx && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(W_up) && aligned16(W_gate) && aligned16(W_down) && aligned16(Up) && aligned16(Gate) &&
                 aligned16(Down) && aligned16(Wr) && aligned16(Y) && aligned16(ctx) && aligned16(workspace),
             PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  hipStream_t s = (hipStream_t)stream;
  char* cx = (char*)ctx;
  char* ws = (char*)workspace;
  // Fv: the width of the 1-bit FFN as the caller's weights have it; F: that width in whole packed words
  const int T = d->tokens, D = d->d_model, Fv = d->d_ffn, F = (Fv + 31) / 32 * 32, r = d->hp_rank, E = d->n_experts, k = d->top_k, S = T * k;
  double* part = (double*)(ws + L.stat);
  void* sk = ws + L.splitk;

  int8_t* Xq = (int8_t*)(cx + L.Xq);
  float* gx = (float*)(cx + L.gx);
  const bool combo = T > 0 && D <= 8192;   // the quantiser of X shares the launch of W_up's statistics
  if (combo) {
    const size_t n = (size_t)Fv * D;
    const int nb = pq_stats_blocks(n);
    if (int e = pq_launch_wstats_quant(W_up, n, part, nb, X, T, D, Xq, gx, (uint16_t*)(cx + L.Xt), s)) return e;
    if (int e = pq_launch_pack(W_up, PQ_BF16, Fv, D, part, nb, (uint32_t*)(cx + L.P_up), (uint32_t*)(cx + L.Pt_up),
                               (float*)(cx + L.ml_up), s)) return e;
  } else if (int e = pack_weight(W_up, Fv, D, cx, L.P_up, L.Pt_up, L.ml_up, part, s)) return e;
  // the packer pads partial words with +1 bits (columns Fv.. of P_down's rows, rows Fv.. of the transposed packings of
  // W_up and W_gate); rows Fv.. of P_up, P_gate and Pt_down are never written: whatever they hold lands in columns of
  // U, G and dHd that the gated unit and its backward replace by zeros
  if (int e = pack_weight(W_gate, Fv, D, cx, L.P_gate, L.Pt_gate, L.ml_gate, part, s)) return e;
  if (int e = pack_weight(W_down, D, Fv, cx, L.P_down, L.Pt_down, L.ml_down, part, s)) return e;
  const bool hp8 = d->hp_kind == PQ_HP_LOWRANK_INT8;
  if (hp8) {  // the experts' weight rows on the AbsMax grid (codes, gamma per row, de-quantised copy for the backward)
    if (int e = pq_launch_concat_expert_rows(Up, Gate, E, r, D, cx + L.UG, s)) return e;
    if (int e = pq_launch_quant_act(cx + L.UG, PQ_BF16, E * 2 * r, D, (int8_t*)(cx + L.UGQ), (float*)(cx + L.gUG), (uint16_t*)(cx + L.UGT), s)) return e;
    if (int e = pq_launch_quant_act(Down, PQ_BF16, E * D, r, (int8_t*)(cx + L.DownQ), (float*)(cx + L.gDown), (uint16_t*)(cx + L.DownT), s)) return e;
  }
  if (T == 0)  // no tokens: leave empty expert segments behind so that a backward call is well defined
    return pq_launch_route((const int*)(cx + L.idx), 0, E, (int*)(cx + L.counts), (int*)(cx + L.offsets), (int*)(cx + L.perm),
                           (int*)(cx + L.inv), s);

  if (!combo)
    if (int e = pq_launch_quant_act(X, PQ_BF16, T, D, Xq, gx, (uint16_t*)(cx + L.Xt), s)) return e;
  {  // U and G: pure 1-bit linears (no feature scale of their own)
    pq_operand A{Xq, D, PQ_SRC_KC8, nullptr};
    pq_operand Bu{cx + L.P_up, D / 8, PQ_SRC_BITS8, nullptr};
    pq_epilogue e = epi0();
    e.C = cx + L.U; e.ldc = F; e.out_kind = PQ_OUT_BF16; e.dev_scale = (const float*)(cx + L.ml_up) + 1; e.row_div = gx;
    if (int err = pq_launch_gemm(0, T, F, D, A, Bu, e, s, PQP_GEMM_ONEBIT, sk)) return err;
    pq_operand Bg{cx + L.P_gate, D / 8, PQ_SRC_BITS8, nullptr};
    e.C = cx + L.G; e.dev_scale = (const float*)(cx + L.ml_gate) + 1;
    if (int err = pq_launch_gemm(0, T, F, D, A, Bg, e, s, PQP_GEMM_ONEBIT, sk)) return err;
  }
  int8_t* Hq = (int8_t*)(cx + L.Hq);
  float* gh = (float*)(cx + L.gh);
  if (int e = pq_launch_swiglu_quant(cx + L.U, cx + L.G, T, F, Fv, Hq, gh, cx + L.Ht, s)) return e;
  {  // Y = beta * (lambda_d / gamma_h) * acc
    pq_operand A{Hq, F, PQ_SRC_KC8, nullptr};
    pq_operand B{cx + L.P_down, F / 8, PQ_SRC_BITS8, nullptr};
    pq_epilogue e = epi0();
    e.C = Y; e.ldc = D; e.out_kind = PQ_OUT_BF16; e.scale = d->beta; e.dev_scale = (const float*)(cx + L.ml_down) + 1; e.row_div = gh;
    if (int err = pq_launch_gemm(0, T, D, F, A, B, e, s, PQP_GEMM_ONEBIT, sk)) return err;
  }
  // routed experts: router -> stable permutation by expert -> gather -> grouped GEMMs -> combine
  int* idx = (int*)(cx + L.idx);
  float* gate = (float*)(cx + L.gate);
  int* offsets = (int*)(cx + L.offsets);
  int* perm = (int*)(cx + L.perm);
  int* inv = (int*)(cx + L.inv);
  // a single branch (the paper's default, N = 1) has nothing to route: gate 1, identity permutation, X itself in slot order
  const bool one = E == 1;
  if (one) {
    if (int e = pq_launch_route_single(S, idx, gate, (float*)(cx + L.probs), (int*)(cx + L.counts), offsets, perm, inv, s)) return e;
  } else {
    if (int e = pq_launch_router(X, Wr, PQ_BF16, T, D, E, k, idx, gate, (float*)(cx + L.probs), s)) return e;
    if (int e = pq_launch_route(idx, S, E, (int*)(cx + L.counts), offsets, perm, inv, s)) return e;
  }
  pq_gemm_group g1{offsets, E, 1, 0, 0, S};
  // a single branch (the paper's default, N = 1): every slot belongs to it, so its products are plain GEMMs over all slots
  // (they then take the split rules and kernels of plain GEMMs, the four-wavefront weight-gradient kernel among them)
  const pq_gemm_group* pg1 = one ? nullptr : &g1;
  if (hp8) {
    // slot-ordered X~ (for the backward), codes (int8 rows moved as D/2 16-bit units) and gamma of x; with a single
    // branch the slot order is the token order and the originals serve
    const void* xqp = one ? (const void*)Xq : (const void*)(cx + L.XqP);
    const float* gxp = one ? (const float*)gx : (const float*)(cx + L.gxP);
    if (!one) {
      if (int e = pq_launch_gather_rows(cx + L.Xt, perm, k, S, D, cx + L.Xp, s)) return e;
      if (int e = pq_launch_gather_rows(Xq, perm, k, S, D / 2, cx + L.XqP, s)) return e;
      if (int e = pq_launch_gather_f32(gx, perm, k, S, (float*)(cx + L.gxP), s)) return e;
    }
    {  // [u | g] = (q_x q_w^T) / (gamma_x gamma_w), bf16: both projections as one product with 2 r outputs per slot
      pq_operand A{xqp, D, PQ_SRC_KC8, nullptr};
      pq_operand B{cx + L.UGQ, D, PQ_SRC_KC8, nullptr};
      pq_epilogue e = epi0();
      e.C = cx + L.ue; e.ldc = 2 * r; e.out_kind = PQ_OUT_BF16; e.row_div = gxp; e.col_div = (const float*)(cx + L.gUG);
      g1.b_stride = (long)2 * r * D; g1.coldiv_stride = 2 * r;
      if (int err = pq_launch_gemm(0, S, 2 * r, D, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
    }
    if (int e = pq_launch_expert_act(cx + L.ue, cx + L.ue + (size_t)r * 2, 2 * r, S, r, cx + L.a, s)) return e;
    if (int e = pq_launch_quant_act(cx + L.a, PQ_BF16, S, r, (int8_t*)(cx + L.aQ), (float*)(cx + L.gA), (uint16_t*)(cx + L.aT), s)) return e;
    {
      pq_operand A{cx + L.aQ, r, PQ_SRC_KC8, nullptr};
      pq_operand B{cx + L.DownQ, r, PQ_SRC_KC8, nullptr};
      pq_epilogue e = epi0();
      e.C = cx + L.Ys; e.ldc = D; e.out_kind = PQ_OUT_BF16; e.row_div = (const float*)(cx + L.gA); e.col_div = (const float*)(cx + L.gDown);
      g1.b_stride = (long)D * r; g1.coldiv_stride = D;
      if (int err = pq_launch_gemm(0, S, D, r, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
    }
    return pq_launch_combine_fwd(Y, cx + L.Ys, inv, gate, d->alpha, T, k, D, s);
  }
  const void* xp = one ? X : cx + L.Xp;
  if (!one)
    if (int e = pq_launch_gather_rows(X, perm, k, S, D, cx + L.Xp, s)) return e;
  // [u | g] = Xp [Up_e; Gate_e]^T: both projections as one product with 2 r outputs per slot
  if (int e = pq_launch_concat_expert_rows(Up, Gate, E, r, D, cx + L.UG, s)) return e;
  {
    pq_operand A{xp, D, PQ_SRC_KC16, nullptr};
    pq_operand B{cx + L.UG, D, PQ_SRC_KC16, nullptr};
    pq_epilogue e = epi0();
    e.C = cx + L.ue; e.ldc = 2 * r; e.out_kind = PQ_OUT_BF16;
    g1.b_stride = (long)2 * r * D;
    if (int err = pq_launch_gemm(0, S, 2 * r, D, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
  }
  if (int e = pq_launch_expert_act(cx + L.ue, cx + L.ue + (size_t)r * 2, 2 * r, S, r, cx + L.a, s)) return e;
  {
    pq_operand A{cx + L.a, r, PQ_SRC_KC16, nullptr};
    pq_operand B{Down, r, PQ_SRC_KC16, nullptr};
    pq_epilogue e = epi0();
    e.C = cx + L.Ys; e.ldc = D; e.out_kind = PQ_OUT_BF16;
    g1.b_stride = (long)D * r;
    if (int err = pq_launch_gemm(0, S, D, r, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
  }
  return pq_launch_combine_fwd(Y, cx + L.Ys, inv, gate, d->alpha, T, k, D, s);
}

extern "C" int pq_ffn_bwd(const pq_ffn_desc* d, const void* dY, const void* X, const void* Up, const void* Gate,
                          const void* Down, const void* Wr, const void* ctx, size_t ctx_bytes, void* dX, float* dW_up,
                          float* dW_gate, float* dW_down, float* dUp, float* dGate, float* dDown, float* dWr,
                          float* dalpha_dbeta, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_ffn(d)) return e;
  const ffn_layout L = make_layout(*d);
  PQ_REQUIRE(dY && X && Up && Gate && Down && Wr && ctx && dX && dW_up && dW_gate && dW_down && dUp && dGate && dDown && dWr &&
                 dalpha_dbeta && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(dY) && aligned16(X) && aligned16(Up) && aligned16(Gate) && aligned16(Down) && aligned16(Wr) &&
                 aligned16(ctx) && aligned16(dX) && aligned16(dW_up) && aligned16(dW_gate) && aligned16(dW_down) &&
                 aligned16(dUp) && aligned16(dGate) && aligned16(dDown) && aligned16(workspace),
             PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  hipStream_t s = (hipStream_t)stream;
  const char* cx = (const char*)ctx;
  char* ws = (char*)workspace;
  const int T = d->tokens, D = d->d_model, Fv = d->d_ffn, F = (Fv + 31) / 32 * 32, r = d->hp_rank, E = d->n_experts, k = d->top_k, S = T * k;
  void* sk = ws + L.splitk;
  if (d->hp_kind == PQ_HP_LOWRANK_INT8) {  // STE: each product is differentiated with the de-quantised factors it multiplied
    Down = cx + L.DownT;
  }
  const void* a_fwd = d->hp_kind == PQ_HP_LOWRANK_INT8 ? cx + L.aT : cx + L.a;
  const float* ml_up = (const float*)(cx + L.ml_up);
  const float* ml_gate = (const float*)(cx + L.ml_gate);
  const float* ml_down = (const float*)(cx + L.ml_down);
  double* red_a = (double*)(ws + L.red_a);
  double* red_b = (double*)(ws + L.red_b);

  {  // dW_down = beta * dY^T Ht ;  d beta = lambda_d * sum S_d .* (dY^T Ht)
    pq_operand A{dY, D, PQ_SRC_KS16, nullptr};
    pq_operand B{cx + L.Ht, F, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi0();
    e.C = dW_down; e.ldc = Fv; e.out_kind = PQ_OUT_F32; e.scale = d->beta;
    if (Fv != F) e.n_limit = Fv;                     // the padded columns (zero: Ht is zero there) are not part of dW_down
    e.sign_bytes = (const uint8_t*)(cx + L.P_down); e.ld_sign = F / 8; e.partials = red_b;
    if (int err = pq_launch_gemm(0, D, F, T, A, B, e, s, PQP_GEMM_DW, sk)) return err;
  }
  if (T > 0) {
    {  // dHd = beta * lambda_d * dY S_d
      pq_operand A{dY, D, PQ_SRC_KC16, nullptr};
      pq_operand B{cx + L.Pt_down, D / 8, PQ_SRC_BITS16, nullptr};
      pq_epilogue e = epi0();
      e.C = ws + L.dHd; e.ldc = F; e.out_kind = PQ_OUT_BF16; e.scale = d->beta; e.dev_scale = ml_down + 1;
      if (int err = pq_launch_gemm(0, T, F, D, A, B, e, s, PQP_GEMM_DX, sk)) return err;
    }
    if (int err = pq_launch_swiglu_bwd(ws + L.dHd, cx + L.U, cx + L.G, T, F, Fv, ws + L.dU, ws + L.dG, s)) return err;
    {  // dX = lambda_u dU S_u + lambda_g dG S_g
      pq_operand A{ws + L.dU, F, PQ_SRC_KC16, nullptr};
      pq_operand B{cx + L.Pt_up, F / 8, PQ_SRC_BITS16, nullptr};
      pq_epilogue e = epi0();
      e.C = dX; e.ldc = D; e.out_kind = PQ_OUT_BF16; e.dev_scale = ml_up + 1;
      if (int err = pq_launch_gemm(0, T, D, F, A, B, e, s, PQP_GEMM_DX, sk)) return err;
      pq_operand A2{ws + L.dG, F, PQ_SRC_KC16, nullptr};
      pq_operand B2{cx + L.Pt_gate, F / 8, PQ_SRC_BITS16, nullptr};
      e.accumulate = 1; e.dev_scale = ml_gate + 1;
      if (int err = pq_launch_gemm(0, T, D, F, A2, B2, e, s, PQP_GEMM_DX, sk)) return err;
    }
  }
  {  // dW_up = dU^T Xt, dW_gate = dG^T Xt
    pq_operand B{cx + L.Xt, D, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi0();
    e.ldc = D; e.out_kind = PQ_OUT_F32;
    if (Fv != F) e.m_limit = Fv;                     // rows Fv.. of the padded product do not exist in dW_up / dW_gate
    pq_operand A{ws + L.dU, F, PQ_SRC_KS16, nullptr};
    e.C = dW_up;
    if (int err = pq_launch_gemm(0, F, D, T, A, B, e, s, PQP_GEMM_DW, sk)) return err;
    pq_operand A2{ws + L.dG, F, PQ_SRC_KS16, nullptr};
    e.C = dW_gate;
    if (int err = pq_launch_gemm(0, F, D, T, A2, B, e, s, PQP_GEMM_DW, sk)) return err;
  }
  // experts
  const int* idx = (const int*)(cx + L.idx);
  const float* gate = (const float*)(cx + L.gate);
  const int* offsets = (const int*)(cx + L.offsets);
  const int* perm = (const int*)(cx + L.perm);
  const int* inv = (const int*)(cx + L.inv);
  float* rd = (float*)(ws + L.rd);
  const bool hp8 = d->hp_kind == PQ_HP_LOWRANK_INT8;
  const bool one = E == 1;                           // a single branch: identity permutation, plain GEMMs over all slots (see the forward)
  const void* dyp = one ? dY : ws + L.dYp;
  // what the up and gate products multiplied: X, or with INT8 experts its de-quantised codes
  const void* xp = one ? (hp8 ? (const void*)(cx + L.Xt) : X) : (const void*)(cx + L.Xp);
  if (!one)
    if (int e = pq_launch_gather_rows(dY, perm, k, S, D, ws + L.dYp, s)) return e;
  if (int e = pq_launch_rowdot(dyp, cx + L.Ys, perm, gate, S, D, rd, red_a, s)) return e;
  // d alpha (row dots above) and d beta (partials of the dW_down GEMM): one launch for both fixed-order sums
  if (int e = pq_launch_reduce_partials2(red_a, S > 0 ? L.n_red_a : 0, 1.0f, nullptr, dalpha_dbeta, red_b, L.n_red_b, 1.0f, ml_down + 1,
                                         dalpha_dbeta + 1, s)) return e;
  pq_gemm_group g1{offsets, E, 1, 0, 0, S};
  pq_gemm_group g2{offsets, E, 2, 0, 0, S};
  const pq_gemm_group* pg1 = one ? nullptr : &g1;
  const pq_gemm_group* pg2 = one ? nullptr : &g2;
  if (S > 0) {  // da = dYp Down_e  (scaled by alpha*gate inside the activation backward)
    pq_operand A{dyp, D, PQ_SRC_KC16, nullptr};
    pq_operand B{Down, r, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi0();
    e.C = ws + L.da; e.ldc = r; e.out_kind = PQ_OUT_BF16;
    g1.b_stride = (long)D * r;
    if (int err = pq_launch_gemm(0, S, r, D, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
  }
  // u | g and du | dg lie side by side in [S][2 r] matrices (Up and Gate are one weight matrix per expert, in both forms)
  if (int e = pq_launch_expert_act_bwd(ws + L.da, cx + L.ue, cx + L.ue + (size_t)r * 2, a_fwd, perm, gate, d->alpha, S, r, 2 * r,
                                       ws + L.du, ws + L.du + (size_t)r * 2, ws + L.as, s)) return e;
  {  // per-expert weight gradients: contraction over the expert's slots
    pq_operand A{dyp, D, PQ_SRC_KS16, nullptr};
    pq_operand B{ws + L.as, r, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi0();
    e.C = dDown; e.ldc = r; e.out_kind = PQ_OUT_F32;
    g2.c_stride = (long)D * r;
    if (int err = pq_launch_gemm(0, D, r, S, A, B, e, s, PQP_GEMM_EXPERT, sk, pg2)) return err;
    pq_operand Bx{xp, D, PQ_SRC_KS16, nullptr};
    {   // d[Up_e; Gate_e] = [du | dg]^T Xp, then split into the caller's two gradients
      pq_operand Aug{ws + L.du, 2 * r, PQ_SRC_KS16, nullptr};
      e.C = ws + L.dUG; e.ldc = D;
      g2.c_stride = (long)2 * r * D;
      if (int err = pq_launch_gemm(0, 2 * r, D, S, Aug, Bx, e, s, PQP_GEMM_EXPERT, sk, pg2)) return err;
      if (int err = pq_launch_split_expert_rows((const float*)(ws + L.dUG), E, r, D, dUp, dGate, s)) return err;
    }
  }
  if (S > 0) {  // dXs = [du | dg] [Up_e; Gate_e]  (INT8 experts: the de-quantised rows)
    pq_operand A{ws + L.du, 2 * r, PQ_SRC_KC16, nullptr};
    pq_operand B{hp8 ? cx + L.UGT : cx + L.UG, D, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi0();
    e.C = ws + L.dXs; e.ldc = D; e.out_kind = PQ_OUT_BF16;
    g1.b_stride = (long)2 * r * D;
    if (int err = pq_launch_gemm(0, S, D, 2 * r, A, B, e, s, PQP_GEMM_EXPERT, sk, pg1)) return err;
  }
  float* dlogit = (float*)(ws + L.dlogit);
  if (one) {   // softmax over one logit is constant: no gradient reaches the router
    if (int e = pq_launch_zero_f32(dWr, (size_t)D, s)) return e;
    return pq_launch_combine_bwd(dX, ws + L.dXs, inv, nullptr, Wr, T, k, D, 0, s);
  }
  if (int e = pq_launch_router_bwd(rd, inv, idx, (const float*)(cx + L.probs), d->alpha, T, k, E, dlogit, s)) return e;
  if (int e = pq_launch_dwr(dlogit, X, T, D, E, (float*)(ws + L.dwr), dWr, s)) return e;
  return pq_launch_combine_bwd(dX, ws + L.dXs, inv, dlogit, Wr, T, k, D, E, s);
}
