// C-ABI entry points of libpquant: argument validation, buffer layout, kernel sequencing.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include "pq_internal.h"

static thread_local char g_err[512] = "";

int pq_set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

extern "C" const char* pq_last_error_string(void) { return g_err; }
extern "C" int pq_version(void) { return 100; }

// ---------------------------------------------------------------------------------------------
// Optional per-kernel event timing
// ---------------------------------------------------------------------------------------------
#include <mutex>
#include <vector>
namespace {
struct prof_sample { hipEvent_t a, b; int label; bool closed; };
bool g_prof_on = false;
std::mutex g_prof_mu;
std::vector<prof_sample*> g_prof_samples;
const char* const g_prof_names[PQP_COUNT] = {
    "quant_act", "wstats_partial", "pack_sign", "router", "reduce_partials",
    "gemm_onebit_fwd", "gemm_hp_H", "gemm_hp_Y", "gemm_dH", "gemm_dX", "gemm_dX_hp",
    "gemm_dW", "gemm_dB", "gemm_dA", "gemm_other", "decode_prep", "decode_h", "decode_main", "moe_route", "moe_elementwise", "swiglu", "gemm_expert", "glue", "splitk_reduce", "rmsnorm_quant", "rmsnorm_bwd"};
}  // namespace

pq_prof_scope::pq_prof_scope(int label_, hipStream_t s_) : label(label_), s(s_), slot(nullptr) {
  if (!g_prof_on) return;
  prof_sample* ps = new prof_sample{nullptr, nullptr, label_, false};
  if (hipEventCreate(&ps->a) != hipSuccess || hipEventCreate(&ps->b) != hipSuccess) { delete ps; return; }
  (void)hipEventRecord(ps->a, s);
  slot = ps;
}
pq_prof_scope::~pq_prof_scope() {
  if (!slot) return;
  prof_sample* ps = (prof_sample*)slot;
  (void)hipEventRecord(ps->b, s);
  ps->closed = true;
  std::lock_guard<std::mutex> g(g_prof_mu);
  g_prof_samples.push_back(ps);
}

extern "C" int pq_prof_enable(int on) { g_prof_on = on != 0; return PQ_OK; }
extern "C" int pq_prof_count(void) { return PQP_COUNT; }
extern "C" const char* pq_prof_label(int label) { return (label >= 0 && label < PQP_COUNT) ? g_prof_names[label] : ""; }
extern "C" int pq_prof_read(int label, double* total_ms, int* launches) {
  if (!total_ms || !launches) return pq_set_error(PQ_ERR_BAD_ARG, "NULL output");
  std::lock_guard<std::mutex> g(g_prof_mu);
  double tot = 0.0; int n = 0;
  for (prof_sample* ps : g_prof_samples) {
    if (ps->label != label || !ps->closed) continue;
    float ms = 0.f;
    PQ_CHECK_HIP(hipEventSynchronize(ps->b));
    PQ_CHECK_HIP(hipEventElapsedTime(&ms, ps->a, ps->b));
    tot += ms; ++n;
  }
  *total_ms = tot; *launches = n;
  return PQ_OK;
}
extern "C" int pq_prof_reset(void) {
  std::lock_guard<std::mutex> g(g_prof_mu);
  for (prof_sample* ps : g_prof_samples) { (void)hipEventDestroy(ps->a); (void)hipEventDestroy(ps->b); delete ps; }
  g_prof_samples.clear();
  return PQ_OK;
}

namespace {

inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
inline size_t esize(int dtype) { return dtype == PQ_BF16 ? 2 : 4; }
inline int out_kind_of(int dtype) { return dtype == PQ_BF16 ? PQ_OUT_BF16 : PQ_OUT_F32; }

#define PQ_REQUIRE(cond, code, ...) \
  do { if (!(cond)) return pq_set_error(code, __VA_ARGS__); } while (0)

int check_dtype(int dtype) {
  PQ_REQUIRE(dtype == PQ_F32 || dtype == PQ_BF16, PQ_ERR_DTYPE, "dtype %d is not PQ_F32 or PQ_BF16", dtype);
  return PQ_OK;
}

pq_epilogue epi_zero() {
  pq_epilogue e;
  memset(&e, 0, sizeof(e));
  e.scale = 1.0f;
  return e;
}

// Buffer layout of one linear.  Sections are 256-byte aligned.
struct lin_layout {
  // ctx (saved by forward for backward)
  size_t mulam, P, Pt, Xq, gamma, Xt, H, ctx_total;
  // routed experts (n_experts > 1): routing decisions, the permuted activations, per-slot hidden states and outputs
  size_t idx, gate, probs, counts, offsets, perm, inv, Xp, Hs, Ys;
  // INT8 form of the dense branch: the ctx of pq_hp_int8_* behind the linear's own
  size_t hp8, hp8_bytes;
  // workspace (scratch)
  size_t stat_partials, red_a, red_b, dH, w_Xq, w_gamma, w_H, splitk, splitk2, ws_total;
  size_t dYp, rd, dHs, dXs, dlogit, dwr, hp8_ws, hp8_ws_bytes;
  int n_red_a, n_red_b;
};

struct cursor {
  size_t off = 0;
  size_t take(size_t bytes) {
    size_t o = off;
    off = pq_align_up(off + bytes, 256);
    return o;
  }
};

lin_layout make_layout(const pq_linear_desc& d) {
  lin_layout L;
  memset(&L, 0, sizeof(L));
  const bool routed = d.n_experts > 1 && d.hp_rank > 0;
  const bool hp8 = d.hp_kind == PQ_HP_LOWRANK_INT8 && d.hp_rank > 0;
  // the dense-branch sections (H, dH, the rank-r GEMM plans) are sized for the dense branch only
  const size_t T = d.tokens, K = d.d_in, N = d.d_out, r = (routed || hp8) ? 0 : d.hp_rank, es = esize(d.io_dtype);
  const int engine = d.io_dtype == PQ_BF16 ? 0 : 1;
  cursor c;
  L.mulam = c.take(2 * sizeof(float));
  L.P = c.take(N * K / 8);
  L.Pt = c.take(N * K / 8);
  L.Xq = c.take(T * K);
  L.gamma = c.take(T * sizeof(float));
  L.Xt = c.take(d.io_dtype == PQ_BF16 ? T * K * 2 : 0);
  L.H = c.take(T * r * es);
  const size_t S = T * (size_t)d.top_k, E = d.n_experts, re = d.hp_rank;
  if (routed) {
    L.idx = c.take(S * 4); L.gate = c.take(S * 4); L.probs = c.take(T * E * 4);
    L.counts = c.take(E * 4); L.offsets = c.take((E + 1) * 4); L.perm = c.take(S * 4); L.inv = c.take(S * 4);
    L.Xp = c.take(S * K * 2); L.Hs = c.take(S * re * 2); L.Ys = c.take(S * N * 2);
  }
  if (hp8) {
    L.hp8_bytes = pq_hp_int8_ctx_bytes(d.tokens, d.d_in, d.d_out, d.hp_rank);
    L.hp8 = c.take(L.hp8_bytes);
  }
  L.ctx_total = c.off > 0 ? c.off : 256;
  cursor w;
  L.stat_partials = w.take(2 * sizeof(double) * 1024);
  const int Ti = d.tokens, Ki = d.d_in, Ni = d.d_out, ri = (int)r;
  L.n_red_a = r ? pq_plan_gemm(engine, Ti, ri, Ni).red_blocks : 0;       // dH GEMM
  if (r && pq_skinny_blocks(Ti) > L.n_red_a) L.n_red_a = pq_skinny_blocks(Ti);   // room for the streaming rank-r kernel's partials
  L.n_red_b = pq_plan_gemm(engine, Ni, Ki, Ti).red_blocks;                // dW GEMM
  size_t sk = 0;
  const int shapes[8][3] = {{Ti, ri, Ki}, {Ti, Ni, ri}, {Ti, ri, Ni}, {Ti, Ki, Ni},
                            {Ti, Ki, ri}, {Ni, Ki, Ti}, {Ni, ri, Ti}, {ri, Ki, Ti}};
  for (const auto& sh : shapes) {
    if (sh[0] <= 0 || sh[1] <= 0) continue;
    const size_t b = pq_plan_gemm(engine, sh[0], sh[1], sh[2]).ws_bytes;
    if (b > sk) sk = b;
  }
  if (routed) {
    L.n_red_a = pq_rowdot_blocks((int)S);
    if (8 * S * re * sizeof(float) > sk) sk = 8 * S * re * sizeof(float);   // narrow grouped GEMMs split the contraction up to 8 ways
    // so do the per-expert factor gradients over their slot ranges
    if (pq_mode2_ws_bytes(Ni, (int)re, d.n_experts, (int)S) > sk) sk = pq_mode2_ws_bytes(Ni, (int)re, d.n_experts, (int)S);
    if (pq_mode2_ws_bytes((int)re, Ki, d.n_experts, (int)S) > sk) sk = pq_mode2_ws_bytes((int)re, Ki, d.n_experts, (int)S);
  }
  if (hp8) L.n_red_a = pq_plan_gemm(0, Ti, d.hp_rank, Ni).red_blocks;      // the INT8 branch's dH GEMM leaves the partials of d alpha
  L.red_a = w.take(sizeof(double) * (size_t)(L.n_red_a > 0 ? L.n_red_a : 1));
  L.red_b = w.take(sizeof(double) * (size_t)L.n_red_b);
  L.dH = w.take(T * r * es);
  L.w_Xq = w.take(T * K);          // used when forward runs without a ctx (inference)
  L.w_gamma = w.take(T * sizeof(float));
  L.w_H = w.take(T * r * es);
  L.splitk = w.take(sk);
  // slabs of dA, which shares a launch with dB (whose slabs are in the region above)
  L.splitk2 = w.take((ri > 0 && Ki > 0) ? pq_plan_gemm(engine, ri, Ki, Ti).ws_bytes : 0);
  if (routed) {
    L.dYp = w.take(S * N * 2); L.rd = w.take(S * 4); L.dHs = w.take(S * re * 2); L.dXs = w.take(S * K * 2);
    L.dlogit = w.take(T * E * 4);
    L.dwr = w.take(pq_dwr_scratch_bytes(d.tokens, d.d_in, d.n_experts));
  }
  if (hp8) {
    L.hp8_ws_bytes = pq_hp_int8_workspace_bytes(d.tokens, d.d_in, d.d_out, d.hp_rank);
    L.hp8_ws = w.take(L.hp8_ws_bytes);
  }
  L.ws_total = w.off;
  return L;
}

int check_desc(const pq_linear_desc* d, bool training) {
  PQ_REQUIRE(d != nullptr, PQ_ERR_BAD_ARG, "desc is NULL");
  PQ_REQUIRE(d->tokens >= 0 && d->d_in > 0 && d->d_out > 0 && d->hp_rank >= 0, PQ_ERR_BAD_ARG,
             "negative or zero dimension (tokens=%d d_in=%d d_out=%d hp_rank=%d)", d->tokens, d->d_in,
             d->d_out, d->hp_rank);
  if (int e = check_dtype(d->io_dtype)) return e;
  PQ_REQUIRE(d->w_kind == PQ_W_MASTER || d->w_kind == PQ_W_PACKED, PQ_ERR_BAD_ARG, "unknown w_kind %d", d->w_kind);
  PQ_REQUIRE(d->ste_mode == PQ_STE_IDENTITY || d->ste_mode == PQ_STE_CLIP, PQ_ERR_BAD_ARG, "unknown ste_mode %d", d->ste_mode);
  PQ_REQUIRE(d->d_in % 32 == 0, PQ_ERR_SHAPE, "d_in=%d must be a multiple of 32", d->d_in);
  PQ_REQUIRE(d->d_out % 8 == 0, PQ_ERR_SHAPE, "d_out=%d must be a multiple of 8", d->d_out);
  PQ_REQUIRE(d->hp_rank % 8 == 0, PQ_ERR_SHAPE, "hp_rank=%d must be a multiple of 8", d->hp_rank);
  PQ_REQUIRE(d->n_experts >= 1 && d->n_experts <= 64, PQ_ERR_BAD_ARG, "n_experts=%d must be in 1..64", d->n_experts);
  PQ_REQUIRE(d->top_k >= 1 && d->top_k <= d->n_experts, PQ_ERR_BAD_ARG, "top_k=%d must be in 1..n_experts", d->top_k);
  if (training) {
    PQ_REQUIRE(d->d_out % 32 == 0, PQ_ERR_SHAPE, "training needs d_out=%d to be a multiple of 32", d->d_out);
    PQ_REQUIRE(d->w_kind == PQ_W_MASTER, PQ_ERR_BAD_ARG, "backward needs latent weights (PQ_W_MASTER)");
  }
  PQ_REQUIRE(d->hp_kind == PQ_HP_LOWRANK_BF16 || d->hp_kind == PQ_HP_LOWRANK_INT8, PQ_ERR_BAD_ARG, "unknown hp_kind %d", d->hp_kind);
  if (d->n_experts > 1 && d->hp_rank > 0) {
    PQ_REQUIRE(d->io_dtype == PQ_BF16, PQ_ERR_DTYPE, "routed experts (n_experts=%d) run on bf16 I/O only", d->n_experts);
    PQ_REQUIRE(d->hp_kind == PQ_HP_LOWRANK_BF16, PQ_ERR_BAD_ARG, "routed experts take the 16-bit form of the high-precision branch");
    PQ_REQUIRE(d->d_out % 32 == 0, PQ_ERR_SHAPE, "routed experts need d_out=%d to be a multiple of 32", d->d_out);
  }
  if (d->hp_kind == PQ_HP_LOWRANK_INT8 && d->hp_rank > 0) {
    PQ_REQUIRE(d->io_dtype == PQ_BF16, PQ_ERR_DTYPE, "the INT8 high-precision branch runs on bf16 I/O only");
    PQ_REQUIRE(d->d_out % 32 == 0 && d->hp_rank % 32 == 0, PQ_ERR_SHAPE,
               "the INT8 high-precision branch needs d_out=%d and hp_rank=%d to be multiples of 32", d->d_out, d->hp_rank);
  }
  return PQ_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" int pq_quant_act(const void* X, int32_t dtype, int32_t T, int32_t K, int8_t* Xq, float* gamma,
                            void* stream) {
  if (int e = check_dtype(dtype)) return e;
  PQ_REQUIRE(T >= 0 && K > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d", T, K);
  PQ_REQUIRE(K % 32 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 32", K);
  if (T == 0) return PQ_OK;
  PQ_REQUIRE(X && Xq && gamma, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(Xq), PQ_ERR_SHAPE, "X and Xq must be 16-byte aligned");
  return pq_launch_quant_act(X, dtype, T, K, Xq, gamma, nullptr, (hipStream_t)stream);
}

extern "C" int pq_rmsnorm_quant_fwd(const void* X, const void* gain, int32_t dtype, int32_t T, int32_t K, float eps, void* Xn,
                                    int8_t* Xq, float* gamma, void* Xt, float* rstd, void* stream) {
  if (int e = check_dtype(dtype)) return e;
  PQ_REQUIRE(T >= 0 && K > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d", T, K);
  PQ_REQUIRE(K % 32 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 32", K);
  PQ_REQUIRE(eps >= 0.0f, PQ_ERR_BAD_ARG, "eps must not be negative");
  PQ_REQUIRE(K <= (dtype == PQ_F32 ? 4096 : 8192), PQ_ERR_SHAPE, "K=%d exceeds the row length this call keeps in registers", K);
  if (T == 0) return PQ_OK;
  PQ_REQUIRE(X && gain && Xq && gamma, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(gain) && aligned16(Xq) && aligned16(Xn) && aligned16(Xt), PQ_ERR_SHAPE,
             "buffers must be 16-byte aligned");
  return pq_launch_rmsnorm_quant(X, gain, dtype, T, K, eps, Xn, Xq, gamma, (uint16_t*)Xt, rstd, (hipStream_t)stream);
}

extern "C" size_t pq_rmsnorm_bwd_workspace_bytes(int32_t T, int32_t K) {
  if (T < 0 || K <= 0) return 0;
  return pq_rmsnorm_bwd_scratch_bytes(T, K) + 256;
}

extern "C" int pq_rmsnorm_bwd(const void* dXn, const void* X, const void* gain, const float* rstd, int32_t dtype, int32_t T,
                              int32_t K, void* dX, float* dgain, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_dtype(dtype)) return e;
  PQ_REQUIRE(T >= 0 && K > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d", T, K);
  PQ_REQUIRE(K % 32 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 32", K);
  PQ_REQUIRE(K <= (dtype == PQ_F32 ? 2048 : 4096), PQ_ERR_SHAPE, "K=%d exceeds the row length this call keeps in registers", K);
  PQ_REQUIRE(dgain && gain, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(T == 0 || (dXn && X && rstd && dX), PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(dXn) && aligned16(X) && aligned16(gain) && aligned16(dX), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(workspace_bytes >= pq_rmsnorm_bwd_workspace_bytes(T, K), PQ_ERR_WORKSPACE, "workspace too small");
  PQ_REQUIRE(T == 0 || workspace, PQ_ERR_BAD_ARG, "NULL workspace");
  float* part = (float*)(((uintptr_t)workspace + 255) & ~(uintptr_t)255);
  return pq_launch_rmsnorm_bwd(dXn, X, gain, rstd, dtype, T, K, dX, dgain, part, (hipStream_t)stream);
}

extern "C" size_t pq_rmsnorm_bwd_static_max_bytes(void) { return pq_static_scratch_bytes(); }

extern "C" int pq_rmsnorm_bwd_static(const void* dXn, const void* X, const void* gain, const float* rstd, int32_t dtype, int32_t T,
                                     int32_t K, void* dX, float* dgain, void* stream) {
  if (int e = check_dtype(dtype)) return e;
  PQ_REQUIRE(T >= 0 && K > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d", T, K);
  PQ_REQUIRE(K % 32 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 32", K);
  PQ_REQUIRE(K <= (dtype == PQ_F32 ? 2048 : 4096), PQ_ERR_SHAPE, "K=%d exceeds the row length this call keeps in registers", K);
  PQ_REQUIRE(dgain && gain, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(T == 0 || (dXn && X && rstd && dX), PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(dXn) && aligned16(X) && aligned16(gain) && aligned16(dX), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  const size_t need = pq_rmsnorm_bwd_scratch_bytes(T, K);
  PQ_REQUIRE(need <= pq_static_scratch_bytes(), PQ_ERR_WORKSPACE,
             "T=%d x K=%d needs %zu bytes of partial rows, the static scratch holds %zu: use pq_rmsnorm_bwd with a workspace",
             T, K, need, pq_static_scratch_bytes());
  void* part = nullptr;
  if (int e = pq_static_scratch(&part)) return e;
  return pq_launch_rmsnorm_bwd(dXn, X, gain, rstd, dtype, T, K, dX, dgain, (float*)part, (hipStream_t)stream);
}

extern "C" size_t pq_pack_workspace_bytes(int32_t N, int32_t K) {
  (void)N; (void)K;
  return 2 * sizeof(double) * 1024;
}

extern "C" int pq_pack_sign(const void* W, int32_t w_dtype, int32_t N, int32_t K, uint32_t* packed,
                            uint32_t* packed_t, float* mu_lambda, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (int e = check_dtype(w_dtype)) return e;
  PQ_REQUIRE(N > 0 && K > 0, PQ_ERR_BAD_ARG, "bad size N=%d K=%d", N, K);
  PQ_REQUIRE(K % 4 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 4", K);
  PQ_REQUIRE(((size_t)N * K) % 8 == 0, PQ_ERR_SHAPE, "N*K=%zu must be a multiple of 8", (size_t)N * K);
  PQ_REQUIRE(W && packed && mu_lambda && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(W) && aligned16(workspace), PQ_ERR_SHAPE, "W and workspace must be 16-byte aligned");
  PQ_REQUIRE(workspace_bytes >= pq_pack_workspace_bytes(N, K), PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu",
             workspace_bytes, pq_pack_workspace_bytes(N, K));
  hipStream_t s = (hipStream_t)stream;
  const size_t n = (size_t)N * K;
  const int nb = pq_stats_blocks(n);
  if (int e = pq_launch_wstats_partial(W, w_dtype, n, (double*)workspace, nb, s)) return e;
  return pq_launch_pack(W, w_dtype, N, K, (const double*)workspace, nb, packed, packed_t, mu_lambda, s);
}

extern "C" int pq_router_topk(const void* X, const void* Wr, int32_t dtype, int32_t T, int32_t K, int32_t E,
                              int32_t k, int32_t* idx, float* gate, float* probs, void* stream) {
  if (int e = check_dtype(dtype)) return e;
  PQ_REQUIRE(T >= 0 && K > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d", T, K);
  PQ_REQUIRE(E >= 1 && E <= 64, PQ_ERR_BAD_ARG, "E=%d must be in 1..64", E);
  PQ_REQUIRE(k >= 1 && k <= E, PQ_ERR_BAD_ARG, "k=%d must be in 1..E", k);
  PQ_REQUIRE(K % 8 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 8", K);
  if (T == 0) return PQ_OK;
  PQ_REQUIRE(X && Wr && idx && gate, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(Wr), PQ_ERR_SHAPE, "X and Wr must be 16-byte aligned");
  return pq_launch_router(X, Wr, dtype, T, K, E, k, idx, gate, probs, (hipStream_t)stream);
}

extern "C" int pq_onebit_acc(const int8_t* Xq, const uint32_t* packed, int32_t T, int32_t K, int32_t N,
                             int32_t* acc, void* stream) {
  PQ_REQUIRE(T >= 0 && K > 0 && N > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d N=%d", T, K, N);
  PQ_REQUIRE(K % 32 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 32", K);
  if (T == 0) return PQ_OK;
  PQ_REQUIRE(Xq && packed && acc, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(N % 8 == 0 && aligned16(acc), PQ_ERR_SHAPE, "N=%d must be a multiple of 8 and acc 16-byte aligned", N);
  PQ_REQUIRE(aligned16(Xq) && aligned16(packed), PQ_ERR_SHAPE, "Xq and packed must be 16-byte aligned");
  pq_operand A{Xq, K, PQ_SRC_KC8, nullptr};
  pq_operand B{packed, K / 8, PQ_SRC_BITS8, nullptr};
  pq_epilogue e = epi_zero();
  e.C = acc; e.ldc = N; e.out_kind = PQ_OUT_I32;
  return pq_launch_gemm(0, T, N, K, A, B, e, (hipStream_t)stream);
}

extern "C" size_t pq_linear_ctx_bytes(const pq_linear_desc* d) {
  if (check_desc(d, false) != PQ_OK) return 0;
  return make_layout(*d).ctx_total;
}

extern "C" size_t pq_linear_workspace_bytes(const pq_linear_desc* d) {
  if (check_desc(d, false) != PQ_OK) return 0;
  return make_layout(*d).ws_total;
}

// ---------------------------------------------------------------------------------------------
// Forward: [stats -> pack] -> quantise -> int8 MFMA GEMM with de-quantising epilogue -> hp branch
// ---------------------------------------------------------------------------------------------
// prequant: the quantised activations (codes, gamma, q/gamma) are already in ctx and X is what the
// high-precision branch reads (the normalising entry point runs the fused quantiser first)
static int linear_fwd_impl(const pq_linear_desc* d, const void* X, const void* W_or_packed,
                           const float* mu_lambda, const void* hpA, const void* hpB, const void* Wr, void* Y,
                           void* ctx, size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream, bool prequant) {
  if (int e = check_desc(d, false)) return e;
  const lin_layout L = make_layout(*d);
  const bool routed = d->n_experts > 1 && d->hp_rank > 0;                 // Sec. 3.3: top-k routed low-rank experts
  const bool hp8 = d->hp_kind == PQ_HP_LOWRANK_INT8 && d->hp_rank > 0;    // Sec. 3.2: the branch in its INT8 form
  // r is the rank of the dense 16-bit branch handled inline below; the other two forms run behind the 1-bit GEMM
  const int T = d->tokens, K = d->d_in, N = d->d_out, r = (routed || hp8) ? 0 : d->hp_rank;
  PQ_REQUIRE((d->tokens == 0 || (X && Y)) && W_or_packed && workspace, PQ_ERR_BAD_ARG, "NULL buffer (X, W, Y or workspace)");
  PQ_REQUIRE(d->hp_rank == 0 || (hpA && hpB), PQ_ERR_BAD_ARG, "hp_rank=%d but hpA/hpB is NULL", d->hp_rank);
  PQ_REQUIRE(!routed || Wr, PQ_ERR_BAD_ARG, "n_experts=%d needs the router weights Wr", d->n_experts);
  PQ_REQUIRE(!(routed || hp8) || ctx, PQ_ERR_BAD_ARG, "routed experts and the INT8 high-precision branch need a ctx");
  PQ_REQUIRE(aligned16(Wr), PQ_ERR_SHAPE, "Wr must be 16-byte aligned");
  PQ_REQUIRE(d->w_kind == PQ_W_MASTER || mu_lambda, PQ_ERR_BAD_ARG, "packed weights need mu_lambda");
  PQ_REQUIRE(d->w_kind == PQ_W_PACKED || ctx, PQ_ERR_BAD_ARG, "latent weights need a ctx to hold the packed bits");
  PQ_REQUIRE(aligned16(X) && aligned16(W_or_packed) && aligned16(Y) && aligned16(workspace) && aligned16(ctx) &&
                 aligned16(hpA) && aligned16(hpB), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  PQ_REQUIRE(!ctx || ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  hipStream_t s = (hipStream_t)stream;
  char* cx = (char*)ctx;
  char* ws = (char*)workspace;
  void* sk_ws = ws + L.splitk;
  const bool bf16 = d->io_dtype == PQ_BF16;
  const int engine = bf16 ? 0 : 1;
  const int ok = out_kind_of(d->io_dtype);

  int8_t* Xq = (int8_t*)(ctx ? cx + L.Xq : ws + L.w_Xq);
  float* gamma = (float*)(ctx ? cx + L.gamma : ws + L.w_gamma);
  uint16_t* Xt = (ctx && bf16) ? (uint16_t*)(cx + L.Xt) : nullptr;
  bool quant_done = prequant;
  void* H = r > 0 ? (ctx ? (void*)(cx + L.H) : (void*)(ws + L.w_H)) : nullptr;
  // H = X A^T.  A rank of 128 over many tokens takes the streaming rank-r kernel (whole contraction per workgroup,
  // nothing to reduce); other shapes go through the tile engine, which may split the contraction.
  bool H_skinny = false;
  if (r > 0 && bf16 && T > 0) {
    pq_operand A{X, K, PQ_SRC_KC16, nullptr}, B{hpA, K, PQ_SRC_KC16, nullptr};
    pq_epilogue e = epi_zero();
    e.C = H; e.ldc = r; e.out_kind = ok;
    H_skinny = pq_skinny_applies(T, r, K, A, B, e);
  }
  auto launch_H = [&](bool defer) -> int {
    pq_operand A{X, K, bf16 ? PQ_SRC_KC16 : PQ_SRC_KC32, nullptr};
    pq_operand B{hpA, K, bf16 ? PQ_SRC_KC16 : PQ_SRC_KC32, nullptr};
    pq_epilogue e = epi_zero();
    e.C = H; e.ldc = r; e.out_kind = ok; e.defer_reduce = defer ? 1 : 0;
    if (H_skinny) return pq_launch_skinny(T, K, A, B, e, s, PQP_GEMM_HP_H);
    return pq_launch_gemm(engine, T, r, K, A, B, e, s, PQP_GEMM_HP_H, sk_ws);
  };
  // The weight statistics' first stage and the activation quantiser share a launch (rows of up to 8192 elements stay
  // in registers); when H = X A^T splits its contraction it goes first and the sum of its slabs rides along too.
  const bool combo = d->w_kind == PQ_W_MASTER && bf16 && !prequant && T > 0 && K <= 8192;
  bool H_done = false;
  int H_splits = 0;
  if (combo && r > 0) {
    H_splits = H_skinny ? 1 : pq_plan_gemm(0, T, r, K).splits;
    if (int e = launch_H(H_splits > 1)) return e;
    H_done = true;
  }
  const uint32_t* P;
  const float* mulam;
  if (d->w_kind == PQ_W_MASTER) {
    const size_t n = (size_t)N * K;
    const int nb = pq_stats_blocks(n);
    double* part = (double*)(ws + L.stat_partials);
    if (combo) {
      const bool sum = H_done && H_splits > 1;
      if (int e = pq_launch_wstats_quant(W_or_packed, n, part, nb, X, T, K, Xq, gamma, Xt, s, sum ? (const float*)sk_ws : nullptr, H_splits,
                                         T, r, H, r)) return e;
      quant_done = true;
    } else if (int e = pq_launch_wstats_partial(W_or_packed, d->io_dtype, n, part, nb, s)) return e;
    uint32_t* Pt = (N % 32 == 0) ? (uint32_t*)(cx + L.Pt) : nullptr;
    if (int e = pq_launch_pack(W_or_packed, d->io_dtype, N, K, part, nb, (uint32_t*)(cx + L.P), Pt,
                               (float*)(cx + L.mulam), s)) return e;
    P = (const uint32_t*)(cx + L.P);
    mulam = (const float*)(cx + L.mulam);
  } else {
    P = (const uint32_t*)W_or_packed;
    mulam = mu_lambda;
  }
  if (T == 0) {   // the weight side is still prepared, so a backward with no tokens is well defined
    if (routed)   // ... and empty expert segments are left behind for it
      return pq_launch_route((const int*)(cx + L.idx), 0, d->n_experts, (int*)(cx + L.counts), (int*)(cx + L.offsets),
                             (int*)(cx + L.perm), (int*)(cx + L.inv), s);
    return PQ_OK;
  }

  if (!quant_done)
    if (int e = pq_launch_quant_act(X, d->io_dtype, T, K, Xq, gamma, Xt, s)) return e;

  // bf16 I/O with a live hp branch: the rank-r product H B^T is accumulated into the 1-bit GEMM's tile
  // (the fused form carries beta / alpha through the tile: only while that ratio stays far from the fp32 range, otherwise
  // the two branches are scaled separately as in the Sec. 3.2 sum)
  const bool fuse_hp = bf16 && r > 0 && d->alpha != 0.0f && fabsf(d->alpha) >= 9.5367431640625e-7f * fabsf(d->beta) &&
                       pq_plan_gemm(0, T, N, K, true).splits == 1;
  if (r > 0 && !H_done)
    if (int err = launch_H(false)) return err;
  {  // 1-bit branch: Y = fl32(fl32(beta*lambda)/gamma_t) * acc   [+ alpha * H B^T when fused]
    pq_operand A{Xq, K, PQ_SRC_KC8, nullptr};
    pq_operand B{P, K / 8, PQ_SRC_BITS8, nullptr};
    pq_epilogue e = epi_zero();
    e.C = Y; e.ldc = N; e.out_kind = ok;
    if (fuse_hp) {   // Y = alpha * ( (beta*lambda/alpha/gamma_t) * acc + H B^T )
      pq_phase2 p2;
      p2.A2 = pq_operand{H, r, PQ_SRC_KC16, nullptr};
      p2.B2 = pq_operand{hpB, r, PQ_SRC_KC16, nullptr};
      p2.K2 = r; p2.scale1 = d->beta / d->alpha; p2.dev_scale1 = mulam + 1; p2.row_div1 = gamma;
      e.scale = d->alpha;
      if (int err = pq_launch_gemm(0, T, N, K, A, B, e, s, PQP_GEMM_ONEBIT, sk_ws, nullptr, &p2)) return err;
    } else {
      e.scale = d->beta; e.dev_scale = mulam + 1; e.row_div = gamma;
      if (int err = pq_launch_gemm(0, T, N, K, A, B, e, s, PQP_GEMM_ONEBIT, sk_ws)) return err;
    }
  }
  if (r > 0 && !fuse_hp && d->alpha != 0.0f) {  // Y += alpha * H B^T
    pq_operand A{H, r, bf16 ? PQ_SRC_KC16 : PQ_SRC_KC32, nullptr};
    pq_operand B{hpB, r, bf16 ? PQ_SRC_KC16 : PQ_SRC_KC32, nullptr};
    pq_epilogue e = epi_zero();
    e.C = Y; e.ldc = N; e.out_kind = ok; e.accumulate = 1; e.scale = d->alpha;
    if (int err = pq_launch_gemm(engine, T, N, r, A, B, e, s, PQP_GEMM_HP_Y, sk_ws)) return err;
  }
  if (hp8)   // Y += alpha * B~ Q(A~ Q(x)) on the codes and gamma formed above
    return pq_hp_int8_fwd(Xq, gamma, hpA, hpB, PQ_BF16, T, K, N, d->hp_rank, d->alpha, Y, 1, cx + L.hp8, L.hp8_bytes,
                          ws + L.hp8_ws, L.hp8_ws_bytes, stream);
  if (routed) {
    // router -> stable permutation by expert -> gather -> H_e = X_e A_e^T -> Y_e = H_e B_e^T -> gate-weighted combine
    const int E = d->n_experts, k = d->top_k, S = T * k, re = d->hp_rank;
    int* idx = (int*)(cx + L.idx);
    float* gate = (float*)(cx + L.gate);
    int* offsets = (int*)(cx + L.offsets);
    int* perm = (int*)(cx + L.perm);
    int* inv = (int*)(cx + L.inv);
    if (int e = pq_launch_router(X, Wr, PQ_BF16, T, K, E, k, idx, gate, (float*)(cx + L.probs), s)) return e;
    if (int e = pq_launch_route(idx, S, E, (int*)(cx + L.counts), offsets, perm, inv, s)) return e;
    if (int e = pq_launch_gather_rows(X, perm, k, S, K, cx + L.Xp, s)) return e;
    pq_gemm_group g1{offsets, E, 1, 0, 0, S};
    {
      pq_operand A{cx + L.Xp, K, PQ_SRC_KC16, nullptr};
      pq_operand B{hpA, K, PQ_SRC_KC16, nullptr};
      pq_epilogue e = epi_zero();
      e.C = cx + L.Hs; e.ldc = re; e.out_kind = PQ_OUT_BF16;
      g1.b_stride = (long)re * K;
      if (int err = pq_launch_gemm(0, S, re, K, A, B, e, s, PQP_GEMM_EXPERT, sk_ws, &g1)) return err;
    }
    {
      pq_operand A{cx + L.Hs, re, PQ_SRC_KC16, nullptr};
      pq_operand B{hpB, re, PQ_SRC_KC16, nullptr};
      pq_epilogue e = epi_zero();
      e.C = cx + L.Ys; e.ldc = N; e.out_kind = PQ_OUT_BF16;
      g1.b_stride = (long)N * re;
      if (int err = pq_launch_gemm(0, S, N, re, A, B, e, s, PQP_GEMM_EXPERT, sk_ws, &g1)) return err;
    }
    return pq_launch_combine_fwd(Y, cx + L.Ys, inv, gate, d->alpha, T, k, N, s);
  }
  return PQ_OK;
}

extern "C" int pq_linear_fwd(const pq_linear_desc* d, const void* X, const void* W_or_packed,
                             const float* mu_lambda, const void* hpA, const void* hpB, const void* Wr, void* Y,
                             void* ctx, size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream) {
  return linear_fwd_impl(d, X, W_or_packed, mu_lambda, hpA, hpB, Wr, Y, ctx, ctx_bytes, workspace, workspace_bytes, stream, false);
}

// ---------------------------------------------------------------------------------------------
// STE backward
// ---------------------------------------------------------------------------------------------
// pq_hp_int8_bwd with the per-workgroup partial sums of <dY, Y_hp> (= d alpha) left in red_a when it is not NULL
static int hp_int8_bwd_impl(const void* dY, const void* Xt, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t r, float alpha,
                            const void* ctx, size_t ctx_bytes, void* dX, int32_t accumulate_dX, float* dA, float* dB, void* workspace,
                            size_t workspace_bytes, void* stream, double* red_a);

extern "C" int pq_linear_bwd(const pq_linear_desc* d, const void* dY, const void* X, const void* W,
                             const void* hpA, const void* hpB, const void* Wr, const void* ctx, size_t ctx_bytes,
                             void* dX, float* dW, float* dhpA, float* dhpB, float* dWr, float* dalpha_dbeta,
                             void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_desc(d, true)) return e;
  const lin_layout L = make_layout(*d);
  const bool routed = d->n_experts > 1 && d->hp_rank > 0;
  const bool hp8 = d->hp_kind == PQ_HP_LOWRANK_INT8 && d->hp_rank > 0;
  const int T = d->tokens, K = d->d_in, N = d->d_out, r = (routed || hp8) ? 0 : d->hp_rank;
  PQ_REQUIRE((d->tokens == 0 || (dY && X && dX)) && ctx && dW && dalpha_dbeta && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(d->hp_rank == 0 || (hpA && hpB && dhpA && dhpB), PQ_ERR_BAD_ARG, "hp_rank=%d but an hp buffer is NULL", d->hp_rank);
  PQ_REQUIRE(!routed || (Wr && dWr), PQ_ERR_BAD_ARG, "n_experts=%d needs Wr and dWr", d->n_experts);
  PQ_REQUIRE(aligned16(Wr) && aligned16(dhpA) && aligned16(dhpB), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(d->ste_mode == PQ_STE_IDENTITY || W, PQ_ERR_BAD_ARG, "PQ_STE_CLIP needs the latent W");
  PQ_REQUIRE(aligned16(dY) && aligned16(X) && aligned16(ctx) && aligned16(dX) && aligned16(dW) && aligned16(workspace) &&
                 aligned16(hpA) && aligned16(hpB) && aligned16(W), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  PQ_REQUIRE(ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  hipStream_t s = (hipStream_t)stream;
  const char* cx = (const char*)ctx;
  char* ws = (char*)workspace;
  void* sk_ws = ws + L.splitk;
  const bool bf16 = d->io_dtype == PQ_BF16;
  const int engine = bf16 ? 0 : 1;
  const int ok = out_kind_of(d->io_dtype);
  const int KC = bf16 ? PQ_SRC_KC16 : PQ_SRC_KC32, KS = bf16 ? PQ_SRC_KS16 : PQ_SRC_KS32;
  const float* mulam = (const float*)(cx + L.mulam);
  const float* gamma = (const float*)(cx + L.gamma);
  const void* H = cx + L.H;
  void* dH = ws + L.dH;
  double* red_a = (double*)(ws + L.red_a);
  double* red_b = (double*)(ws + L.red_b);
  int n_red_a = r > 0 ? pq_plan_gemm(engine, T, r, N).red_blocks : 0;   // partial sums of d alpha that the dH GEMM leaves

  if (T > 0 && r > 0) {  // dH = alpha * dY B ; d alpha = <H, dY B>
    pq_operand A{dY, N, KC, nullptr};
    pq_operand B{hpB, r, KS, nullptr};
    pq_epilogue e = epi_zero();
    e.C = dH; e.ldc = r; e.out_kind = ok; e.scale = d->alpha;
    e.dot_comp = H; e.ld_comp = r; e.comp_kind = ok; e.partials = red_a;
    if (engine == 0 && pq_skinny_applies(T, r, N, A, B, e)) {   // many tokens at rank 128: nothing to split or reduce
      n_red_a = pq_skinny_blocks(T);
      if (int err = pq_launch_skinny(T, N, A, B, e, s, PQP_GEMM_DH)) return err;
    } else if (int err = pq_launch_gemm(engine, T, r, N, A, B, e, s, PQP_GEMM_DH, sk_ws)) return err;
  }

  if (T > 0) {  // dX = beta*lambda * dY S  (+ dH A, fused into the same tile for bf16 I/O)
    pq_operand A{dY, N, KC, nullptr};
    pq_operand B{cx + L.Pt, N / 8, bf16 ? PQ_SRC_BITS16 : PQ_SRC_BITSF, nullptr};
    pq_epilogue e = epi_zero();
    e.C = dX; e.ldc = K; e.out_kind = ok;
    const bool fuse = bf16 && r > 0 && pq_plan_gemm(0, T, K, N).splits == 1;
    if (fuse) {
      pq_phase2 p2;
      p2.A2 = pq_operand{dH, r, PQ_SRC_KC16, nullptr};
      p2.B2 = pq_operand{hpA, K, PQ_SRC_KS16, nullptr};
      p2.K2 = r; p2.scale1 = d->beta; p2.dev_scale1 = mulam + 1; p2.row_div1 = nullptr;
      if (int err = pq_launch_gemm(0, T, K, N, A, B, e, s, PQP_GEMM_DX, sk_ws, nullptr, &p2)) return err;
    } else {
      e.scale = d->beta; e.dev_scale = mulam + 1;
      if (int err = pq_launch_gemm(engine, T, K, N, A, B, e, s, PQP_GEMM_DX, sk_ws)) return err;
      if (r > 0) {
        pq_operand A2{dH, r, KC, nullptr};
        pq_operand B2{hpA, K, KS, nullptr};
        pq_epilogue e2 = epi_zero();
        e2.C = dX; e2.ldc = K; e2.out_kind = ok; e2.accumulate = 1;
        if (int err = pq_launch_gemm(engine, T, K, r, A2, B2, e2, s, PQP_GEMM_DX_HP, sk_ws)) return err;
      }
    }
  }
  {  // dW = beta * (dY/gamma)^T q  [masked];  d beta = lambda * sum S .* (dY/gamma)^T q
    pq_operand A{dY, N, KS, nullptr};
    pq_operand B = bf16 ? pq_operand{cx + L.Xt, K, PQ_SRC_KS16, nullptr}
                        : pq_operand{cx + L.Xq, K, PQ_SRC_KS8, gamma};
    pq_epilogue e = epi_zero();
    e.C = dW; e.ldc = K; e.out_kind = PQ_OUT_F32; e.scale = d->beta;
    e.sign_bytes = (const uint8_t*)(cx + L.P); e.ld_sign = K / 8; e.partials = red_b;
    if (d->ste_mode == PQ_STE_CLIP) {
      e.maskW = W; e.mask_kind = ok; e.mu_dev = mulam; e.tau = d->ste_tau;
    }
    if (int err = pq_launch_gemm(engine, N, K, T, A, B, e, s, PQP_GEMM_DW, sk_ws)) return err;
  }
  if (routed) {
    // Sec. 3.3 backward: upstream of expert e's output for slot (t, j) is alpha gate_tj dY_t; the gate itself
    // receives dgate_tj = alpha <dY_t, Y_e(x_t)> and is differentiated through the softmax into Wr and X.
    const int E = d->n_experts, k = d->top_k, S = T * k, re = d->hp_rank;
    const int* idx = (const int*)(cx + L.idx);
    const float* gate = (const float*)(cx + L.gate);
    const int* offsets = (const int*)(cx + L.offsets);
    const int* perm = (const int*)(cx + L.perm);
    const int* inv = (const int*)(cx + L.inv);
    float* rd = (float*)(ws + L.rd);
    n_red_a = S > 0 ? pq_rowdot_blocks(S) : 0;
    if (int e = pq_launch_gather_rows(dY, perm, k, S, N, ws + L.dYp, s)) return e;
    if (int e = pq_launch_rowdot(ws + L.dYp, cx + L.Ys, perm, gate, S, N, rd, red_a, s)) return e;
    if (int e = pq_launch_scale_rows(ws + L.dYp, perm, gate, d->alpha, S, N, s)) return e;   // dYp <- alpha gate dYp
    pq_gemm_group g1{offsets, E, 1, 0, 0, S};
    pq_gemm_group g2{offsets, E, 2, 0, 0, S};
    if (S > 0) {  // dH_e = (alpha gate dY)_e B_e
      pq_operand A{ws + L.dYp, N, PQ_SRC_KC16, nullptr};
      pq_operand B{hpB, re, PQ_SRC_KS16, nullptr};
      pq_epilogue e = epi_zero();
      e.C = ws + L.dHs; e.ldc = re; e.out_kind = PQ_OUT_BF16;
      g1.b_stride = (long)N * re;
      if (int err = pq_launch_gemm(0, S, re, N, A, B, e, s, PQP_GEMM_EXPERT, sk_ws, &g1)) return err;
    }
    {  // per-expert weight gradients: the contraction runs over the expert's slots
      pq_operand A{ws + L.dYp, N, PQ_SRC_KS16, nullptr};
      pq_operand B{cx + L.Hs, re, PQ_SRC_KS16, nullptr};
      pq_epilogue e = epi_zero();
      e.C = dhpB; e.ldc = re; e.out_kind = PQ_OUT_F32;
      g2.c_stride = (long)N * re;
      if (int err = pq_launch_gemm(0, N, re, S, A, B, e, s, PQP_GEMM_EXPERT, sk_ws, &g2)) return err;
      pq_operand A2{ws + L.dHs, re, PQ_SRC_KS16, nullptr};
      pq_operand B2{cx + L.Xp, K, PQ_SRC_KS16, nullptr};
      e.C = dhpA; e.ldc = K;
      g2.c_stride = (long)re * K;
      if (int err = pq_launch_gemm(0, re, K, S, A2, B2, e, s, PQP_GEMM_EXPERT, sk_ws, &g2)) return err;
    }
    if (S > 0) {  // dXs = dH_e A_e (slot order), then scattered back with the router's share
      pq_operand A{ws + L.dHs, re, PQ_SRC_KC16, nullptr};
      pq_operand B{hpA, K, PQ_SRC_KS16, nullptr};
      pq_epilogue e = epi_zero();
      e.C = ws + L.dXs; e.ldc = K; e.out_kind = PQ_OUT_BF16;
      g1.b_stride = (long)re * K;
      if (int err = pq_launch_gemm(0, S, K, re, A, B, e, s, PQP_GEMM_EXPERT, sk_ws, &g1)) return err;
    }
    float* dlogit = (float*)(ws + L.dlogit);
    if (int e = pq_launch_router_bwd(rd, inv, idx, (const float*)(cx + L.probs), d->alpha, T, k, E, dlogit, s)) return e;
    if (int e = pq_launch_dwr(dlogit, X, T, K, E, (float*)(ws + L.dwr), dWr, s)) return e;
    if (int e = pq_launch_combine_bwd(dX, ws + L.dXs, inv, dlogit, Wr, T, k, K, E, s)) return e;
  }
  if (hp8) {   // STE backward of the INT8 branch on the de-quantised factors; its dH GEMM leaves the partials of d alpha
    n_red_a = T > 0 ? pq_plan_gemm(0, T, d->hp_rank, N).red_blocks : 0;
    if (int e = hp_int8_bwd_impl(dY, cx + L.Xt, PQ_BF16, T, K, N, d->hp_rank, d->alpha, cx + L.hp8, L.hp8_bytes, dX, 1, dhpA, dhpB,
                                 ws + L.hp8_ws, L.hp8_ws_bytes, stream, red_a)) return e;
  }
  // d alpha and d beta: both fixed-order sums of per-workgroup partials
  const pq_reduce_job jobs[2] = {{red_a, (T > 0 && (r > 0 || routed || hp8)) ? n_red_a : 0, 1.0f, nullptr, dalpha_dbeta},
                                 {red_b, L.n_red_b, 1.0f, mulam + 1, dalpha_dbeta + 1}};
  bool jobs_done = false;
  if (r > 0 && bf16 && T > 0) {
    // dB = alpha * dY^T H and dA = dH^T X (dH already carries alpha): two narrow GEMMs over the same contraction,
    // one launch when their plans agree; the two scalar reductions then ride along with their split reduction
    pq_operand A0{dY, N, PQ_SRC_KS16, nullptr}, B0{H, r, PQ_SRC_KS16, nullptr};
    pq_operand A1{dH, r, PQ_SRC_KS16, nullptr}, B1{X, K, PQ_SRC_KS16, nullptr};
    if (int err = pq_launch_gemm_pair_ks16(T, N, r, A0, B0, dhpB, r, d->alpha, r, K, A1, B1, dhpA, K, 1.0f, s, PQP_GEMM_DB, PQP_GEMM_DA,
                                           sk_ws, ws + L.splitk2, jobs, &jobs_done)) return err;
  }
  if (!jobs_done)
    if (int err = pq_launch_reduce_partials2(jobs[0].partials, jobs[0].n, 1.0f, nullptr, jobs[0].out, jobs[1].partials, jobs[1].n, 1.0f,
                                             jobs[1].dev_factor, jobs[1].out, s)) return err;
  if (r > 0 && !(bf16 && T > 0)) {
    {  // dB = alpha * dY^T H
      pq_operand A{dY, N, KS, nullptr};
      pq_operand B{H, r, KS, nullptr};
      pq_epilogue e = epi_zero();
      e.C = dhpB; e.ldc = r; e.out_kind = PQ_OUT_F32; e.scale = d->alpha;
      if (int err = pq_launch_gemm(engine, N, r, T, A, B, e, s, PQP_GEMM_DB, sk_ws)) return err;
    }
    {  // dA = dH^T X   (dH already carries alpha)
      pq_operand A{dH, r, KS, nullptr};
      pq_operand B{X, K, KS, nullptr};
      pq_epilogue e = epi_zero();
      e.C = dhpA; e.ldc = K; e.out_kind = PQ_OUT_F32;
      if (int err = pq_launch_gemm(engine, r, K, T, A, B, e, s, PQP_GEMM_DA, sk_ws)) return err;
    }
  }
  return PQ_OK;
}

// ---------------------------------------------------------------------------------------------
// The linear with its normalisation (Sec. 3.1: Y = (lambda/gamma) W Q(Norm(X))): the fused normalising
// quantiser writes codes, gamma and q/gamma straight into the linear's ctx, the high-precision branch reads
// the stored normalised activations, and the backward chains the linear's dX into the normalisation backward.
// ctx = [linear ctx][x_hat T*K][rstd T]; workspace = [linear workspace][d x_hat T*K][dgain partial rows].
// ---------------------------------------------------------------------------------------------
namespace {
struct norm_layout { size_t Xn, rstd, ctx_total, dXn, part, ws_total; };
norm_layout make_norm_layout(const pq_linear_desc& d, const lin_layout& L) {
  norm_layout n;
  const size_t T = d.tokens, K = d.d_in, es = esize(d.io_dtype);
  cursor c; c.off = pq_align_up(L.ctx_total, 256);
  n.Xn = c.take(T * K * es);
  n.rstd = c.take(T * sizeof(float));
  n.ctx_total = c.off;
  cursor w; w.off = pq_align_up(L.ws_total, 256);
  n.dXn = w.take(T * K * es);
  n.part = w.take(pq_rmsnorm_bwd_scratch_bytes(d.tokens, d.d_in) + 256);
  n.ws_total = w.off;
  return n;
}
int check_norm(const pq_linear_desc* d, bool bwd) {
  const int lim = d->io_dtype == PQ_F32 ? (bwd ? 2048 : 4096) : (bwd ? 4096 : 8192);
  PQ_REQUIRE(d->d_in <= lim, PQ_ERR_SHAPE, "d_in=%d exceeds the row length the fused normalisation keeps in registers (%d)", d->d_in, lim);
  return PQ_OK;
}
}  // namespace

extern "C" size_t pq_linear_norm_ctx_bytes(const pq_linear_desc* d) {
  if (check_desc(d, false) != PQ_OK) return 0;
  return make_norm_layout(*d, make_layout(*d)).ctx_total;
}
extern "C" size_t pq_linear_norm_workspace_bytes(const pq_linear_desc* d) {
  if (check_desc(d, false) != PQ_OK) return 0;
  return make_norm_layout(*d, make_layout(*d)).ws_total;
}

extern "C" int pq_linear_norm_fwd(const pq_linear_desc* d, const void* X, const void* gain, float eps, const void* W,
                                  const void* hpA, const void* hpB, const void* Wr, void* Y, void* ctx, size_t ctx_bytes,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_desc(d, false)) return e;
  if (int e = check_norm(d, false)) return e;
  PQ_REQUIRE(d->w_kind == PQ_W_MASTER, PQ_ERR_BAD_ARG, "the normalising entry point takes latent weights");
  PQ_REQUIRE(X && gain && ctx && workspace, PQ_ERR_BAD_ARG, "NULL buffer (X, gain, ctx or workspace)");
  PQ_REQUIRE(eps >= 0.0f, PQ_ERR_BAD_ARG, "eps must not be negative");
  PQ_REQUIRE(aligned16(X) && aligned16(gain) && aligned16(ctx), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  const lin_layout L = make_layout(*d);
  const norm_layout NL = make_norm_layout(*d, L);
  PQ_REQUIRE(ctx_bytes >= NL.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, NL.ctx_total);
  PQ_REQUIRE(workspace_bytes >= NL.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, NL.ws_total);
  char* cx = (char*)ctx;
  const bool bf16 = d->io_dtype == PQ_BF16;
  void* Xn = cx + NL.Xn;
  if (int e = pq_launch_rmsnorm_quant(X, gain, d->io_dtype, d->tokens, d->d_in, eps, Xn, (int8_t*)(cx + L.Xq), (float*)(cx + L.gamma),
                                      bf16 ? (uint16_t*)(cx + L.Xt) : nullptr, (float*)(cx + NL.rstd), (hipStream_t)stream))
    return e;
  return linear_fwd_impl(d, Xn, W, nullptr, hpA, hpB, Wr, Y, ctx, L.ctx_total, workspace, L.ws_total, stream, true);
}

extern "C" int pq_linear_norm_bwd(const pq_linear_desc* d, const void* dY, const void* X, const void* gain, const void* W,
                                  const void* hpA, const void* hpB, const void* Wr, const void* ctx, size_t ctx_bytes, void* dX,
                                  float* dgain, float* dW, float* dhpA, float* dhpB, float* dWr, float* dalpha_dbeta,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_desc(d, true)) return e;
  if (int e = check_norm(d, true)) return e;
  PQ_REQUIRE(X && gain && ctx && dX && dgain && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(gain) && aligned16(dX) && aligned16(workspace), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  const lin_layout L = make_layout(*d);
  const norm_layout NL = make_norm_layout(*d, L);
  PQ_REQUIRE(ctx_bytes >= NL.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, NL.ctx_total);
  PQ_REQUIRE(workspace_bytes >= NL.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, NL.ws_total);
  const char* cx = (const char*)ctx;
  char* ws = (char*)workspace;
  void* dXn = ws + NL.dXn;
  if (int e = pq_linear_bwd(d, dY, cx + NL.Xn, W, hpA, hpB, Wr, ctx, L.ctx_total, dXn, dW, dhpA, dhpB, dWr, dalpha_dbeta, workspace,
                            L.ws_total, stream))
    return e;
  float* part = (float*)(((uintptr_t)(ws + NL.part) + 255) & ~(uintptr_t)255);
  return pq_launch_rmsnorm_bwd(dXn, X, gain, (const float*)(cx + NL.rstd), d->io_dtype, d->tokens, d->d_in, dX, dgain, part,
                               (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// INT8 form of the two-factor high-precision branch (Sec. 3.2): rows of A and B and the hidden state are
// quantised like activations; both products run on the int8 MFMA path with exact int32 accumulation and a
// de-quantising epilogue (row scale as a reciprocal per row, column scale by division).  The backward is the
// STE one: bf16 GEMMs on the de-quantised factors saved by the forward.
// ctx: [Aq r*K][gA r][At r*K bf16][Bq N*r][gB N][Bt N*r bf16][H T*r bf16][Hq T*r][gH T][Ht T*r bf16]
// workspace: [dH T*r bf16][split-contraction slabs]
// ---------------------------------------------------------------------------------------------
namespace {
struct hp8_layout { size_t Aq, gA, At, Bq, gB, Bt, H, Hq, gH, Ht, ctx_total, dH, splitk, splitk2, ws_total; };
hp8_layout make_hp8_layout(int T, int K, int N, int r) {
  hp8_layout L;
  const size_t t = T, k = K, n = N, rr = r;
  cursor c;
  L.Aq = c.take(rr * k); L.gA = c.take(rr * sizeof(float)); L.At = c.take(rr * k * 2);
  L.Bq = c.take(n * rr); L.gB = c.take(n * sizeof(float)); L.Bt = c.take(n * rr * 2);
  L.H = c.take(t * rr * 2); L.Hq = c.take(t * rr); L.gH = c.take(t * sizeof(float)); L.Ht = c.take(t * rr * 2);
  L.ctx_total = c.off;
  cursor w;
  L.dH = w.take(t * rr * 2);
  size_t sk = 0;
  const int shapes[4][3] = {{T, r, N}, {N, r, T}, {r, K, T}, {T, K, r}};
  for (const auto& sh : shapes) {
    if (sh[0] <= 0 || sh[1] <= 0) continue;
    const size_t b = pq_plan_gemm(0, sh[0], sh[1], sh[2]).ws_bytes;
    if (b > sk) sk = b;
  }
  if (T > 0) {   // the int8 H product splits its contraction (int32 slabs)
    const size_t b = pq_plan_gemm(0, T, r, K, true, true).ws_bytes;
    if (b > sk) sk = b;
  }
  L.splitk = w.take(sk);
  L.splitk2 = w.take((r > 0 && K > 0) ? pq_plan_gemm(0, r, K, T).ws_bytes : 0);   // dA's slabs when dB and dA share a launch
  L.ws_total = w.off;
  return L;
}
int check_hp8(int dtype, int T, int K, int N, int r) {
  PQ_REQUIRE(dtype == PQ_BF16, PQ_ERR_DTYPE, "the INT8 high-precision branch takes bf16 tensors");
  PQ_REQUIRE(T >= 0 && K > 0 && N > 0 && r > 0, PQ_ERR_BAD_ARG, "bad size T=%d K=%d N=%d r=%d", T, K, N, r);
  PQ_REQUIRE(K % 32 == 0 && N % 32 == 0 && r % 32 == 0, PQ_ERR_SHAPE, "K=%d, N=%d and r=%d must be multiples of 32", K, N, r);
  return PQ_OK;
}
}  // namespace

extern "C" size_t pq_hp_int8_ctx_bytes(int32_t T, int32_t K, int32_t N, int32_t r) {
  if (check_hp8(PQ_BF16, T, K, N, r) != PQ_OK) return 0;
  return make_hp8_layout(T, K, N, r).ctx_total;
}
extern "C" size_t pq_hp_int8_workspace_bytes(int32_t T, int32_t K, int32_t N, int32_t r) {
  if (check_hp8(PQ_BF16, T, K, N, r) != PQ_OK) return 0;
  return make_hp8_layout(T, K, N, r).ws_total;
}

extern "C" int pq_hp_int8_fwd(const int8_t* Xq, const float* gamma_x, const void* A, const void* B, int32_t dtype, int32_t T,
                              int32_t K, int32_t N, int32_t r, float alpha, void* Y, int32_t accumulate, void* ctx,
                              size_t ctx_bytes, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_hp8(dtype, T, K, N, r)) return e;
  const hp8_layout L = make_hp8_layout(T, K, N, r);
  PQ_REQUIRE(A && B && ctx && workspace, PQ_ERR_BAD_ARG, "NULL buffer (A, B, ctx or workspace)");
  PQ_REQUIRE(T == 0 || (Xq && gamma_x && Y), PQ_ERR_BAD_ARG, "NULL buffer (Xq, gamma_x or Y)");
  PQ_REQUIRE(aligned16(Xq) && aligned16(A) && aligned16(B) && aligned16(Y) && aligned16(ctx) && aligned16(workspace), PQ_ERR_SHAPE,
             "buffers must be 16-byte aligned");
  PQ_REQUIRE(ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  hipStream_t s = (hipStream_t)stream;
  char* cx = (char*)ctx;
  void* sk = (char*)workspace + L.splitk;
  // weight side: rows of A and B on the activation grid (codes, gamma, bf16 de-quantised copy for the backward)
  if (int e = pq_launch_quant_act(A, dtype, r, K, (int8_t*)(cx + L.Aq), (float*)(cx + L.gA), (uint16_t*)(cx + L.At), s)) return e;
  if (int e = pq_launch_quant_act(B, dtype, N, r, (int8_t*)(cx + L.Bq), (float*)(cx + L.gB), (uint16_t*)(cx + L.Bt), s)) return e;
  if (T == 0) return PQ_OK;
  {  // H = (q_x q_a^T) / (gamma_x gamma_a)
    pq_operand a{Xq, K, PQ_SRC_KC8, nullptr};
    pq_operand b{cx + L.Aq, K, PQ_SRC_KC8, nullptr};
    pq_epilogue e = epi_zero();
    e.C = cx + L.H; e.ldc = r; e.out_kind = PQ_OUT_BF16; e.row_div = gamma_x; e.col_div = (const float*)(cx + L.gA);
    e.split_int8 = 1;
    if (int err = pq_launch_gemm(0, T, r, K, a, b, e, s, PQP_GEMM_HP_H, sk)) return err;
  }
  if (int e = pq_launch_quant_act(cx + L.H, dtype, T, r, (int8_t*)(cx + L.Hq), (float*)(cx + L.gH), (uint16_t*)(cx + L.Ht), s)) return e;
  {  // Y (+)= alpha * (q_h q_b^T) / (gamma_h gamma_b)
    pq_operand a{cx + L.Hq, r, PQ_SRC_KC8, nullptr};
    pq_operand b{cx + L.Bq, r, PQ_SRC_KC8, nullptr};
    pq_epilogue e = epi_zero();
    e.C = Y; e.ldc = N; e.out_kind = PQ_OUT_BF16; e.accumulate = accumulate ? 1 : 0; e.scale = alpha;
    e.row_div = (const float*)(cx + L.gH); e.col_div = (const float*)(cx + L.gB);
    if (int err = pq_launch_gemm(0, T, N, r, a, b, e, s, PQP_GEMM_HP_Y, sk)) return err;
  }
  return PQ_OK;
}

extern "C" int pq_hp_int8_bwd(const void* dY, const void* Xt, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t r,
                              float alpha, const void* ctx, size_t ctx_bytes, void* dX, int32_t accumulate_dX, float* dA, float* dB,
                              void* workspace, size_t workspace_bytes, void* stream) {
  return hp_int8_bwd_impl(dY, Xt, dtype, T, K, N, r, alpha, ctx, ctx_bytes, dX, accumulate_dX, dA, dB, workspace, workspace_bytes, stream,
                          nullptr);
}

static int hp_int8_bwd_impl(const void* dY, const void* Xt, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t r, float alpha,
                            const void* ctx, size_t ctx_bytes, void* dX, int32_t accumulate_dX, float* dA, float* dB, void* workspace,
                            size_t workspace_bytes, void* stream, double* red_a) {
  if (int e = check_hp8(dtype, T, K, N, r)) return e;
  const hp8_layout L = make_hp8_layout(T, K, N, r);
  PQ_REQUIRE(ctx && dA && dB && workspace, PQ_ERR_BAD_ARG, "NULL buffer (ctx, dA, dB or workspace)");
  PQ_REQUIRE(T == 0 || (dY && Xt && dX), PQ_ERR_BAD_ARG, "NULL buffer (dY, Xt or dX)");
  PQ_REQUIRE(aligned16(dY) && aligned16(Xt) && aligned16(ctx) && aligned16(dX) && aligned16(dA) && aligned16(dB) && aligned16(workspace),
             PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  PQ_REQUIRE(ctx_bytes >= L.ctx_total, PQ_ERR_WORKSPACE, "ctx too small: %zu < %zu", ctx_bytes, L.ctx_total);
  PQ_REQUIRE(workspace_bytes >= L.ws_total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.ws_total);
  hipStream_t s = (hipStream_t)stream;
  const char* cx = (const char*)ctx;
  char* ws = (char*)workspace;
  void* sk = ws + L.splitk;
  void* dH = ws + L.dH;
  if (T > 0) {  // dH = alpha * dY B~
    pq_operand a{dY, N, PQ_SRC_KC16, nullptr};
    pq_operand b{cx + L.Bt, r, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi_zero();
    e.C = dH; e.ldc = r; e.out_kind = PQ_OUT_BF16; e.scale = alpha;
    if (red_a) {   // sum H~ .* (dY B~) = <dY, H~ B~^T>: the gradient of alpha, one partial per workgroup
      e.dot_comp = cx + L.Ht; e.ld_comp = r; e.comp_kind = PQ_OUT_BF16; e.partials = red_a;
    }
    if (int err = pq_launch_gemm(0, T, r, N, a, b, e, s, PQP_GEMM_DH, sk)) return err;
  }
  {  // dB = alpha * dY^T H~ and dA = dH^T X~ (dH already carries alpha): one launch when their shapes allow it
    pq_operand a0{dY, N, PQ_SRC_KS16, nullptr}, b0{cx + L.Ht, r, PQ_SRC_KS16, nullptr};
    pq_operand a1{dH, r, PQ_SRC_KS16, nullptr}, b1{Xt, K, PQ_SRC_KS16, nullptr};
    if (int err = pq_launch_gemm_pair_ks16(T, N, r, a0, b0, dB, r, alpha, r, K, a1, b1, dA, K, 1.0f, s, PQP_GEMM_DB, PQP_GEMM_DA, sk,
                                           ws + L.splitk2, nullptr, nullptr)) return err;
  }
  if (T > 0) {  // dX (+)= dH A~
    pq_operand a{dH, r, PQ_SRC_KC16, nullptr};
    pq_operand b{cx + L.At, K, PQ_SRC_KS16, nullptr};
    pq_epilogue e = epi_zero();
    e.C = dX; e.ldc = K; e.out_kind = PQ_OUT_BF16; e.accumulate = accumulate_dX ? 1 : 0;
    if (int err = pq_launch_gemm(0, T, K, r, a, b, e, s, PQP_GEMM_DX_HP, sk)) return err;
  }
  return PQ_OK;
}

// ---------------------------------------------------------------------------------------------
// Decode on packed weights
// ---------------------------------------------------------------------------------------------
namespace {
int check_decode(const pq_decode_desc* d) {
  PQ_REQUIRE(d != nullptr, PQ_ERR_BAD_ARG, "desc is NULL");
  PQ_REQUIRE(d->batch >= 1 && d->batch <= 16, PQ_ERR_BAD_ARG, "batch=%d must be in 1..16", d->batch);
  PQ_REQUIRE(d->d_in > 0 && d->d_out > 0 && d->hp_rank >= 0 && d->n_layers >= 1, PQ_ERR_BAD_ARG, "bad dimension");
  PQ_REQUIRE(d->d_out % 4 == 0, PQ_ERR_SHAPE, "d_out=%d must be a multiple of 4", d->d_out);
  PQ_REQUIRE(d->d_in <= 16384, PQ_ERR_SHAPE, "d_in=%d exceeds 16384 (one token's activations are staged in LDS)", d->d_in);
  PQ_REQUIRE(d->packed_layout == PQ_PACKED_ROWMAJOR || d->packed_layout == PQ_PACKED_TILED64, PQ_ERR_BAD_ARG,
             "packed_layout=%d is not a known layout", d->packed_layout);
  const bool tiled = d->packed_layout == PQ_PACKED_TILED64;
  if (d->batch == 1) {
    PQ_REQUIRE(d->d_in % 128 == 0, PQ_ERR_SHAPE, "d_in=%d must be a multiple of 128", d->d_in);
    PQ_REQUIRE(d->hp_rank % 8 == 0, PQ_ERR_SHAPE, "hp_rank=%d must be a multiple of 8", d->hp_rank);
  } else {
    if (tiled) PQ_REQUIRE(d->d_in % 128 == 0, PQ_ERR_SHAPE, "d_in=%d must be a multiple of 128", d->d_in);
    else PQ_REQUIRE(d->d_in % 512 == 0, PQ_ERR_SHAPE, "batch > 1 on the row-major packing needs d_in=%d to be a multiple of 512", d->d_in);
    PQ_REQUIRE(d->hp_rank % 32 == 0, PQ_ERR_SHAPE, "batch > 1 needs hp_rank=%d to be a multiple of 32", d->hp_rank);
  }
  if (d->hp_rank > 0) {
    PQ_REQUIRE(d->n_experts >= 1 && d->n_experts <= 64, PQ_ERR_BAD_ARG, "n_experts=%d must be in 1..64", d->n_experts);
    PQ_REQUIRE(d->top_k >= 1 && d->top_k <= d->n_experts, PQ_ERR_BAD_ARG, "top_k=%d must be in 1..n_experts", d->top_k);
    if (d->batch > 1) PQ_REQUIRE((d->n_experts * d->hp_rank) % 64 == 0, PQ_ERR_SHAPE, "batch > 1 needs n_experts*hp_rank %% 64 == 0");
  }
  if (d->batch > 1) {
    // LDS of the small-batch kernels: 8 or 16 token rows of codes and expert hidden states; on the
    // row-interleaved packing the hidden states share their space with 8 KiB of per-wavefront patches
    const size_t toks = d->batch <= 8 ? 8 : 16;
    const size_t er = d->hp_rank > 0 ? (size_t)d->n_experts * d->hp_rank : 0;
    const size_t hm = 2 * toks * er;
    // (the row-interleaved kernel walks the codes in blocks of 32 KiB)
    const size_t codes = tiled && toks * (size_t)d->d_in > 32768 ? 32768 : toks * (size_t)d->d_in;
    PQ_REQUIRE(codes + ((tiled && hm < 8192) ? 8192 : hm) <= 160 * 1024, PQ_ERR_SHAPE,
               "activations and expert hidden states do not fit the 160 KiB LDS");
  }
  return PQ_OK;
}
}  // namespace

extern "C" size_t pq_decode_workspace_bytes(const pq_decode_desc* d) {
  if (check_decode(d) != PQ_OK) return 0;
  pq_decode_desc dd = *d;
  if (dd.hp_rank == 0) dd.top_k = 0;
  size_t off[7];
  return pq_decode_ws_layout(dd, off);
}

extern "C" int pq_decode_gemv(const pq_decode_desc* d, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                              const void* hpA, const void* hpB, const void* Wr, void* Y, int32_t* acc_out, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (int e = check_decode(d)) return e;
  PQ_REQUIRE(X && packed && scale_fp16 && Y && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(d->hp_rank == 0 || (hpA && hpB && Wr), PQ_ERR_BAD_ARG, "hp_rank=%d but an expert buffer is NULL", d->hp_rank);
  PQ_REQUIRE(aligned16(X) && aligned16(packed) && aligned16(Y) && aligned16(workspace) && aligned16(hpA) && aligned16(hpB) &&
                 aligned16(Wr) && aligned16(acc_out), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  pq_decode_desc dd = *d;
  if (dd.hp_rank == 0) dd.top_k = 0;
  size_t off[7];
  const size_t need = pq_decode_ws_layout(dd, off);
  PQ_REQUIRE(workspace_bytes >= need, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, need);
  return pq_launch_decode(dd, X, packed, scale_fp16, hpA, hpB, Wr, Y, acc_out, workspace, (hipStream_t)stream);
}

extern "C" int pq_decode_gemv_int8(const pq_decode_desc* d, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                                   const int8_t* hpA_q, const float* gamma_A, const int8_t* hpB_q, const float* gamma_B,
                                   const void* Wr, void* Y, int32_t* acc_out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  if (int e = check_decode(d)) return e;
  PQ_REQUIRE(d->hp_rank > 0 && d->hp_rank % 32 == 0, PQ_ERR_SHAPE, "hp_rank=%d must be a positive multiple of 32", d->hp_rank);
  if (d->batch == 1) {
    PQ_REQUIRE(d->top_k <= 8 && d->top_k * d->hp_rank <= 2048, PQ_ERR_SHAPE, "top_k=%d (at most 8) times hp_rank=%d exceeds 2048",
               d->top_k, d->hp_rank);
    PQ_REQUIRE((size_t)d->d_in * 5 <= 64 * 1024, PQ_ERR_SHAPE, "d_in=%d exceeds 13056 (activations and their codes are staged in LDS)", d->d_in);
  } else {
    PQ_REQUIRE(d->packed_layout == PQ_PACKED_TILED64, PQ_ERR_SHAPE, "INT8 experts with batch > 1 need the row-interleaved packing");
    PQ_REQUIRE(d->hp_rank % 64 == 0 && (d->n_experts * d->hp_rank) % 128 == 0, PQ_ERR_SHAPE,
               "INT8 experts with batch > 1 need hp_rank=%d %% 64 == 0 and n_experts * hp_rank %% 128 == 0", d->hp_rank);
    PQ_REQUIRE(d->d_out % 4 == 0, PQ_ERR_SHAPE, "d_out=%d must be a multiple of 4", d->d_out);
  }
  PQ_REQUIRE(X && packed && scale_fp16 && Y && workspace && hpA_q && gamma_A && hpB_q && gamma_B && Wr, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(packed) && aligned16(Y) && aligned16(workspace) && aligned16(hpA_q) && aligned16(hpB_q) &&
                 aligned16(Wr) && aligned16(acc_out), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  size_t off[7];
  const size_t need = pq_decode_ws_layout(*d, off);
  PQ_REQUIRE(workspace_bytes >= need, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, need);
  return pq_launch_decode(*d, X, packed, scale_fp16, hpA_q, hpB_q, Wr, Y, acc_out, workspace, (hipStream_t)stream, gamma_A, gamma_B);
}

// ---------------------------------------------------------------------------------------------
// Decoupled FFN at inference: workspace = [decode workspace of the up/gate stage (rank 2r)][U and G, 2 L F bf16]
// [decode workspace of the down stage]
// ---------------------------------------------------------------------------------------------
namespace {
struct dffn_layout { size_t ws1, UG, ws2, amax, total; };
int check_dffn(const pq_decode_ffn_desc* d) {
  PQ_REQUIRE(d != nullptr, PQ_ERR_BAD_ARG, "desc is NULL");
  PQ_REQUIRE(d->d_model > 0 && d->d_ffn > 0 && d->hp_rank > 0 && d->n_layers >= 1, PQ_ERR_BAD_ARG, "bad dimension");
  PQ_REQUIRE(d->d_model % 128 == 0 && d->d_ffn % 128 == 0, PQ_ERR_SHAPE, "d_model=%d and d_ffn=%d must be multiples of 128", d->d_model, d->d_ffn);
  PQ_REQUIRE(d->d_model <= 16384 && d->d_ffn <= 16384, PQ_ERR_SHAPE, "d_model=%d / d_ffn=%d exceed 16384 (a token's activations are staged in LDS)", d->d_model, d->d_ffn);
  PQ_REQUIRE(d->hp_rank % 8 == 0, PQ_ERR_SHAPE, "hp_rank=%d must be a multiple of 8", d->hp_rank);
  PQ_REQUIRE(d->n_experts >= 1 && d->n_experts <= 64, PQ_ERR_BAD_ARG, "n_experts=%d must be in 1..64", d->n_experts);
  PQ_REQUIRE(d->top_k >= 1 && d->top_k <= d->n_experts, PQ_ERR_BAD_ARG, "top_k=%d must be in 1..n_experts", d->top_k);
  PQ_REQUIRE(d->batch >= 0 && d->batch <= 16, PQ_ERR_BAD_ARG, "batch=%d must be in 1..16 (0 stands for 1)", d->batch);
  if (d->batch > 1) {
    PQ_REQUIRE(d->hp_rank % 32 == 0 && (d->n_experts * d->hp_rank) % 64 == 0, PQ_ERR_SHAPE,
               "batch > 1 needs hp_rank=%d %% 32 == 0 and n_experts * hp_rank %% 64 == 0", d->hp_rank);
    // LDS of the small-batch kernels: a block of the 8 or 16 token rows of codes, and for the down product the expert hidden states
    const size_t toks = d->batch <= 8 ? 8 : 16;
    const size_t hm = 2 * toks * (size_t)d->n_experts * d->hp_rank;
    PQ_REQUIRE(32768 + (hm < 8192 ? 8192 : hm) <= 160 * 1024, PQ_ERR_SHAPE,
               "expert hidden states of %d tokens do not fit the 160 KiB LDS next to a 32 KiB block of codes", d->batch);
  }
  return PQ_OK;
}
dffn_layout make_dffn_layout(const pq_decode_ffn_desc& d) {
  const int B = d.batch > 1 ? d.batch : 1;
  pq_decode_desc d1{B, d.d_model, d.d_ffn, 2 * d.hp_rank, d.n_experts, d.top_k, d.n_layers, PQ_PACKED_TILED64, d.alpha};
  pq_decode_desc d2{B, d.d_ffn, d.d_model, d.hp_rank, d.n_experts, d.top_k, d.n_layers, PQ_PACKED_TILED64, d.alpha};
  size_t off[7];
  dffn_layout L;
  cursor c;
  L.ws1 = c.take(pq_decode_ws_layout(d1, off));
  L.UG = c.take((size_t)2 * d.n_layers * B * d.d_ffn * 2);
  L.ws2 = c.take(pq_decode_ws_layout(d2, off));
  L.amax = c.take((size_t)d.n_layers * B * 8 * sizeof(float));   // the parts' maxima of the gated hidden state
  L.total = c.off;
  return L;
}
}  // namespace

extern "C" size_t pq_decode_ffn_workspace_bytes(const pq_decode_ffn_desc* d) {
  if (check_dffn(d) != PQ_OK) return 0;
  return make_dffn_layout(*d).total;
}

extern "C" int pq_decode_ffn(const pq_decode_ffn_desc* d, const void* X, const uint32_t* packed_upgate, const uint16_t* scale_upgate,
                             const uint32_t* packed_down, const uint16_t* scale_down, const void* UpGate, const void* Down,
                             const void* Wr, void* Y, int32_t* acc_upgate, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = check_dffn(d)) return e;
  PQ_REQUIRE(X && packed_upgate && scale_upgate && packed_down && scale_down && UpGate && Down && Wr && Y && workspace, PQ_ERR_BAD_ARG,
             "NULL buffer");
  PQ_REQUIRE(aligned16(X) && aligned16(packed_upgate) && aligned16(packed_down) && aligned16(UpGate) && aligned16(Down) && aligned16(Wr) &&
                 aligned16(Y) && aligned16(acc_upgate) && aligned16(workspace), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  const dffn_layout L = make_dffn_layout(*d);
  PQ_REQUIRE(workspace_bytes >= L.total, PQ_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, L.total);
  char* ws = (char*)workspace;
  return pq_launch_decode_ffn(d->n_layers, d->batch > 1 ? d->batch : 1, d->d_model, d->d_ffn, d->hp_rank, d->n_experts, d->top_k, d->alpha, X, packed_upgate,
                              scale_upgate, packed_down, scale_down, UpGate, Down, Wr, Y, acc_upgate, ws + L.UG, ws + L.ws1, ws + L.ws2,
                              (float*)(ws + L.amax), (hipStream_t)stream);
}

extern "C" size_t pq_pack_tiled64_bytes(int32_t N, int32_t K) {
  if (N <= 0 || K <= 0 || K % 128 != 0) return 0;
  return (size_t)((N + 63) / 64) * 64 * (K / 32) * sizeof(uint32_t);
}

extern "C" int pq_pack_retile64(const uint32_t* packed, int32_t N, int32_t K, uint32_t* tiled, void* stream) {
  PQ_REQUIRE(N > 0 && K > 0, PQ_ERR_BAD_ARG, "bad size N=%d K=%d", N, K);
  PQ_REQUIRE(K % 128 == 0, PQ_ERR_SHAPE, "K=%d must be a multiple of 128", K);
  PQ_REQUIRE(packed && tiled, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(packed) && aligned16(tiled), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  return pq_launch_retile64(packed, N, K, tiled, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// Glue for chaining linears into a layer stack (not part of the method: residual adds, row gather)
// ---------------------------------------------------------------------------------------------
extern "C" int pq_glue_lincomb(void* out, const void* x0, const void* x1, const void* x2, const void* x3, float c0,
                               float c1, float c2, float c3, size_t n, void* stream) {
  PQ_REQUIRE(out && x0, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(n % 8 == 0, PQ_ERR_SHAPE, "n=%zu must be a multiple of 8", n);
  PQ_REQUIRE(aligned16(out) && aligned16(x0) && aligned16(x1) && aligned16(x2) && aligned16(x3), PQ_ERR_SHAPE,
             "buffers must be 16-byte aligned");
  return pq_launch_lincomb(out, x0, x1, x2, x3, c0, c1, c2, c3, n, (hipStream_t)stream);
}

extern "C" int pq_glue_gather_rows(const void* table, const int32_t* ids, int32_t T, int32_t d, void* out, void* stream) {
  PQ_REQUIRE(T >= 0 && d > 0 && d % 8 == 0, PQ_ERR_SHAPE, "bad shape T=%d d=%d (d must be a multiple of 8)", T, d);
  if (T == 0) return PQ_OK;
  PQ_REQUIRE(table && ids && out, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(aligned16(table) && aligned16(out), PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  return pq_launch_gather_rows(table, ids, 1, T, d, out, (hipStream_t)stream);
}
