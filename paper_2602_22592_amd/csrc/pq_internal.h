// Internal launch interface between the C-ABI layer (pq_api.hip) and the kernel files.
#pragma once
#include "pq_common.h"

// ---- profiling labels (pq_api.hip) ---------------------------------------------------------
enum pq_prof_id {
  PQP_QUANT = 0, PQP_WSTATS, PQP_PACK, PQP_ROUTER, PQP_REDUCE,
  PQP_GEMM_ONEBIT, PQP_GEMM_HP_H, PQP_GEMM_HP_Y, PQP_GEMM_DH, PQP_GEMM_DX, PQP_GEMM_DX_HP,
  PQP_GEMM_DW, PQP_GEMM_DB, PQP_GEMM_DA, PQP_GEMM_OTHER, PQP_DECODE_PREP, PQP_DECODE_H, PQP_DECODE_MAIN, PQP_MOE_ROUTE, PQP_MOE_ELEMENTWISE, PQP_SWIGLU, PQP_GEMM_EXPERT, PQP_GLUE, PQP_SPLITK_REDUCE, PQP_NORM_QUANT, PQP_NORM_BWD, PQP_COUNT
};
struct pq_prof_scope {   // records an event pair around the launches made while it is alive
  int label; hipStream_t s; void* slot;
  pq_prof_scope(int label, hipStream_t s);
  ~pq_prof_scope();
};

// ---- pq_quant.hip -------------------------------------------------------------------------
// Per-token AbsMax INT8 quantiser.  Xt (optional, bf16) receives q/gamma, the de-quantised
// activation that the STE backward multiplies with.
int pq_launch_quant_act(const void* X, int dtype, int T, int K, int8_t* Xq, float* gamma,
                        uint16_t* Xt, hipStream_t s);
// RMSNorm fused with the quantiser: Xn (optional, I/O type) receives the stored normalised activations,
// Xt (optional, bf16) q/gamma, rstd (optional) the per-token reciprocal RMS.  Rows of up to 16*64 16-byte
// vectors (8 for the backward).
int pq_launch_rmsnorm_quant(const void* X, const void* gain, int dtype, int T, int K, float eps, void* Xn, int8_t* Xq,
                            float* gamma, uint16_t* Xt, float* rstd, hipStream_t s);
size_t pq_rmsnorm_bwd_scratch_bytes(int T, int K);
int pq_launch_rmsnorm_bwd(const void* dXn, const void* X, const void* gain, const float* rstd, int dtype, int T, int K, void* dX,
                          float* dgain, float* part, hipStream_t s);
// The library's static device scratch (for entry points that must not allocate): its size, and its address on the
// current device (looked up once per device).
size_t pq_static_scratch_bytes();
int pq_static_scratch(void** out);
// Weight statistics, stage 1: per-block fp64 partial sums {sum W, sum |W|}.
int pq_stats_blocks(size_t n_elems);
// slabs != nullptr: `splits` fp32 slabs [M][N] of a deferred split contraction are summed in slab order into the bf16
// matrix C [M][ldc] by further workgroups of the same launch (N % 8 == 0)
int pq_launch_wstats_quant(const void* W, size_t n_elems, double* partials, int nblocks, const void* X, int T, int K,
                           int8_t* Xq, float* gamma, uint16_t* Xt, hipStream_t s, const float* slabs = nullptr, int splits = 0,
                           int M = 0, int N = 0, void* C = nullptr, int ldc = 0);
int pq_launch_wstats_partial(const void* W, int dtype, size_t n_elems, double* partials, int nblocks,
                             hipStream_t s);
// Stage 2 + binarise + pack (both orientations).  Every block re-reduces the partials in the
// same order, block 0 writes mu_lambda.
int pq_launch_pack(const void* W, int dtype, int N, int K, const double* partials, int nblocks,
                   uint32_t* P, uint32_t* Pt, float* mu_lambda, hipStream_t s);
int pq_launch_router(const void* X, const void* Wr, int dtype, int T, int K, int E, int k, int* idx,
                     float* gate, float* probs, hipStream_t s);
// out[0] = factor * sum(partials[0..n)) (+ optionally factor2 read from device: *dev_factor)
int pq_launch_reduce_partials(const double* partials, int n, float factor, const float* dev_factor,
                              float* out, hipStream_t s);
int pq_launch_reduce_partials2(const double* pa, int na, float fa, const float* dfa, float* oa, const double* pb, int nb, float fb,
                               const float* dfb, float* ob, hipStream_t s);

// ---- pq_gemm.hip --------------------------------------------------------------------------
enum pq_src_kind {
  PQ_SRC_KC16 = 0,   // bf16, contraction index contiguous: elem(row,k) = p[row*ld + k]
  PQ_SRC_KS16 = 1,   // bf16, contraction index strided:   elem(row,k) = p[k*ld + row]
  PQ_SRC_KC8 = 2,    // int8, contraction contiguous
  PQ_SRC_BITS8 = 3,  // +/-1 as int8 from packed bits, ld = bytes per row
  PQ_SRC_BITS16 = 4, // +/-1 as bf16 from packed bits, ld = bytes per row
  // reference-precision engine only:
  PQ_SRC_KC32 = 5,   // fp32, contraction contiguous
  PQ_SRC_KS32 = 6,   // fp32, contraction strided
  PQ_SRC_KS8 = 7,    // int8, contraction strided
  PQ_SRC_BITSF = 8   // +/-1 from packed bits as a real number
};

struct pq_operand {
  const void* p;
  long ld;             // leading dimension in elements (bytes per row for the BITS kinds)
  int kind;
  const float* kdiv;   // optional: divide element by kdiv[k] (per contraction index); ref engine only
};

enum pq_out_kind { PQ_OUT_F32 = 0, PQ_OUT_BF16 = 1, PQ_OUT_I32 = 2 };

struct pq_epilogue {
  void* C;                    // [M][ldc]
  long ldc;
  int out_kind;
  int accumulate;             // C = C + value
  float scale;                // value = scale * acc, or (scale / row_div[m]) * acc
  const float* dev_scale;     // optional device scalar multiplied into `scale` first (fp32 product)
  const float* row_div;       // optional per-row divisor (gamma_t)
  const float* col_div;       // optional per-column divisor applied after the row scale: value / col_div[n]
  int defer_reduce;           // a split contraction leaves its fp32 slabs in the scratch and launches no reduction: the
                              // caller sums them itself (plain epilogues only, see pq_slab_sum_bf16_body)
  int split_int8;             // int8 GEMM: the contraction may be split (int32 slabs summed exactly); callers that set it
                              // size their scratch with pq_plan_gemm(..., int8 = true, split_int8 = true)
  // optional fixed-order partial reductions, one double per block:
  const void* dot_comp;       // sum_{m,n} comp[m][n] * acc   (comp of the io dtype)
  long ld_comp;
  int comp_kind;              // PQ_OUT_F32 / PQ_OUT_BF16
  const uint8_t* sign_bytes;  // sum_{m,n} (+/-1 from bit n of packed row m) * acc
  long ld_sign;               // bytes per packed row
  double* partials;
  // optional STE clipping mask on the stored value: keep iff |W[m][n] - mu| <= tau
  const void* maskW;
  int mask_kind;              // PQ_OUT_F32 / PQ_OUT_BF16
  const float* mu_dev;        // device pointer to mu
  float tau;
  // optional store limits for outputs narrower than the computed tile range (padded widths): rows >= m_limit and
  // columns >= n_limit are computed but not stored (0 = no limit; n_limit % 4 == 0; plain stores only: no
  // accumulate, mask or dot_comp, whose loads would run past a row's end)
  int m_limit, n_limit;
};

// Optional second contraction accumulated into the same output tile (the rank-r branch fused into
// the 1-bit GEMM): after the main contraction acc1, the accumulator becomes
//     acc = (scale1 * [*dev_scale1] / [row_div1[m]]) * acc1 + sum_{k<K2} A2(m,k) * B2(n,k)
// and the epilogue then applies its own scale.  bf16 operands (KC16 x KC16 or KC16 x KS16).
struct pq_phase2 {
  pq_operand A2, B2;
  int K2;                    // 0 = no second contraction
  float scale1;
  const float* dev_scale1;
  const float* row_div1;
};

// C[M][N] (+)= epilogue( sum_k A(m,k) * B(n,k) ).  `engine` 0 = MFMA (bf16 or int8 operands),
// 1 = reference precision (fp64 products and sums on the fp64 MFMA, any operand kind).
// Grouped execution over expert segments (Sec. 3.3): `offsets` [n_groups+1] is a device array of
// slot positions.  mode 1: rows [offsets[e], offsets[e+1]) of A and C belong to group e and use
// B + e*b_stride (elements of B's type) -- the per-expert GEMMs of the forward pass;  mode 2: the
// contraction index runs over [offsets[e], offsets[e+1]) and the result goes to C + e*c_stride
// (elements of C's type) -- the per-expert weight gradients.  max_rows bounds a segment (launch size).
// mode 3: two independent GEMMs of the same operand kinds, tile shape, tile count and contraction in one launch;
// workgroups with blockIdx.z == 1 work on `second` (plain epilogue: C = scale * acc, or raw slabs when split).
struct pq_gemm_second {
  pq_operand A, B;
  void* C;
  int ldc;
  float scale;
  float* part;       // split slabs of the second problem
  int M, N, nbn;
};
struct pq_gemm_group {
  const int* offsets;
  int n_groups;
  int mode;          // 0 = not grouped
  long b_stride;
  long c_stride;
  int max_rows;
  pq_gemm_second second;
  long coldiv_stride;  // mode 1: group e divides its columns by col_div[e * coldiv_stride + n] (per-expert weight-row scales)
};

struct pq_gemm_plan {
  int bm, bn;        // tile
  int splits;        // contraction splits (1 = none)
  int kchunk;        // contraction elements per split
  int red_blocks;    // number of per-block partial sums written when a reduction is requested
  size_t ws_bytes;   // scratch for the split slabs
};
pq_gemm_plan pq_plan_gemm(int engine, int M, int N, int K, bool int8 = false, bool split_int8 = false);
// Scratch a grouped launch over contraction ranges (mode 2; M x N per group, total_k indices over all groups) may use
size_t pq_mode2_ws_bytes(int M, int N, int n_groups, int total_k);
// Two bf16 GEMMs with contraction-strided operands on both sides (the rank-r weight gradients dA and dB) in one
// launch when their plans agree (same tile shape, tile count and contraction split), else one after the other.
// Both have plain epilogues: C (fp32) = scale * acc.
// C[M][128] = scale * A B^T for bf16 operands and many rows (the hidden state of the dense high-precision branch
// and its gradient, Sec. 3.2): one workgroup per 64 rows runs the whole contraction through a six-stage ring of
// direct-to-LDS loads, so nothing is split or reduced.  B is contraction-contiguous or contraction-strided; the
// epilogue may carry dot_comp / partials (one partial sum per workgroup: pq_skinny_blocks(M) of them).
// `applies` states the shapes, alignments and epilogues it takes.
bool pq_skinny_applies(int M, int N, int K, const pq_operand& A, const pq_operand& B, const pq_epilogue& e);
int pq_skinny_blocks(int M);
int pq_launch_skinny(int M, int K, const pq_operand& A, const pq_operand& B, const pq_epilogue& e, hipStream_t s, int prof_label);

int pq_launch_gemm_pair_ks16(int K, int M0, int N0, const pq_operand& A0, const pq_operand& B0, float* C0, int ldc0, float scale0,
                             int M1, int N1, const pq_operand& A1, const pq_operand& B1, float* C1, int ldc1, float scale1,
                             hipStream_t s, int prof_label0, int prof_label1, void* splitk_ws0, void* splitk_ws1,
                             const pq_reduce_job* jobs = nullptr, bool* jobs_done = nullptr);   // jobs: two scalar reductions to ride along
int pq_launch_gemm(int engine, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                   const pq_epilogue& epi, hipStream_t s, int prof_label = PQP_GEMM_OTHER,
                   void* splitk_ws = nullptr, const pq_gemm_group* group = nullptr,
                   const pq_phase2* phase2 = nullptr);

// ---- pq_decode.hip ------------------------------------------------------------------------
size_t pq_decode_ws_layout(const pq_decode_desc& d, size_t* off);
int pq_launch_decode(const pq_decode_desc& d, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                     const void* hpA, const void* hpB, const void* Wr, void* Y, int32_t* acc_out, void* workspace,
                     hipStream_t s, const float* gA = nullptr, const float* gB = nullptr);
int pq_launch_retile64(const uint32_t* packed, int N, int K, uint32_t* tiled, hipStream_t s);
int pq_launch_decode_ffn(int L, int B, int D, int F, int r, int E, int topk, float alpha, const void* X, const uint32_t* packed_upgate,
                         const uint16_t* scale_upgate, const uint32_t* packed_down, const uint16_t* scale_down,
                         const void* UpGate, const void* Down, const void* Wr, void* Y, int32_t* acc_upgate, void* UG,
                         void* ws1, void* ws2, float* amax_part, hipStream_t s);   // amax_part: [L][B][8] floats of scratch

// ---- pq_moe.hip ---------------------------------------------------------------------------
int pq_launch_route(const int* idx, int S, int E, int* counts, int* offsets, int* perm, int* inv, hipStream_t s);
int pq_launch_gather_rows(const void* src, const int* perm, int k, int S, int d, void* dst, hipStream_t s);
// dst[pos] = src[perm[pos] / k]  (fp32 scalars, e.g. a token's gamma carried to its slots)
int pq_launch_gather_f32(const float* src, const int* perm, int k, int S, float* dst, hipStream_t s);
// rows of F elements of which the first Fv exist (padded widths): the rest is written as zero
int pq_launch_swiglu_quant(const void* U, const void* G, int T, int F, int Fv, int8_t* Hq, float* gamma, void* Ht, hipStream_t s);
int pq_launch_swiglu_bwd(const void* dHd, const void* U, const void* G, int T, int F, int Fv, void* dU, void* dG, hipStream_t s);
// ue, ge (and du, dg) have a row stride of ld elements: r, or 2 r when both lie side by side in one [S][2 r] matrix
int pq_launch_expert_act(const void* ue, const void* ge, int ld, int S, int r, void* a, hipStream_t s);
int pq_launch_expert_act_bwd(const void* da, const void* ue, const void* ge, const void* a, const int* perm, const float* gate,
                             float alpha, int S, int r, int ld, void* du, void* dg, void* as, hipStream_t s);
// one expert, top-1: expert 0, gate 1, identity permutation, one segment (what router + counting sort would produce)
int pq_launch_route_single(int S, int* idx, float* gate, float* probs, int* counts, int* offsets, int* perm, int* inv, hipStream_t s);
int pq_launch_zero_f32(float* p, size_t n, hipStream_t s);
// UG[e] = [Up[e]; Gate[e]] (bf16 [E][2 r][d]) and the split of its fp32 gradient back into dUp, dGate
int pq_launch_concat_expert_rows(const void* up, const void* gate_w, int E, int r, int d, void* ug, hipStream_t s);
int pq_launch_split_expert_rows(const float* dug, int E, int r, int d, float* dup, float* dgate, hipStream_t s);
int pq_launch_scale_rows(void* A, const int* perm, const float* gate, float alpha, int S, int d, hipStream_t s);
int pq_rowdot_blocks(int S);
int pq_launch_rowdot(const void* A, const void* B, const int* perm, const float* gate, int S, int d, float* rd, double* partial,
                     hipStream_t s);
int pq_launch_combine_fwd(void* Y, const void* Ys, const int* inv, const float* gate, float alpha, int T, int k, int d, hipStream_t s);
int pq_launch_router_bwd(const float* rd, const int* inv, const int* idx, const float* probs, float alpha, int T, int k, int E,
                         float* dlogit, hipStream_t s);
size_t pq_dwr_scratch_bytes(int T, int d, int E);
int pq_launch_dwr(const float* dlogit, const void* X, int T, int d, int E, float* part, float* dWr, hipStream_t s);
int pq_launch_combine_bwd(void* dX, const void* dXs, const int* inv, const float* dlogit, const void* Wr, int T, int k, int d, int E,
                          hipStream_t s);
int pq_launch_lincomb(void* out, const void* x0, const void* x1, const void* x2, const void* x3, float c0, float c1, float c2,
                      float c3, size_t n, hipStream_t s);
