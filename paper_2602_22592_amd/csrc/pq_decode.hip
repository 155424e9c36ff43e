// Inference on packed 1-bit weights (App. A): the decode product for small token batches.
//
//   y[b][n] = (s / gamma_b) * sum_k q[b][k] * S[n][k]  +  alpha * sum_j gate[b][j] * B_e(A_e x_b),  e = idx[b][j]
//
// with S read from packed bits, s = beta*lambda stored as one fp16 scale, q the INT8 AbsMax codes of
// x_b (Sec. 3.1) and the experts in bf16 (Sec. 3.3, top-k routing).  The packed matrix is the only
// large operand: the kernels stream it through coalesced 16-byte loads exactly once.
//
//   batch 1   bit-plane product: q is split into its 8 two's-complement bit planes (one uint32 per
//             32 columns), so sum_k [S=+1] q_k = sum_p c_p * popcount(bits & plane_p), c_7 = -128;
//             2 VALU ops per (word, plane) with the popcount's built-in accumulate, no multiplies,
//             and sum_k q S = 2 * (that) - sum_k q.  Eight lanes share a row; the planes a lane
//             needs stay in registers for all of its rows.
//   batch >1  int8 MFMA (v_mfma_i32_16x16x64_i8): the weight bits are expanded to {0,-128} bytes in
//             registers (2 VALU ops per 4 weights) once for all tokens, the activations sit in
//             LDS; the same 2*dot - rowsum identity restores the +/-1 product.  Experts run as a
//             dense-masked bf16 MFMA over the experts that some token of the batch selected.
// Several independent layers (weight sets) can be processed by one launch (grid.y), which is how
// the bench keeps the working set larger than the Infinity Cache.
#include <mutex>

#include "pq_internal.h"
#include <type_traits>

namespace {

// streaming 16-byte load: the packed weights are read exactly once, keep them out of the way of the
// small tensors that are re-read (bit planes, expert hidden states)
__device__ __forceinline__ uint4 nt_load16(const uint4* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float fp16_bits_to_f32(uint16_t h) {
  _Float16 x = __builtin_bit_cast(_Float16, h);
  return (float)x;
}

// ------------------------------------------------------------------------------------------
// Prep: quantise (Sec. 3.1), bit planes, row sum, router (Sec. 3.3).  The steps are device functions shared
// by two kernels: one workgroup per (layer, token) doing all of them (any batch), and for batch 1 a fused
// kernel that also produces the expert hidden states so that a decode call is two launches.
// ------------------------------------------------------------------------------------------
struct prep_shared {
  float red[4];
  double dred[4][8];
  float gamma;
  int isum[4];
  double logit[64];
  double expo[64];
  int sel[64];
};

// x -> fp32 in LDS; returns this thread's partial absmax
__device__ __forceinline__ float prep_load_x(const uint16_t* __restrict__ X, size_t tok, int K, float* xs) {
  const int tid = threadIdx.x;
  const uint4* x4 = reinterpret_cast<const uint4*>(X + tok * K);
  float amax = 0.0f;
  // four loads in flight per thread (a load behind a loop-carried wait costs a memory latency each)
  for (int cb = tid; cb < K / 8; cb += 1024) {
    uint4 u4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) u4[i] = x4[min(cb + 256 * i, K / 8 - 1)];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = cb + 256 * i;
      if (c < K / 8) {
        const uint4 u = u4[i];
        const float f[8] = {__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                            __uint_as_float(u.y & 0xFFFF0000u), __uint_as_float(u.z << 16), __uint_as_float(u.z & 0xFFFF0000u),
                            __uint_as_float(u.w << 16), __uint_as_float(u.w & 0xFFFF0000u)};
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(f[j]));
        *reinterpret_cast<float4*>(xs + 8 * c) = make_float4(f[0], f[1], f[2], f[3]);
        *reinterpret_cast<float4*>(xs + 8 * c + 4) = make_float4(f[4], f[5], f[6], f[7]);
      }
    }
  }
  return amax;
}

// INT8 codes, bit planes, row sum and gamma of one token (all threads of the workgroup; xs is complete)
__device__ __forceinline__ void prep_quantise(float amax, size_t tok, int K, const float* xs, prep_shared& sh,
                                              int8_t* __restrict__ xq, uint32_t* __restrict__ planes,
                                              int* __restrict__ rowsum, float* __restrict__ gamma) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  amax = wave_max(amax);
  if (lane == 0) sh.red[wave] = amax;
  __syncthreads();
  if (tid == 0) {
    const float a = fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
    const float g = 128.0f / fmaxf(a, 1e-5f);
    sh.gamma = g;
    gamma[tok] = g;
  }
  __syncthreads();
  const float g = sh.gamma;
  // lane <-> column, a wave-wide ballot per bit plane yields two words
  int isum = 0;
  for (int k0 = wave * 64; k0 < K; k0 += 256) {
    const float y = __fmul_rn(xs[k0 + lane], g);
    const float r = fminf(fmaxf(rintf(y), -128.0f), 127.0f);
    const int q = (int)r;
    // code order inside a 32-column group follows the byte order the small-batch MFMA kernels derive
    // from a weight word: column 8 b + t sits at byte 4 (7 - t) + b
    xq[tok * K + k0 + (lane & 32) + 4 * (7 - (lane & 7)) + ((lane & 31) >> 3)] = (int8_t)q;
    isum += q;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const unsigned long long m = __ballot(((uint32_t)q >> p) & 1u);
      // plane words are grouped per 128 columns: [token][K/128][plane][4 words]
      if (lane < 2) {
        const int wd = (k0 >> 5) + lane;
        planes[((tok * (K / 128) + (wd >> 2)) * 8 + p) * 4 + (wd & 3)] = (uint32_t)(m >> (32 * lane));
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) isum += __shfl_xor(isum, o, 64);
  if (lane == 0) sh.isum[wave] = isum;
  __syncthreads();
  if (tid == 0) rowsum[tok] = sh.isum[0] + sh.isum[1] + sh.isum[2] + sh.isum[3];
}

// The quantiser for a workgroup that holds only its own column groups of a token (group gr of 256 columns belongs to part gr % parts;
// own[256 i + c] is column 256 (part + parts i) + c): codes and bit planes of those columns, gamma by part 0, and the
// row sum as an integer atomic add of the part's share (the caller has it zeroed by an earlier kernel of the call;
// integer sums do not depend on the order).
__device__ __forceinline__ void prep_quantise_own(float amax, size_t tok, int K, const float* own, prep_shared& sh,
                                                  int8_t* __restrict__ xq, uint32_t* __restrict__ planes,
                                                  int* __restrict__ rowsum, float* __restrict__ gamma, int part, int parts) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  amax = wave_max(amax);
  if (lane == 0) sh.red[wave] = amax;
  __syncthreads();
  if (tid == 0) {
    const float a = fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
    const float g = 128.0f / fmaxf(a, 1e-5f);
    sh.gamma = g;
    if (part == 0) gamma[tok] = g;
  }
  __syncthreads();
  const float g = sh.gamma;
  int isum = 0;
  for (int gi = 0;; ++gi) {
    const int k0 = (part + parts * gi) * 256 + wave * 64;
    if (k0 >= K) break;                               // wave-uniform (K % 64 == 0)
    const float y = __fmul_rn(own[gi * 256 + wave * 64 + lane], g);
    const float r = fminf(fmaxf(rintf(y), -128.0f), 127.0f);
    const int q = (int)r;
    isum += q;
    xq[tok * K + k0 + (lane & 32) + 4 * (7 - (lane & 7)) + ((lane & 31) >> 3)] = (int8_t)q;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const unsigned long long m = __ballot(((uint32_t)q >> p) & 1u);
      if (lane < 2) {
        const int wd = (k0 >> 5) + lane;
        planes[((tok * (K / 128) + (wd >> 2)) * 8 + p) * 4 + (wd & 3)] = (uint32_t)(m >> (32 * lane));
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) isum += __shfl_xor(isum, o, 64);
  if (lane == 0) sh.isum[wave] = isum;
  __syncthreads();
  if (tid == 0) atomicAdd(&rowsum[tok], sh.isum[0] + sh.isum[1] + sh.isum[2] + sh.isum[3]);
}

// Router of one token: fp64 logits rounded once to fp32, top-k on logits (ties to the lower index), softmax
// gates over all experts; eight experts per pass over x.  Leaves the selection in sh.sel (valid after the
// closing barrier); when idx is not null it also computes the gates and writes both out.
__device__ __forceinline__ void prep_router(const uint16_t* __restrict__ Wr, int layer, size_t tok, int K, int E, int topk,
                                            const float* xs, prep_shared& sh, int* __restrict__ idx,
                                            float* __restrict__ gate) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int e0 = 0; e0 < E; e0 += 8) {
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int c = tid; c < K / 8; c += 256) {
      // the eight rows are requested together; experts past the end re-read the last one (their sums are dropped)
      uint4 wv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) wv[u] = reinterpret_cast<const uint4*>(Wr + ((size_t)layer * E + min(e0 + u, E - 1)) * K)[c];
      const float4 xa = *reinterpret_cast<const float4*>(xs + 8 * c), xb = *reinterpret_cast<const float4*>(xs + 8 * c + 4);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const uint4 w = wv[u];
        acc[u] += (double)xa.x * (double)__uint_as_float(w.x << 16) + (double)xa.y * (double)__uint_as_float(w.x & 0xFFFF0000u);
        acc[u] += (double)xa.z * (double)__uint_as_float(w.y << 16) + (double)xa.w * (double)__uint_as_float(w.y & 0xFFFF0000u);
        acc[u] += (double)xb.x * (double)__uint_as_float(w.z << 16) + (double)xb.y * (double)__uint_as_float(w.z & 0xFFFF0000u);
        acc[u] += (double)xb.z * (double)__uint_as_float(w.w << 16) + (double)xb.w * (double)__uint_as_float(w.w & 0xFFFF0000u);
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const double t = wave_sum_d(acc[u]);
      if (lane == 0) sh.dred[wave][u] = t;
    }
    __syncthreads();
    if (tid < 8 && e0 + tid < E)
      sh.logit[e0 + tid] = (double)(float)(sh.dred[0][tid] + sh.dred[1][tid] + sh.dred[2][tid] + sh.dred[3][tid]);
  }
  __syncthreads();
  // softmax terms in parallel (one expert per thread), summed in index order by thread 0
  const bool need_gate = idx != nullptr;
  if (need_gate && tid < E) {
    double mx = -1e300;
    for (int e = 0; e < E; ++e) mx = fmax(mx, sh.logit[e]);
    sh.expo[tid] = exp(sh.logit[tid] - mx);
  }
  __syncthreads();
  if (tid == 0) {
    double den = 0.0;
    if (need_gate)
      for (int e = 0; e < E; ++e) den += sh.expo[e];
    unsigned long long taken = 0ull;
    for (int j = 0; j < topk; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e)
        if (!((taken >> e) & 1ull) && (best < 0 || sh.logit[e] > sh.logit[best])) best = e;
      taken |= 1ull << best;
      sh.sel[j] = best;
      if (need_gate) {
        idx[tok * topk + j] = best;
        gate[tok * topk + j] = (float)(sh.expo[best] / den);
      }
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void decode_prep_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wr,
                                                          int B, int K, int E, int topk, int8_t* __restrict__ xq,
                                                          uint32_t* __restrict__ planes, int* __restrict__ rowsum,
                                                          float* __restrict__ gamma, int* __restrict__ idx,
                                                          float* __restrict__ gate, int* __restrict__ zero_rs) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // the token's activations as fp32 [K]
  __shared__ prep_shared sh;
  // two workgroups per token when there is a router: one quantises, the other routes (independent work
  // that would otherwise run back to back inside one workgroup)
  const bool split = E > 0;
  const size_t tok = split ? blockIdx.x >> 1 : blockIdx.x;   // layer * B + b
  const int layer = (int)(tok / B);
  const float amax = prep_load_x(X, tok, K, xs);
  if (!split || (blockIdx.x & 1) == 0) {
    if (zero_rs && threadIdx.x == 0) zero_rs[tok] = 0;   // a row sum that a later kernel of the call adds up with atomics
    prep_quantise(amax, tok, K, xs, sh, xq, planes, rowsum, gamma);
  } else {
    __syncthreads();                                  // xs complete
    prep_router(Wr, layer, tok, K, E, topk, xs, sh, idx, gate);
  }
}

// Batch 1 with experts: workgroup 0 of a layer quantises the token; each of the other workgroups repeats the
// (cheap) router for itself and computes PREP_H_ROWS rows of the selected experts' hidden state
// h = A_e x (bf16 inputs, fp32 accumulate), two rows per wavefront.
#ifndef PQ_PREP_H_ROWS
#define PQ_PREP_H_ROWS 16
#endif
constexpr int PREP_H_ROWS = PQ_PREP_H_ROWS;   // rows per workgroup: few enough workgroups that the repeated router stays cheap

// I8 (Sec. 3.2, experts on the INT8 grid): hpA holds INT8 codes [L][E][r][K] with one gamma per row in gA; the
// hidden state is the exact integer product of the token's codes with a row, de-quantised as
// fl32(fl32(1/gamma_x) * acc) / gamma_a and rounded to bf16 (stored as fp32).  The token's codes (natural column
// order) sit in LDS behind its fp32 activations.
template <bool I8>
__global__ __launch_bounds__(256) void decode_prep_h_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ Wr,
                                                            const void* __restrict__ hpA_, const float* __restrict__ gA,
                                                            int K, int E, int r, int topk,
                                                            int parts, int8_t* __restrict__ xq, uint32_t* __restrict__ planes,
                                                            int* __restrict__ rowsum, float* __restrict__ gamma,
                                                            int* __restrict__ idx, float* __restrict__ gate,
                                                            float* __restrict__ h, int* __restrict__ zero_rs) {
  extern __shared__ __attribute__((aligned(16))) float xs[];
  __shared__ prep_shared sh;
  const uint16_t* __restrict__ hpA = (const uint16_t*)hpA_;
  // Consecutive workgroups go to different XCDs (each with its own L2): number them so that all parts of a
  // layer land on one XCD and its router matrix and activations are fetched from memory once.
  int layer, part;
  {
    const int L = (int)gridDim.x / parts, b = blockIdx.x;
    if ((L & 7) == 0) {
      const int g = b / (8 * parts), rem = b - g * (8 * parts);
      layer = 8 * g + (rem & 7);
      part = rem >> 3;
    } else {
      layer = b / parts;
      part = b - layer * parts;
    }
  }
  const size_t tok = layer;
  const float amax = prep_load_x(X, tok, K, xs);
  if (part == 0) {
    if (zero_rs && threadIdx.x == 0) zero_rs[tok] = 0;   // see decode_prep_kernel
    prep_quantise(amax, tok, K, xs, sh, xq, planes, rowsum, gamma);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gx = 0.0f;
  if constexpr (I8) {                                 // the quantiser's gamma, as prep_quantise forms it
    const float wm = wave_max(amax);
    if (lane == 0) sh.red[wave] = wm;
  }
  __syncthreads();                                    // xs complete
  if constexpr (I8) gx = 128.0f / fmaxf(fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3])), 1e-5f);
  prep_router(Wr, layer, tok, K, E, topk, xs, sh, part == 1 ? idx : nullptr, gate);
  const int oend = min(part * PREP_H_ROWS, topk * r);
  if constexpr (I8) {
    uint32_t* xc = reinterpret_cast<uint32_t*>(xs + K);          // K code bytes
    for (int c = threadIdx.x; c < K / 4; c += 256) {
      const float4 v = *reinterpret_cast<const float4*>(xs + 4 * c);
      const float f[4] = {v.x, v.y, v.z, v.w};
      uint32_t w = 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int q = (int)fminf(fmaxf(rintf(__fmul_rn(f[j], gx)), -128.0f), 127.0f);
        w |= (uint32_t)(q & 0xFF) << (8 * j);
      }
      xc[c] = w;
    }
    __syncthreads();
    const int8_t* __restrict__ A8 = (const int8_t*)hpA_;
    const float sx = 1.0f / gx;
    for (int o0 = (part - 1) * PREP_H_ROWS + 2 * wave; o0 < oend; o0 += 8) {
      const bool two = o0 + 1 < oend;
      const int o1 = two ? o0 + 1 : o0;
      const size_t row0 = ((size_t)layer * E + sh.sel[o0 / r]) * r + o0 % r;
      const size_t row1 = ((size_t)layer * E + sh.sel[o1 / r]) * r + o1 % r;
      const uint4* a0 = reinterpret_cast<const uint4*>(A8 + row0 * K);
      const uint4* a1 = reinterpret_cast<const uint4*>(A8 + row1 * K);
      int s0 = 0, s1 = 0;
      for (int cb = lane; cb < K / 16; cb += 256) {     // eight loads in flight per lane
        uint4 ua[4], va[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int cc = min(cb + 64 * i, K / 16 - 1);
          ua[i] = nt_load16(a0 + cc);
          va[i] = nt_load16(a1 + cc);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int c = cb + 64 * i;
          if (c < K / 16) {
            const uint4 q = *reinterpret_cast<const uint4*>(xc + 4 * c);
            s0 = __builtin_amdgcn_sdot4((int)ua[i].x, (int)q.x, s0, false);
            s0 = __builtin_amdgcn_sdot4((int)ua[i].y, (int)q.y, s0, false);
            s0 = __builtin_amdgcn_sdot4((int)ua[i].z, (int)q.z, s0, false);
            s0 = __builtin_amdgcn_sdot4((int)ua[i].w, (int)q.w, s0, false);
            s1 = __builtin_amdgcn_sdot4((int)va[i].x, (int)q.x, s1, false);
            s1 = __builtin_amdgcn_sdot4((int)va[i].y, (int)q.y, s1, false);
            s1 = __builtin_amdgcn_sdot4((int)va[i].z, (int)q.z, s1, false);
            s1 = __builtin_amdgcn_sdot4((int)va[i].w, (int)q.w, s1, false);
          }
        }
      }
      s0 = wave_sum_i(s0);
      s1 = wave_sum_i(s1);
      if (lane == 0) {
        h[(size_t)layer * topk * r + o0] = bf16_to_f32(f32_to_bf16(__fmul_rn(sx, (float)s0) / gA[row0]));
        if (two) h[(size_t)layer * topk * r + o1] = bf16_to_f32(f32_to_bf16(__fmul_rn(sx, (float)s1) / gA[row1]));
      }
    }
    return;
  }
  for (int o0 = (part - 1) * PREP_H_ROWS + 2 * wave; o0 < oend; o0 += 8) {   // rows of the [topk][r] hidden state
    const bool two = o0 + 1 < oend;
    const int o1 = two ? o0 + 1 : o0;
    const uint4* a0 = reinterpret_cast<const uint4*>(hpA + (((size_t)layer * E + sh.sel[o0 / r]) * r + o0 % r) * K);
    const uint4* a1 = reinterpret_cast<const uint4*>(hpA + (((size_t)layer * E + sh.sel[o1 / r]) * r + o1 % r) * K);
    float s0 = 0.0f, s1 = 0.0f;
    for (int cb = lane; cb < K / 8; cb += 256) {       // eight loads in flight per lane
      uint4 ua[4], va[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int cc = min(cb + 64 * i, K / 8 - 1);
        ua[i] = nt_load16(a0 + cc);
        va[i] = nt_load16(a1 + cc);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = cb + 64 * i;
        if (c < K / 8) {
          const uint4 u = ua[i], v = va[i];
          const float4 xa = *reinterpret_cast<const float4*>(xs + 8 * c), xb = *reinterpret_cast<const float4*>(xs + 8 * c + 4);
          s0 += __uint_as_float(u.x << 16) * xa.x + __uint_as_float(u.x & 0xFFFF0000u) * xa.y;
          s0 += __uint_as_float(u.y << 16) * xa.z + __uint_as_float(u.y & 0xFFFF0000u) * xa.w;
          s0 += __uint_as_float(u.z << 16) * xb.x + __uint_as_float(u.z & 0xFFFF0000u) * xb.y;
          s0 += __uint_as_float(u.w << 16) * xb.z + __uint_as_float(u.w & 0xFFFF0000u) * xb.w;
          s1 += __uint_as_float(v.x << 16) * xa.x + __uint_as_float(v.x & 0xFFFF0000u) * xa.y;
          s1 += __uint_as_float(v.y << 16) * xa.z + __uint_as_float(v.y & 0xFFFF0000u) * xa.w;
          s1 += __uint_as_float(v.z << 16) * xb.x + __uint_as_float(v.z & 0xFFFF0000u) * xb.y;
          s1 += __uint_as_float(v.w << 16) * xb.z + __uint_as_float(v.w & 0xFFFF0000u) * xb.w;
        }
      }
    }
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    if (lane == 0) {
      h[(size_t)layer * topk * r + o0] = s0;
      if (two) h[(size_t)layer * topk * r + o1] = s1;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Expert hidden state: one wavefront per (layer, token, slot, r): h = A_e[r,:] . x   (bf16 in, fp32 out)
// ------------------------------------------------------------------------------------------
// INT8 experts: hpA holds INT8 codes with one gamma per row (gA).  One workgroup per (layer, expert, group of 16
// rows); its four wavefronts share out the tokens of the layer that selected the expert (found by scanning the
// layer's index list), so the 16 rows are fetched from memory once however many tokens use them.  Per token the
// codes are formed once per 4096 columns from x and its gamma (the quantiser's arithmetic) and kept in
// registers for the 16 rows; the products are exact integers, de-quantised as
// fl32(fl32(1/gamma_x) * acc) / gamma_a and rounded to bf16 (held as fp32).  Columns past the end carry zero
// codes and re-read the last chunk, so no load sits behind a branch.
constexpr int H8_ROWS = 16;
__device__ __forceinline__ void h_int8_slot(const uint16_t* __restrict__ X, const int8_t* __restrict__ A8,
                                            const float* __restrict__ gA, const float* __restrict__ gamma, int K, int r,
                                            int slot, int tok, size_t arow0, int rg, float* __restrict__ h) {
  const int lane = threadIdx.x & 63;
  const uint4* x4 = reinterpret_cast<const uint4*>(X + (size_t)tok * K);
  const float gx = gamma[tok];
  const int nch = K / 16;
  int acc[H8_ROWS];
#pragma unroll
  for (int rr = 0; rr < H8_ROWS; ++rr) acc[rr] = 0;
  for (int c0 = 0; c0 < nch; c0 += 256) {
    uint32_t xw[4][4];
    int cc[4];
    uint4 xv[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      cc[i] = min(c0 + lane + 64 * i, nch - 1);
      xv[2 * i] = x4[2 * cc[i]];
      xv[2 * i + 1] = x4[2 * cc[i] + 1];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = c0 + lane + 64 * i < nch;
      const uint32_t w8[8] = {xv[2 * i].x, xv[2 * i].y, xv[2 * i].z, xv[2 * i].w, xv[2 * i + 1].x, xv[2 * i + 1].y, xv[2 * i + 1].z, xv[2 * i + 1].w};
#pragma unroll
      for (int d = 0; d < 4; ++d) {                    // four codes per word: columns 4 d .. 4 d + 3 of the chunk
        const float f[4] = {__uint_as_float(w8[2 * d] << 16), __uint_as_float(w8[2 * d] & 0xFFFF0000u),
                            __uint_as_float(w8[2 * d + 1] << 16), __uint_as_float(w8[2 * d + 1] & 0xFFFF0000u)};
        uint32_t w = 0u;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int q = (int)fminf(fmaxf(rintf(__fmul_rn(f[t], gx)), -128.0f), 127.0f);
          w |= (uint32_t)(q & 0xFF) << (8 * t);
        }
        xw[i][d] = ok ? w : 0u;
      }
    }
#pragma unroll 4
    for (int rr = 0; rr < H8_ROWS; ++rr) {
      const uint4* a4 = reinterpret_cast<const uint4*>(A8 + (arow0 + rr) * K);
      uint4 av[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = a4[cc[i]];        // cached: the other wavefronts of the workgroup read the same rows
      int a = acc[rr];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a = __builtin_amdgcn_sdot4((int)av[i].x, (int)xw[i][0], a, false);
        a = __builtin_amdgcn_sdot4((int)av[i].y, (int)xw[i][1], a, false);
        a = __builtin_amdgcn_sdot4((int)av[i].z, (int)xw[i][2], a, false);
        a = __builtin_amdgcn_sdot4((int)av[i].w, (int)xw[i][3], a, false);
      }
      acc[rr] = a;
    }
  }
  const float sx = 1.0f / gx;
#pragma unroll
  for (int rr = 0; rr < H8_ROWS; ++rr) {
    const int t = wave_sum_i(acc[rr]);
    if (lane == 0) h[(size_t)slot * r + rg * H8_ROWS + rr] = bf16_to_f32(f32_to_bf16(__fmul_rn(sx, (float)t) / gA[arow0 + rr]));
  }
}

__global__ __launch_bounds__(256) void decode_h_int8_kernel(const uint16_t* __restrict__ X, const int8_t* __restrict__ A8,
                                                            const float* __restrict__ gA, const float* __restrict__ gamma,
                                                            const int* __restrict__ idx, int B, int K, int E, int r, int topk,
                                                            float* __restrict__ h) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ngrp = r / H8_ROWS;
  const int rg = blockIdx.x % ngrp, le = blockIdx.x / ngrp;    // le = layer * E + e
  const int layer = le / E, e = le - layer * E;
  const int nslot = B * topk;
  const int* lidx = idx + (size_t)layer * nslot;
  const size_t arow0 = (size_t)le * r + (size_t)rg * H8_ROWS;
  int cnt = 0;
  for (int sl = 0; sl < nslot; ++sl) {                // uniform scan: the cnt-th user of this expert goes to wave cnt % 4
    if (lidx[sl] != e) continue;
    if ((cnt & 3) == wave) h_int8_slot(X, A8, gA, gamma, K, r, layer * nslot + sl, layer * B + sl / topk, arow0, rg, h);
    ++cnt;
  }
}

__global__ __launch_bounds__(256) void decode_h_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ hpA,
                                                       const int* __restrict__ idx, int B, int K, int E, int r, int topk,
                                                       int total, float* __restrict__ h) {
  const int lane = threadIdx.x & 63;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);   // ((layer*B + b)*topk + j)*r + rr
  if (o >= total) return;
  const int rr = o % r, slot = o / r;
  const int tok = slot / topk, layer = tok / B;
  const int e = idx[slot];
  const uint4* a4 = reinterpret_cast<const uint4*>(hpA + (((size_t)layer * E + e) * r + rr) * K);
  const uint4* x4 = reinterpret_cast<const uint4*>(X + (size_t)tok * K);
  float acc = 0.0f;
  for (int cb = lane; cb < K / 8; cb += 512) {         // sixteen loads in flight per lane
    uint4 av[8], xv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int cc = min(cb + 64 * i, K / 8 - 1);
      av[i] = a4[cc];
      xv[i] = x4[cc];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (cb + 64 * i < K / 8) {
        const uint4 a = av[i], x = xv[i];
        acc += __uint_as_float(a.x << 16) * __uint_as_float(x.x << 16) + __uint_as_float(a.x & 0xFFFF0000u) * __uint_as_float(x.x & 0xFFFF0000u);
        acc += __uint_as_float(a.y << 16) * __uint_as_float(x.y << 16) + __uint_as_float(a.y & 0xFFFF0000u) * __uint_as_float(x.y & 0xFFFF0000u);
        acc += __uint_as_float(a.z << 16) * __uint_as_float(x.z << 16) + __uint_as_float(a.z & 0xFFFF0000u) * __uint_as_float(x.z & 0xFFFF0000u);
        acc += __uint_as_float(a.w << 16) * __uint_as_float(x.w << 16) + __uint_as_float(a.w & 0xFFFF0000u) * __uint_as_float(x.w & 0xFFFF0000u);
      }
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) h[o] = acc;
}

// The same hidden states computed expert by expert (K = 512 NV <= 4096, at most 64 slots per layer): a workgroup owns
// HG_ROWS rows of one expert of one layer, a wavefront two of them, held packed in registers (a row of 4096 bf16 is
// eight 16-byte pieces per lane); every token of the batch that selected the expert is then run against them, so an
// expert's rows are read from memory once instead of once per selecting token.  The layer's selections are fetched with
// one vector load and turned into a mask of the expert's slots (a scan with scalar loads is a chain of memory latencies);
// workgroups of experts nobody selected return at once.  Per (slot, row) the sum runs in the order of decode_h_kernel.
constexpr int HG_ROWS = 8;
template <int NV>
__global__ __launch_bounds__(256) void decode_h_grouped_kernel(const uint16_t* __restrict__ X, const uint16_t* __restrict__ hpA,
                                                               const int* __restrict__ idx, int B, int E, int r, int topk,
                                                               float* __restrict__ h) {
  constexpr int K = 512 * NV;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ngrp = r / HG_ROWS;
  const int rg = blockIdx.x % ngrp, le = blockIdx.x / ngrp;    // le = layer * E + e
  const int layer = le / E, e = le - layer * E;
  const int nslot = B * topk;
  const int sel = lane < nslot ? idx[(size_t)layer * nslot + lane] : -1;
  unsigned long long users = __ballot(sel == e);
  if (users == 0ull) return;
  const int r0 = rg * HG_ROWS + 2 * wave;
  const uint4* a0 = reinterpret_cast<const uint4*>(hpA + ((size_t)le * r + r0) * K) + lane;
  const uint4* a1 = a0 + K / 8;
  uint4 av0[NV], av1[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    av0[i] = nt_load16(a0 + 64 * i);
    av1[i] = nt_load16(a1 + 64 * i);
  }
  while (users) {
    const int sl = __builtin_ctzll(users);
    users &= users - 1ull;
    const uint4* x4 = reinterpret_cast<const uint4*>(X + ((size_t)layer * B + sl / topk) * K) + lane;
    uint4 xv[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) xv[i] = x4[64 * i];
    float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      // (the rows stay packed: without this the unpacked halves are hoisted out of the loop and held in 128 more registers)
      asm volatile("" : "+v"(av0[i].x), "+v"(av0[i].y), "+v"(av0[i].z), "+v"(av0[i].w), "+v"(av1[i].x), "+v"(av1[i].y), "+v"(av1[i].z), "+v"(av1[i].w));
      const uint4 x = xv[i], a = av0[i], b = av1[i];
      s0 += __uint_as_float(a.x << 16) * __uint_as_float(x.x << 16) + __uint_as_float(a.x & 0xFFFF0000u) * __uint_as_float(x.x & 0xFFFF0000u);
      s0 += __uint_as_float(a.y << 16) * __uint_as_float(x.y << 16) + __uint_as_float(a.y & 0xFFFF0000u) * __uint_as_float(x.y & 0xFFFF0000u);
      s0 += __uint_as_float(a.z << 16) * __uint_as_float(x.z << 16) + __uint_as_float(a.z & 0xFFFF0000u) * __uint_as_float(x.z & 0xFFFF0000u);
      s0 += __uint_as_float(a.w << 16) * __uint_as_float(x.w << 16) + __uint_as_float(a.w & 0xFFFF0000u) * __uint_as_float(x.w & 0xFFFF0000u);
      s1 += __uint_as_float(b.x << 16) * __uint_as_float(x.x << 16) + __uint_as_float(b.x & 0xFFFF0000u) * __uint_as_float(x.x & 0xFFFF0000u);
      s1 += __uint_as_float(b.y << 16) * __uint_as_float(x.y << 16) + __uint_as_float(b.y & 0xFFFF0000u) * __uint_as_float(x.y & 0xFFFF0000u);
      s1 += __uint_as_float(b.z << 16) * __uint_as_float(x.z << 16) + __uint_as_float(b.z & 0xFFFF0000u) * __uint_as_float(x.z & 0xFFFF0000u);
      s1 += __uint_as_float(b.w << 16) * __uint_as_float(x.w << 16) + __uint_as_float(b.w & 0xFFFF0000u) * __uint_as_float(x.w & 0xFFFF0000u);
    }
    s0 = wave_sum(s0);
    s1 = wave_sum(s1);
    if (lane == 0) {
      float* hs = h + ((size_t)layer * nslot + sl) * r + r0;
      hs[0] = s0;
      hs[1] = s1;
    }
  }
}

// launches the expert-grouped kernel when the shape allows it (then returns true)
static bool launch_h_grouped(const uint16_t* X, const uint16_t* A, const int* idx, int L, int B, int K, int E, int r, int topk, float* h,
                             hipStream_t s) {
  if (r % HG_ROWS != 0 || B * topk > 64) return false;
  const dim3 grid(L * E * (r / HG_ROWS)), block(256);
  if (K == 4096) decode_h_grouped_kernel<8><<<grid, block, 0, s>>>(X, A, idx, B, E, r, topk, h);
  else if (K == 2048) decode_h_grouped_kernel<4><<<grid, block, 0, s>>>(X, A, idx, B, E, r, topk, h);
  else if (K == 1024) decode_h_grouped_kernel<2><<<grid, block, 0, s>>>(X, A, idx, B, E, r, topk, h);
  else if (K == 512) decode_h_grouped_kernel<1><<<grid, block, 0, s>>>(X, A, idx, B, E, r, topk, h);
  else return false;
  return true;
}

// ------------------------------------------------------------------------------------------
// Batch 1: bit-plane GEMV.  A wavefront owns ROWS_PER_WAVE consecutive rows; 8 lanes share a row.
// In step i a lane holds words 32 i + 4 (lane % 8) + {0..3} of its row, so the 8 lanes of a row read
// 128 contiguous bytes per load instruction.
// ------------------------------------------------------------------------------------------
constexpr int GEMV_ITERS = 8;                       // 8 rows per iteration -> 64 rows per wavefront
constexpr int GEMV_ROWS_PER_WAVE = 8 * GEMV_ITERS;
constexpr int GEMV_ROWS_PER_BLOCK = 4 * GEMV_ROWS_PER_WAVE;

struct gemv_params {
  const uint32_t* P;      // [L][N][K/32]
  const uint16_t* scale;  // [L] fp16 bits
  const uint32_t* planes; // [L][K/128][8][4]: the 8 planes of 128 columns are 128 contiguous bytes
  const int* rowsum;      // [L]
  const float* gamma;     // [L]
  const uint16_t* hpB;    // [L][E][N][r] bf16
  const int* idx;         // [L][topk]
  const float* gate;      // [L][topk]
  const float* h;         // [L][topk][r]
  uint16_t* Y;            // [L][N] bf16
  int* acc_out;           // [L][N] or null
  int N, K, E, r, topk;
  float alpha;
  const float* gB;        // INT8 experts: [L][E][N] gammas of the rows of hpB (then hpB is int8 [L][E][N][r])
  int xshare;             // > 1: that many consecutive weight sets read the same token (planes, row sum, gamma of set / xshare)
};

// INT8 experts: the hidden state of every selected expert (bf16 values held as fp32) is put on the INT8 grid
// again (Sec. 3.1 quantiser, one gamma per token and expert) by each wavefront for itself: codes to a
// wave-private LDS patch qh[topk][r/4] (4 codes per word), gammas to gh[topk].  topk <= 8, topk * r <= 2048.
constexpr int I8_MAX_TOPK = 8, I8_MAX_CODE_WORDS = 512;
__device__ __forceinline__ void expert_codes_wave(const float* __restrict__ hh, int topk, int r, uint32_t* qh, float* gh) {
  const int lane = threadIdx.x & 63;
  for (int j = 0; j < topk; ++j) {
    const float* hj = hh + (size_t)j * r;
    float amax = 0.0f;
    for (int d = lane; d < r / 4; d += 64) {
      const float4 v = *reinterpret_cast<const float4*>(hj + 4 * d);
      amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
    amax = wave_max(amax);
    const float g = 128.0f / fmaxf(amax, 1e-5f);
    for (int d = lane; d < r / 4; d += 64) {
      const float4 v = *reinterpret_cast<const float4*>(hj + 4 * d);
      const float f[4] = {v.x, v.y, v.z, v.w};
      uint32_t w = 0u;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int q = (int)fminf(fmaxf(rintf(__fmul_rn(f[t], g)), -128.0f), 127.0f);
        w |= (uint32_t)(q & 0xFF) << (8 * t);
      }
      qh[j * (r / 4) + d] = w;
    }
    if (lane == 0) gh[j] = g;
  }
  // wave-private patch: order this wave's LDS writes before its reads of other lanes' words
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One row of one selected expert against the token's hidden-state codes: this lane's share (16-byte chunks
// sub, sub + 8, ... of the row's r codes) of the exact integer product
__device__ __forceinline__ int expert_dot_i8(const int8_t* __restrict__ brow, const uint32_t* qhj, int r, int sub) {
  int part = 0;
  for (int c = sub; c < r / 16; c += 8) {
    const uint4 b = nt_load16(reinterpret_cast<const uint4*>(brow + c * 16));
    const uint4 q = *reinterpret_cast<const uint4*>(qhj + 4 * c);
    part = __builtin_amdgcn_sdot4((int)b.x, (int)q.x, part, false);
    part = __builtin_amdgcn_sdot4((int)b.y, (int)q.y, part, false);
    part = __builtin_amdgcn_sdot4((int)b.z, (int)q.z, part, false);
    part = __builtin_amdgcn_sdot4((int)b.w, (int)q.w, part, false);
  }
  return part;
}

template <bool I8>
__global__ __launch_bounds__(256) void decode_gemv_b1_kernel(gemv_params p) {
  const int layer = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane & 7, rl = lane >> 3;          // 8 lanes per row, 8 rows per iteration
  const int nw = p.K / 32;                           // words per row
  const int row_base = blockIdx.x * GEMV_ROWS_PER_BLOCK + wave * GEMV_ROWS_PER_WAVE;
  if (row_base >= p.N) return;
  const uint32_t* P = p.P + (size_t)layer * p.N * nw;
  const uint32_t* planes = p.planes + (size_t)layer * 8 * nw;

  int dot[GEMV_ITERS];
#pragma unroll
  for (int it = 0; it < GEMV_ITERS; ++it) dot[it] = 0;

  for (int wc = 0; wc < nw; wc += 128) {             // 128 words (4096 columns) of planes in registers at a time
    uint32_t pl[4][8][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int w0 = wc + 32 * i + 4 * sub;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint4 v = (w0 < nw) ? *reinterpret_cast<const uint4*>(planes + ((size_t)(w0 >> 2) * 8 + q) * 4) : make_uint4(0, 0, 0, 0);
        pl[i][q][0] = v.x; pl[i][q][1] = v.y; pl[i][q][2] = v.z; pl[i][q][3] = v.w;
      }
    }
#pragma unroll
    for (int it = 0; it < GEMV_ITERS; ++it) {
      const int row = row_base + it * 8 + rl;
      const bool okr = row < p.N;
      const uint32_t* prow = P + (size_t)(okr ? row : 0) * nw;
      uint4 w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int w0 = wc + 32 * i + 4 * sub;
        const bool ok = okr && (w0 < nw);
        const uint4 t = *reinterpret_cast<const uint4*>(prow + (ok ? w0 : 0));
        const uint32_t m = ok ? 0xFFFFFFFFu : 0u;
        w[i] = make_uint4(t.x & m, t.y & m, t.z & m, t.w & m);
      }
      int a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t ww[4] = {w[i].x, w[i].y, w[i].z, w[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int q = 0; q < 8; ++q) a[q] += __builtin_popcount(ww[j] & pl[i][q][j]);
      }
      int d = 0;
#pragma unroll
      for (int q = 0; q < 7; ++q) d += a[q] << q;
      d -= a[7] << 7;
      dot[it] += d;
    }
  }

  // experts: lane `sub` covers r-chunks sub, sub+8, ... (8 bf16 each) of its row, for every selected expert
  const float gam = p.gamma[layer];
  const float sc = fp16_bits_to_f32(p.scale[layer]) / gam;
  const int rs = p.rowsum[layer];
  __shared__ __attribute__((aligned(16))) uint32_t s_qh[I8 ? 4 : 1][I8 ? I8_MAX_CODE_WORDS : 4];
  __shared__ float s_gh[I8 ? 4 : 1][I8_MAX_TOPK];
  if constexpr (I8) expert_codes_wave(p.h + (size_t)layer * p.topk * p.r, p.topk, p.r, s_qh[wave], s_gh[wave]);
#pragma unroll
  for (int it = 0; it < GEMV_ITERS; ++it) {
    const int row = row_base + it * 8 + rl;
    const bool okr = row < p.N;
    float yh = 0.0f;
    if constexpr (I8) {
      const int8_t* B8 = (const int8_t*)p.hpB;
      for (int j = 0; j < p.topk; ++j) {
        const int e = p.idx[layer * p.topk + j];
        const float gt = p.gate[layer * p.topk + j];
        const size_t brow = ((size_t)layer * p.E + e) * p.N + (okr ? row : 0);
        int part = expert_dot_i8(B8 + brow * p.r, s_qh[wave] + j * (p.r / 4), p.r, sub);
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
        const float ys = __fmul_rn(1.0f / s_gh[wave][j], (float)part) / p.gB[brow];
        yh += gt * ys;                                 // the same value in all 8 lanes of the row
      }
    } else if (p.r > 0) {
      for (int j = 0; j < p.topk; ++j) {
        const int e = p.idx[layer * p.topk + j];
        const float gt = p.gate[layer * p.topk + j];
        const uint16_t* brow = p.hpB + (((size_t)layer * p.E + e) * p.N + (okr ? row : 0)) * p.r;
        const float* hh = p.h + ((size_t)layer * p.topk + j) * p.r;
        float part = 0.0f;
        for (int c = sub; c < p.r / 8; c += 8) {
          const uint4 b = *reinterpret_cast<const uint4*>(brow + c * 8);
          const float4 h0 = *reinterpret_cast<const float4*>(hh + c * 8);
          const float4 h1 = *reinterpret_cast<const float4*>(hh + c * 8 + 4);
          part += __uint_as_float(b.x << 16) * h0.x + __uint_as_float(b.x & 0xFFFF0000u) * h0.y;
          part += __uint_as_float(b.y << 16) * h0.z + __uint_as_float(b.y & 0xFFFF0000u) * h0.w;
          part += __uint_as_float(b.z << 16) * h1.x + __uint_as_float(b.z & 0xFFFF0000u) * h1.y;
          part += __uint_as_float(b.w << 16) * h1.z + __uint_as_float(b.w & 0xFFFF0000u) * h1.w;
        }
        yh += gt * part;
      }
    }
    int d = dot[it];
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) {
      d += __shfl_xor(d, o, 64);
      if constexpr (!I8) yh += __shfl_xor(yh, o, 64);
    }
    if (sub == 0 && okr) {
      const int acc = 2 * d - rs;
      if (p.acc_out) p.acc_out[(size_t)layer * p.N + row] = acc;
      const float y = __fmul_rn(sc, (float)acc) + p.alpha * yh;
      p.Y[(size_t)layer * p.N + row] = f32_to_bf16(y);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Batch 1 on the row-interleaved packing (PQ_PACKED_TILED64): rows are grouped by 64 and stored as
// [group][word/4][row % 64][word % 4], so lane l of a wavefront owns row 64 g + l and a wave-wide
// 16-byte load is 1 KiB of contiguous HBM.  The activation bit planes are then the same for all
// lanes: they are fetched with scalar loads and used as scalar operands, no cross-lane reduction is
// needed, and a lane needs only its weight words and 8 counters in VGPRs, so many waves are
// resident and many loads are in flight.  The 4 wavefronts of a workgroup split the columns.
// ------------------------------------------------------------------------------------------
template <int GPB, bool I8>   // row groups (of 64 rows) per workgroup: all their loads are issued before the popcounts start
__global__ __launch_bounds__(256) void decode_gemv_tiled_kernel(gemv_params p) {
  __shared__ int s_dot[GPB][4][64];
  __shared__ float s_yh[GPB][64];
  __shared__ __attribute__((aligned(16))) uint32_t s_qh[I8 ? 4 : 1][I8 ? I8_MAX_CODE_WORDS : 4];
  __shared__ float s_gh[I8 ? 4 : 1][I8_MAX_TOPK];
  const int layer = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = p.K / 32, nq = nw / 4;
  const int G = (p.N + 63) / 64;
  const int xl = p.xshare > 1 ? layer / p.xshare : layer;   // the token this weight set reads
  const uint32_t* __restrict__ planes = p.planes + (size_t)xl * 8 * nw;

  int a[GPB][8];
#pragma unroll
  for (int g = 0; g < GPB; ++g)
#pragma unroll
    for (int pp = 0; pp < 8; ++pp) a[g][pp] = 0;
  // 32 chunks of 128 columns per pass, 8 per wavefront.  Whole passes run without any condition, so the
  // loads stay in flight while the wait counter releases one chunk at a time; the ragged last pass
  // clamps its addresses and skips the chunks beyond the row.
  auto pass = [&](const int q0, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    uint4 w[GPB][8];
#pragma unroll
    for (int g = 0; g < GPB; ++g) {
      const int grp = blockIdx.x * GPB + g;
      const uint4* __restrict__ Pg = reinterpret_cast<const uint4*>(p.P) + ((size_t)layer * G + (grp < G ? grp : G - 1)) * nq * 64;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = q0 + 4 * i + wave;
        w[g][i] = nt_load16(&Pg[(size_t)((FULL || q < nq) ? q : nq - 1) * 64 + lane]);
      }
    }
    // full passes request the 32 plane words of chunk i+1 (scalar loads, uniform address) before the
    // popcounts of chunk i start
    if constexpr (FULL) {
      uint32_t pc[32], pn[32];
      {
        const uint32_t* pl = planes + (size_t)(q0 + wave) * 32;
#pragma unroll
        for (int t = 0; t < 32; ++t) pc[t] = pl[t];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i + 1 < 8) {
          const uint32_t* pl = planes + (size_t)(q0 + 4 * (i + 1) + wave) * 32;
#pragma unroll
          for (int t = 0; t < 32; ++t) pn[t] = pl[t];
        }
#pragma unroll
        for (int pp = 0; pp < 8; ++pp)
#pragma unroll
          for (int g = 0; g < GPB; ++g)
            a[g][pp] += __builtin_popcount(w[g][i].x & pc[4 * pp]) + __builtin_popcount(w[g][i].y & pc[4 * pp + 1]) +
                        __builtin_popcount(w[g][i].z & pc[4 * pp + 2]) + __builtin_popcount(w[g][i].w & pc[4 * pp + 3]);
#pragma unroll
        for (int t = 0; t < 32; ++t) pc[t] = pn[t];
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = q0 + 4 * i + wave;
        if (q < nq) {                                  // wave-uniform
          const uint32_t* pl = planes + (size_t)q * 32;
#pragma unroll
          for (int pp = 0; pp < 8; ++pp)
#pragma unroll
            for (int g = 0; g < GPB; ++g)
              a[g][pp] += __builtin_popcount(w[g][i].x & pl[4 * pp]) + __builtin_popcount(w[g][i].y & pl[4 * pp + 1]) +
                          __builtin_popcount(w[g][i].z & pl[4 * pp + 2]) + __builtin_popcount(w[g][i].w & pl[4 * pp + 3]);
        }
      }
    }
  };
  int q0 = 0;
  for (; q0 + 32 <= nq; q0 += 32) pass(q0, std::true_type{});
  if (q0 < nq) pass(q0, std::false_type{});

#pragma unroll
  for (int g = 0; g < GPB; ++g) {
    const int grp = blockIdx.x * GPB + g;
    int d = 0;
#pragma unroll
    for (int pp = 0; pp < 7; ++pp) d += a[g][pp] << pp;
    d -= a[g][7] << 7;
    s_dot[g][wave][lane] = d;
    // experts: wavefront w covers rows 16 w .. 16 w + 15 of the group, 8 lanes per row (one 16-byte chunk
    // of the expert's rank each), so a load instruction reads 8 whole 128-byte rows
    if (p.r > 0) {
      const int sub = lane & 7, rl = lane >> 3;
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int lrow = 16 * wave + 8 * it + rl;
        const int erow = grp * 64 + lrow;
        const bool oke = erow < p.N;
        float yh = 0.0f;
        if constexpr (I8) {
          // The first 16-byte chunk of the row for the first PF selected experts and the rows' gammas are requested
          // together (slots past top_k repeat the last one: no branch around a load); the hidden-state codes are
          // formed while they are on their way.
          constexpr int PF = 4;
          const int8_t* B8 = (const int8_t*)p.hpB;
          const int nch = p.r / 16;
          uint4 bq[PF];
          float gbv[PF];
          size_t browi[PF];
#pragma unroll
          for (int j = 0; j < PF; ++j) {
            const int e = p.idx[layer * p.topk + min(j, p.topk - 1)];
            browi[j] = ((size_t)layer * p.E + e) * p.N + (oke ? erow : 0);
            bq[j] = nt_load16(reinterpret_cast<const uint4*>(B8 + browi[j] * p.r + (sub < nch ? sub : 0) * 16));
            gbv[j] = p.gB[browi[j]];
          }
          if (g == 0 && it == 0) expert_codes_wave(p.h + (size_t)layer * p.topk * p.r, p.topk, p.r, s_qh[wave], s_gh[wave]);
#pragma unroll
          for (int j = 0; j < PF; ++j)
            if (j < p.topk) {
              const uint32_t* qhj = s_qh[wave] + j * (p.r / 4);
              int part = 0;
              if (sub < nch) {
                const uint4 q = *reinterpret_cast<const uint4*>(qhj + 4 * sub);
                part = __builtin_amdgcn_sdot4((int)bq[j].x, (int)q.x, part, false);
                part = __builtin_amdgcn_sdot4((int)bq[j].y, (int)q.y, part, false);
                part = __builtin_amdgcn_sdot4((int)bq[j].z, (int)q.z, part, false);
                part = __builtin_amdgcn_sdot4((int)bq[j].w, (int)q.w, part, false);
                part += expert_dot_i8(B8 + browi[j] * p.r, qhj, p.r, sub + 8);
              }
#pragma unroll
              for (int o = 4; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
              const float ys = __fmul_rn(1.0f / s_gh[wave][j], (float)part) / gbv[j];
              yh += p.gate[layer * p.topk + j] * ys;   // the same value in all 8 lanes of the row
            }
          for (int j = PF; j < p.topk; ++j) {
            const size_t br = ((size_t)layer * p.E + p.idx[layer * p.topk + j]) * p.N + (oke ? erow : 0);
            int part = expert_dot_i8(B8 + br * p.r, s_qh[wave] + j * (p.r / 4), p.r, sub);
#pragma unroll
            for (int o = 4; o > 0; o >>= 1) part += __shfl_xor(part, o, 64);
            const float ys = __fmul_rn(1.0f / s_gh[wave][j], (float)part) / p.gB[br];
            yh += p.gate[layer * p.topk + j] * ys;
          }
          if (sub == 0) s_yh[g][lrow] = yh;
          continue;
        }
        for (int j = 0; j < p.topk; ++j) {
          const int e = p.idx[layer * p.topk + j];
          const float gt = p.gate[layer * p.topk + j];
          const uint16_t* brow = p.hpB + (((size_t)layer * p.E + e) * p.N + (oke ? erow : 0)) * p.r;
          const float* hh = p.h + ((size_t)layer * p.topk + j) * p.r;
          float part = 0.0f;
          for (int c = sub; c < p.r / 8; c += 8) {
            const uint4 b = nt_load16(reinterpret_cast<const uint4*>(brow + c * 8));
            const float4 h0 = *reinterpret_cast<const float4*>(hh + c * 8);
            const float4 h1 = *reinterpret_cast<const float4*>(hh + c * 8 + 4);
            part += __uint_as_float(b.x << 16) * h0.x + __uint_as_float(b.x & 0xFFFF0000u) * h0.y;
            part += __uint_as_float(b.y << 16) * h0.z + __uint_as_float(b.y & 0xFFFF0000u) * h0.w;
            part += __uint_as_float(b.z << 16) * h1.x + __uint_as_float(b.z & 0xFFFF0000u) * h1.y;
            part += __uint_as_float(b.w << 16) * h1.z + __uint_as_float(b.w & 0xFFFF0000u) * h1.w;
          }
          yh += gt * part;
        }
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) yh += __shfl_xor(yh, o, 64);
        if (sub == 0) s_yh[g][lrow] = yh;
      }
    }
  }
  __syncthreads();
  if (wave < GPB) {
    const int g = wave;
    const int row = (blockIdx.x * GPB + g) * 64 + lane;
    if (row < p.N) {
      const int dd = s_dot[g][0][lane] + s_dot[g][1][lane] + s_dot[g][2][lane] + s_dot[g][3][lane];
      const float yy = p.r > 0 ? s_yh[g][lane] : 0.0f;
      const int acc = 2 * dd - p.rowsum[xl];
      if (p.acc_out) p.acc_out[(size_t)layer * p.N + row] = acc;
      const float sc = fp16_bits_to_f32(p.scale[layer]) / p.gamma[xl];
      p.Y[(size_t)layer * p.N + row] = f32_to_bf16(__fmul_rn(sc, (float)acc) + p.alpha * yy);
    }
  }
}

// Offline re-tiling of the row-major packing [N][K/32] into the row-interleaved one (rows padded to 64).
__global__ __launch_bounds__(256) void retile64_kernel(const uint32_t* __restrict__ P, int N, int nw, uint32_t* __restrict__ T,
                                                       size_t total) {
  const size_t o = (size_t)blockIdx.x * 256 + threadIdx.x;   // ((g*nq + q)*64 + lane)*4 + j
  if (o >= total) return;
  const int j = o & 3, lane = (o >> 2) & 63;
  const size_t gq = o >> 8;
  const int nq = nw / 4;
  const int q = (int)(gq % nq), g = (int)(gq / nq);
  const int row = g * 64 + lane;
  T[o] = row < N ? P[(size_t)row * nw + 4 * q + j] : 0u;
}

// ------------------------------------------------------------------------------------------
// Batch 2..16: int8 MFMA with {0,1} weight bytes expanded in registers.
// ------------------------------------------------------------------------------------------
struct gemm16_params {
  const uint32_t* P;      // [L][N][K/32]
  const uint16_t* scale;  // [L]
  const int8_t* xq;       // [L][B][K]
  const int* rowsum;      // [L][B]
  const float* gamma;     // [L][B]
  const uint16_t* hpB;    // [L][E][N][r]
  const int* idx;         // [L][B][topk]
  const float* gate;      // [L][B][topk]
  const float* h;         // [L][B][topk][r]
  uint16_t* Y;            // [L][B][N]
  int* acc_out;           // [L][B][N] or null
  int B, N, K, E, r, topk;
  float alpha;
  const float* gB;        // INT8 experts: [L][E][N] gammas of the rows of hpB (then hpB is int8 [L][E][N][r])
  int xshare;             // > 1: that many consecutive weight sets read the same tokens (codes, row sums, gammas of set / xshare)
};

constexpr int G16_LDS_CODE_BYTES = 32768;           // LDS the row-interleaved kernel spends on the batch's codes
constexpr int G16_RT = 4;                           // 16-row MFMA tiles per wavefront
constexpr int G16_ROWS_PER_WAVE = 16 * G16_RT;
constexpr int G16_ROWS_PER_BLOCK = 4 * G16_ROWS_PER_WAVE;

// Stages the batch's INT8 codes and the gate-weighted expert hidden states into LDS and returns the mask
// of experts that some token selected.  xs: [TOKS][kcols] int8, 16-byte chunk c of token j at chunk c ^ (j & 7);
// hm: [TOKS][E*r] bf16 (zero where a token did not select the expert), same chunk swizzle.
// I8: hm holds INT8 codes instead ([TOKS][E*r] bytes, 16-byte chunk c of token j at chunk c ^ (j & 7)): every
// selected (token, expert) hidden state is put on the INT8 grid with its own gamma (Sec. 3.1 quantiser), one
// wavefront per slot; behind the codes sit 1/gamma_h and the gate per (token, expert), zero where not selected.
// Columns [k0, k0 + kcols) of the batch's codes into xs, rows `stride` bytes apart (kcols and stride multiples of 128)
template <int TOKS>
__device__ __forceinline__ void g16_stage_codes(const gemm16_params& p, int layer, unsigned char* xs, int k0, int kcols, int stride) {
  const int kch = kcols / 16;
  for (int c = threadIdx.x; c < TOKS * kch; c += 256) {
    const int j = c / kch, cc = c % kch;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (j < p.B) v = *reinterpret_cast<const uint4*>(p.xq + ((size_t)layer * p.B + j) * p.K + k0 + cc * 16);
    *reinterpret_cast<uint4*>(xs + (size_t)j * stride + ((cc ^ (j & 7)) << 4)) = v;
  }
}

// kcols: how many columns of the codes are staged now (all K, or the first block of a kernel that walks K in blocks)
template <int TOKS, bool I8 = false>
__device__ __forceinline__ unsigned long long g16_stage_inputs(const gemm16_params& p, int layer, unsigned char* xs,
                                                               uint16_t* hm, int kcols) {
  const int tid = threadIdx.x;
  const int Er = p.E * p.r;
  g16_stage_codes<TOKS>(p, layer, xs, 0, kcols, kcols);
  for (int c = tid; c < TOKS * Er / 8; c += 256) reinterpret_cast<uint4*>(hm)[c] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  unsigned long long used = 0ull;
  if (p.r > 0) {
    // every wavefront builds the mask of selected experts: lane s reads slot s, a ballot per expert bit
    const int nslot = p.B * p.topk;                  // <= 16 * 64
    for (int s0 = 0; s0 < nslot; s0 += 64) {
      const int s = s0 + (tid & 63);
      const int e = s < nslot ? p.idx[(size_t)layer * nslot + s] : -1;
      for (int ee = 0; ee < p.E; ++ee) used |= (__ballot(e == ee) != 0ull) ? (1ull << ee) : 0ull;
    }
    if constexpr (I8) {
      int8_t* hq = reinterpret_cast<int8_t*>(hm);
      float* inv = reinterpret_cast<float*>(hq + (size_t)TOKS * Er);      // [TOKS][E] 1/gamma_h, then [TOKS][E] gates
      float* gts = inv + TOKS * p.E;
      for (int c = tid; c < 2 * TOKS * p.E; c += 256) inv[c] = 0.0f;
      __syncthreads();
      const int lane = tid & 63, wave = tid >> 6;
      for (int s = wave; s < nslot; s += 4) {         // wave-uniform
        const int j = s / p.topk;
        const int e = p.idx[(size_t)layer * nslot + s];
        const float* hs = p.h + ((size_t)layer * nslot + s) * p.r;
        float amax = 0.0f;
        for (int rr = lane; rr < p.r; rr += 64) amax = fmaxf(amax, fabsf(hs[rr]));
        amax = wave_max(amax);
        const float gh = 128.0f / fmaxf(amax, 1e-5f);
        for (int rr = lane; rr < p.r; rr += 64) {
          const int q = (int)fminf(fmaxf(rintf(__fmul_rn(hs[rr], gh)), -128.0f), 127.0f);
          const int col = e * p.r + rr;
          hq[(size_t)j * Er + ((((col >> 4) ^ (j & 7)) << 4) | (col & 15))] = (int8_t)q;
        }
        if (lane == 0) {
          inv[j * p.E + e] = 1.0f / gh;
          gts[j * p.E + e] = p.gate[(size_t)layer * nslot + s];
        }
      }
    } else {
    for (int c = tid; c < p.B * p.topk * p.r; c += 256) {
      const int rr = c % p.r, s = c / p.r, j = s / p.topk;
      const int e = p.idx[(size_t)layer * p.B * p.topk + s];
      const float v = p.gate[(size_t)layer * p.B * p.topk + s] * p.h[((size_t)layer * p.B * p.topk + s) * p.r + rr];
      const int col = e * p.r + rr;                  // 16-byte chunk (col/8) stored at chunk ^ (j & 7)
      hm[(size_t)j * Er + ((((col >> 3) ^ (j & 7)) << 3) | (col & 7))] = f32_to_bf16(v);
    }
    }
  }
  __syncthreads();
  return used;
}

// TOKS = token rows kept in LDS (8 or 16).  With at most 8 tokens the MFMA's columns 8..15 re-read the
// rows of columns 0..7 (their results are never stored), which halves the LDS footprint and doubles the
// resident workgroups per CU.
template <int TOKS>
__global__ __launch_bounds__(256) void decode_gemm16_kernel(gemm16_params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dsm[];
  // dsm: xq [TOKS][K] int8 (16-byte chunk c of token j stored at chunk c ^ (j & 7)), then Hm [TOKS][E*r] bf16
  const int layer = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = p.K, Er = p.E * p.r;
  unsigned char* xs = dsm;
  uint16_t* hm = reinterpret_cast<uint16_t*>(dsm + TOKS * (size_t)K);
  const unsigned long long used = g16_stage_inputs<TOKS>(p, layer, xs, hm, K);

  const int i = lane & 15, g = lane >> 4;
  const int il = i & (TOKS - 1);                     // LDS row read for MFMA column i
  const int row0 = blockIdx.x * G16_ROWS_PER_BLOCK + wave * G16_ROWS_PER_WAVE;
  if (row0 >= p.N) return;
  const int nw = K / 32;
  const uint32_t* P = p.P + (size_t)layer * p.N * nw;

  // A wavefront walks its 64 rows as four 16-row MFMA tiles.  One step covers 4096 columns of a tile:
  // 16 whole rows of 512 bytes = 8 KB of contiguous packed weights, fetched by eight 16-byte loads per
  // lane (lane (i, g) takes bytes 64 j + 16 g of row i), so every DRAM page is visited once.  The loads
  // of the next step are issued before the MFMAs of the current one.
  //
  // Weight bytes for the MFMA are {0, -128}: (x << s) & 0x80808080 puts bit 8 b + 7 - s of the word x
  // into the sign position of byte b, one AND (plus one shift) per four weights.  The accumulator then
  // holds -128 * sum_k [S=+1] q_k; the INT8 codes in LDS are stored in the matching byte order.  Rows
  // past N read row 0 and are never stored.
  constexpr uint32_t SIGNS = 0x80808080u;
  const int ncb = (K + 4095) / 4096;                 // K is a multiple of 512
  const int nsteps = G16_RT * ncb;
  uint4 wn[8];
  auto issue = [&](const int u) {
    const int t = u / ncb, cb = u - t * ncb;
    const int row = row0 + 16 * t + i;
    const uint32_t* pr = P + (size_t)(row < p.N ? row : 0) * nw + 4 * g + cb * 128;
    const int nj = min(8, (K - 4096 * cb) / 512);
#pragma unroll
    for (int j = 0; j < 8; ++j) wn[j] = nt_load16(reinterpret_cast<const uint4*>(pr + (j < nj ? j : 0) * 16));
  };
  issue(0);
  const int nhf = p.r / 32;

  for (int t = 0; t < G16_RT; ++t) {
    if (row0 + 16 * t >= p.N) break;                 // wave-uniform
    i32x4_t acc0 = i32x4_t{0, 0, 0, 0}, acc1 = i32x4_t{0, 0, 0, 0};
    for (int cb = 0; cb < ncb; ++cb) {
      uint4 w[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] = wn[j];
      const int u = t * ncb + cb;
      if (u + 1 < nsteps) issue(u + 1);
      const int nj = min(8, (K - 4096 * cb) / 512);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (j < nj) {                                // block-uniform
#pragma unroll
          for (int ww = 0; ww < 4; ++ww) {
            const int chunk = 256 * cb + 32 * j + 8 * g + 2 * ww;
            const uint4 act0 = *reinterpret_cast<const uint4*>(xs + (size_t)il * K + ((chunk ^ (il & 7)) << 4));
            const uint4 act1 = *reinterpret_cast<const uint4*>(xs + (size_t)il * K + (((chunk + 1) ^ (il & 7)) << 4));
            const uint32_t x = ww == 0 ? w[j].x : ww == 1 ? w[j].y : ww == 2 ? w[j].z : w[j].w;
            const uint4 e0 = make_uint4(x & SIGNS, (x << 1) & SIGNS, (x << 2) & SIGNS, (x << 3) & SIGNS);
            const uint4 e1 = make_uint4((x << 4) & SIGNS, (x << 5) & SIGNS, (x << 6) & SIGNS, (x << 7) & SIGNS);
            acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, e0), __builtin_bit_cast(i32x4_t, act0),
                                                         acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, e1), __builtin_bit_cast(i32x4_t, act1),
                                                         acc1, 0, 0, 0);
          }
        }
      }
    }
    // experts selected by at least one token of the batch: dense-masked bf16 MFMA, 32 columns of r per
    // issue; the rows of up to four experts are requested together
    f32x4_t accf = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (p.r > 0) {
      const int row = row0 + 16 * t + i;
      const size_t roff = (size_t)(row < p.N ? row : 0) * p.r + 8 * g;
      for (int hf = 0; hf < nhf; hf += 2) {
        const bool two = hf + 1 < nhf;
        for (int e0 = 0; e0 < p.E; e0 += 4) {
          if (!((used >> e0) & 0xFull)) continue;
          uint4 a0[4], a1[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int e = (e0 + q < p.E && ((used >> (e0 + q)) & 1ull)) ? e0 + q : -1;
            const uint16_t* br = p.hpB + ((size_t)layer * p.E + (e < 0 ? 0 : e)) * p.N * p.r + roff + 32 * hf;
            if (e >= 0) {                            // block-uniform
              a0[q] = *reinterpret_cast<const uint4*>(br);          // (plain loads: two halves of the same lines, see the tiled kernel)
              a1[q] = *reinterpret_cast<const uint4*>(br + (two ? 32 : 0));
            } else {
              a0[q] = make_uint4(0, 0, 0, 0);
              a1[q] = make_uint4(0, 0, 0, 0);
            }
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int e = e0 + q;
            if (e < p.E && ((used >> e) & 1ull)) {
              const int col = e * p.r + 32 * hf + 8 * g;
              const uint4 b0 = *reinterpret_cast<const uint4*>(hm + (size_t)il * Er + (((col >> 3) ^ (il & 7)) << 3));
              accf = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0[q]), __builtin_bit_cast(bf16x8_t, b0),
                                                             accf, 0, 0, 0);
              if (two) {
                const uint4 b1 = *reinterpret_cast<const uint4*>(hm + (size_t)il * Er + ((((col + 32) >> 3) ^ (il & 7)) << 3));
                accf = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1[q]), __builtin_bit_cast(bf16x8_t, b1),
                                                               accf, 0, 0, 0);
              }
            }
          }
        }
      }
    }
    // D[row 4 g + v][token i]
    const int j = i;
    const int n0 = row0 + 16 * t + 4 * g;
    if (j < p.B && n0 < p.N) {                        // N % 4 == 0: a group of four rows is all in or all out
      const float sc = fp16_bits_to_f32(p.scale[layer]) / p.gamma[layer * p.B + j];
      const int rs = p.rowsum[layer * p.B + j];
      float y[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int a = -((acc0[v] + acc1[v]) >> 6) - rs;   // 2 * (-acc / 128) - rowsum, acc is a multiple of 128
        if (p.acc_out) p.acc_out[((size_t)layer * p.B + j) * p.N + n0 + v] = a;
        y[v] = __fmul_rn(sc, (float)a) + p.alpha * accf[v];
      }
      *reinterpret_cast<uint2*>(p.Y + ((size_t)layer * p.B + j) * p.N + n0) =
          make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
    }
  }
}

// The same product on the row-interleaved packing.  A wavefront owns one group of 64 rows, whose packed
// bits are one contiguous run of K * 8 bytes: each load instruction reads 1 KB of consecutive memory
// (lane = row, 128 columns).  The MFMA wants lane (i, g) to hold row 16 t + i instead, so each 1 KB chunk
// makes a round trip through a wave-private LDS patch: written as loaded, read back one word per tile
// (word g of row 16 t + i, bank-conflict free).  Results leave through the same patch so that a token's
// 64 outputs are stored as one 128-byte run.
template <int TOKS, bool I8 = false>
__global__ __launch_bounds__(256, 4) void decode_gemm16_tiled_kernel(gemm16_params p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dsm[];
  // dsm: xq [TOKS][min(K, KC)] int8 (one block of the codes), then a region that first holds Hm [TOKS][E*r] bf16 (expert phase) and afterwards
  // the four 2 KB wave-private patches (1-bit phase and output staging); it is max(8 KB, Hm) long
  const int layer = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = p.K, Er = p.E * p.r;
  // the codes pass through LDS in blocks of KC columns (32 KB whatever the batch), so that four workgroups fit a CU at any K
  constexpr int KC = G16_LDS_CODE_BYTES / TOKS;
  const int KCs = K < KC ? K : KC;                    // row stride of xs
  unsigned char* xs = dsm;
  uint16_t* hm = reinterpret_cast<uint16_t*>(dsm + TOKS * (size_t)KCs);
  uint32_t* patch = reinterpret_cast<uint32_t*>(dsm + TOKS * (size_t)KCs) + wave * 512;
  const int i = lane & 15, g = lane >> 4;
  const int il = i & (TOKS - 1);
  const int G = (p.N + 63) / 64;
  const int grp = blockIdx.x * 4 + wave;
  const int nq = K / 128;
  const uint4* __restrict__ Pg = reinterpret_cast<const uint4*>(p.P) + ((size_t)layer * G + (grp < G ? grp : G - 1)) * nq * 64 + lane;
  constexpr uint32_t SIGNS = 0x80808080u;             // weight bytes {0, -128}, see decode_gemm16_kernel

  i32x4_t acc[4][2];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t][0] = acc[t][1] = i32x4_t{0, 0, 0, 0};

  // Eight chunks (8 KB per wavefront) are in flight at any time: as soon as a chunk has been written to the
  // patch its registers receive the chunk eight positions ahead.
  uint4 w[8];
#pragma unroll
  for (int jj = 0; jj < 8; ++jj) w[jj] = nt_load16(Pg + (size_t)(jj < nq ? jj : nq - 1) * 64);
  const int lx = p.xshare > 1 ? layer / p.xshare : layer;   // the token block this weight set reads
  const unsigned long long used = g16_stage_inputs<TOKS, I8>(p, lx, xs, hm, KCs);   // overlaps the first loads
  const bool active = grp < G;                        // idle wavefronts of the last workgroup still meet the barrier

  // experts selected by at least one token of the batch (dense-masked bf16 MFMA, 32 columns of r per issue)
  f32x4_t accf[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) accf[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  if constexpr (I8) {
    // INT8 experts: per selected expert an exact int8 MFMA product (64 columns of r per issue, lane (i, g) holds
    // bytes 16 g .. 16 g + 15 of row i resp. token i), then D[row 4 g + v][token i] is de-quantised with the
    // token's 1/gamma_h and the row's gamma_B and added with the gate; scales of unselected pairs are zero.
    if (active) {
      const int8_t* hq = reinterpret_cast<const int8_t*>(hm);
      const float* inv = reinterpret_cast<const float*>(hq + (size_t)TOKS * Er);
      const float* gts = inv + TOKS * p.E;
      const int nblk = p.r / 64;
      size_t roff[4];
      int rowg[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int row = grp * 64 + 16 * t + i;
        roff[t] = (size_t)(row < p.N ? row : 0) * p.r + 16 * g;
        const int r4 = grp * 64 + 16 * t + 4 * g;     // first of the four output rows this lane holds (N % 4 == 0)
        rowg[t] = r4 < p.N ? r4 : 0;
      }
      for (int e = 0; e < p.E; ++e) {
        if (!((used >> e) & 1ull)) continue;
        const int8_t* Be = (const int8_t*)p.hpB + ((size_t)layer * p.E + e) * p.N * p.r;
        i32x4_t ai[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) ai[t] = i32x4_t{0, 0, 0, 0};
        for (int blk = 0; blk < nblk; ++blk) {
          uint4 a[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) a[t] = nt_load16(reinterpret_cast<const uint4*>(Be + roff[t] + 64 * blk));
          const int chunk = (e * p.r + 64 * blk) / 16 + g;
          const uint4 b = *reinterpret_cast<const uint4*>(hq + (size_t)il * Er + ((chunk ^ (il & 7)) << 4));
#pragma unroll
          for (int t = 0; t < 4; ++t)
            ai[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, a[t]), __builtin_bit_cast(i32x4_t, b), ai[t], 0, 0, 0);
        }
        const float ig = inv[il * p.E + e], gt = gts[il * p.E + e];
        const float* gbe = p.gB + ((size_t)layer * p.E + e) * p.N;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          // the row gammas come off through the hardware reciprocal (1 ulp): sixteen IEEE divisions per expert and
          // lane would cost as many instructions as the whole packed product
          const float4 gb = *reinterpret_cast<const float4*>(gbe + rowg[t]);
          accf[t][0] += gt * (__fmul_rn(ig, (float)ai[t][0]) * __builtin_amdgcn_rcpf(gb.x));
          accf[t][1] += gt * (__fmul_rn(ig, (float)ai[t][1]) * __builtin_amdgcn_rcpf(gb.y));
          accf[t][2] += gt * (__fmul_rn(ig, (float)ai[t][2]) * __builtin_amdgcn_rcpf(gb.z));
          accf[t][3] += gt * (__fmul_rn(ig, (float)ai[t][3]) * __builtin_amdgcn_rcpf(gb.w));
        }
      }
    }
  } else if (p.r > 0 && active) {
    const int nhf = p.r / 32;
    size_t roff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int row = grp * 64 + 16 * t + i;
      roff[t] = (size_t)(row < p.N ? row : 0) * p.r + 8 * g;
    }
    for (int e = 0; e < p.E; ++e) {
      if (!((used >> e) & 1ull)) continue;
      const uint16_t* Be = p.hpB + ((size_t)layer * p.E + e) * p.N * p.r;
      for (int hf = 0; hf < nhf; hf += 2) {
        const bool two = hf + 1 < nhf;
        uint4 a0[4], a1[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          // plain loads: the two instructions take the two halves of the same 128-byte lines (16 rows x 64 B each), and
          // with the non-temporal hint the second half was fetched from memory again (1.15 x the algorithmic bytes)
          a0[t] = *reinterpret_cast<const uint4*>(Be + roff[t] + 32 * hf);
          a1[t] = *reinterpret_cast<const uint4*>(Be + roff[t] + 32 * hf + (two ? 32 : 0));
        }
        const int col = e * p.r + 32 * hf + 8 * g;
        const uint4 b0 = *reinterpret_cast<const uint4*>(hm + (size_t)il * Er + (((col >> 3) ^ (il & 7)) << 3));
        const uint4 b1 = *reinterpret_cast<const uint4*>(hm + (size_t)il * Er + ((((col + (two ? 32 : 0)) >> 3) ^ (il & 7)) << 3));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          accf[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0[t]), __builtin_bit_cast(bf16x8_t, b0),
                                                            accf[t], 0, 0, 0);
          if (two)
            accf[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1[t]), __builtin_bit_cast(bf16x8_t, b1),
                                                              accf[t], 0, 0, 0);
        }
      }
    }
  }

  __syncthreads();                                    // Hm is dead: its LDS becomes the patches

  // Passes of 8 chunks; whole passes carry no condition (one basic block: the accumulators stay put and
  // the MFMAs of one chunk overlap the LDS round trip of the next), the ragged last pass checks each chunk.
  int qb = 0;                                         // first 128-column chunk of the staged block
  auto pass = [&](const int q0, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      if (FULL || q0 + jj < nq) {                     // block-uniform
        uint32_t* buf = patch + (jj & 1) * 256;
        *reinterpret_cast<uint4*>(buf + 4 * lane) = w[jj];
        const int qn = q0 + 8 + jj;
        w[jj] = nt_load16(Pg + (size_t)(qn < nq ? qn : nq - 1) * 64);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int chunk = 8 * (q0 - qb + jj) + 2 * g; // 16-column chunk of the staged part of the activation row
        const uint4 act0 = *reinterpret_cast<const uint4*>(xs + (size_t)il * KCs + ((chunk ^ (il & 7)) << 4));
        const uint4 act1 = *reinterpret_cast<const uint4*>(xs + (size_t)il * KCs + (((chunk + 1) ^ (il & 7)) << 4));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint32_t x = buf[(16 * t + i) * 4 + g];
          const uint4 e0 = make_uint4(x & SIGNS, (x << 1) & SIGNS, (x << 2) & SIGNS, (x << 3) & SIGNS);
          const uint4 e1 = make_uint4((x << 4) & SIGNS, (x << 5) & SIGNS, (x << 6) & SIGNS, (x << 7) & SIGNS);
          acc[t][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, e0), __builtin_bit_cast(i32x4_t, act0),
                                                            acc[t][0], 0, 0, 0);
          acc[t][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, e1), __builtin_bit_cast(i32x4_t, act1),
                                                            acc[t][1], 0, 0, 0);
        }
      }
    }
  };
  constexpr int QPC = KC / 128;                       // 128-column chunks per block (a multiple of 8)
  for (qb = 0; qb < nq; qb += QPC) {
    if (qb > 0) {                                     // next block of the codes; the weight loads in flight carry on
      __syncthreads();
      const int left = K - qb * 128;
      g16_stage_codes<TOKS>(p, lx, xs, qb * 128, left < KC ? left : KC, KCs);
      __syncthreads();
    }
    if (active) {
      const int qe = nq < qb + QPC ? nq : qb + QPC;
      int q0 = qb;
      for (; q0 + 8 <= qe; q0 += 8) pass(q0, std::true_type{});
      if (q0 < qe) pass(q0, std::false_type{});         // only the last block can be ragged
    }
  }
  if (!active) return;                                // no workgroup barrier below

  // D[row 4 g + v][token i] -> patch as [token][64 rows] bf16, then 128-byte runs per token
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  uint16_t* stage = reinterpret_cast<uint16_t*>(patch);
  if (i < p.B) {
    const float sc = fp16_bits_to_f32(p.scale[layer]) / p.gamma[lx * p.B + i];
    const int rs = p.rowsum[lx * p.B + i];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float y[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int a = -((acc[t][0][v] + acc[t][1][v]) >> 6) - rs;   // 2 * (-acc / 128) - rowsum
        const int n = grp * 64 + 16 * t + 4 * g + v;
        if (p.acc_out && n < p.N) p.acc_out[((size_t)layer * p.B + i) * p.N + n] = a;
        y[v] = __fmul_rn(sc, (float)a) + p.alpha * accf[t][v];
      }
      *reinterpret_cast<uint2*>(stage + i * 64 + 16 * t + 4 * g) = make_uint2(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]));
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int piece = lane & 7;
  const int n0 = grp * 64 + 8 * piece;
  const bool vec_ok = (p.N % 8 == 0);
  for (int jb = 0; jb < p.B; jb += 8) {
    const int j = jb + (lane >> 3);
    if (j < p.B && n0 < p.N) {
      uint16_t* dst = p.Y + ((size_t)layer * p.B + j) * p.N + n0;
      const uint16_t* src = stage + j * 64 + 8 * piece;
      if (vec_ok) {                                   // N % 8 == 0: the 8 rows are all inside and 16-byte aligned
        *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
      } else {
        for (int v = 0; v < 8 && n0 + v < p.N; ++v) dst[v] = src[v];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Decoupled FFN at inference (Sec. 3.2 FFN equation; App. A), one token per layer: between the up/gate products
// and the down product one workgroup per layer forms Hd = silu(G) * U from the stored bf16 U and G (fp32), puts
// it on the INT8 grid (codes, bit planes, row sum, gamma: the input of the packed down product) and applies the
// experts' gated unit a = silu(Gate_e x) * (Up_e x) to the hidden pairs the prep kernel left in hug [topk][2r].
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }
// Workgroups per (layer, token): each owns every eighth group of 256 columns of Hd.  The row's maximum decides gamma, so
// the work is two passes (two launches): the parts' maxima, then the quantiser of the own groups (6 KB of LDS per
// workgroup, all workgroups of a batch resident at once); the row sum is added up over the parts with integer atomics.
constexpr int FFN_MID_PARTS = 8;

// Hd = silu(G) * U for one vector (eight columns) of a row
__device__ __forceinline__ void ffn_hd8(const uint4& uu, const uint4& gg, float* hd) {
  const uint32_t uw[4] = {uu.x, uu.y, uu.z, uu.w}, gw[4] = {gg.x, gg.y, gg.z, gg.w};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    hd[2 * t] = silu_f(__uint_as_float(gw[t] << 16)) * __uint_as_float(uw[t] << 16);
    hd[2 * t + 1] = silu_f(__uint_as_float(gw[t] & 0xFFFF0000u)) * __uint_as_float(uw[t] & 0xFFFF0000u);
  }
}

// Pass 1 (one workgroup per (layer, token, part)): Hd over the part's own column groups, its largest magnitude to
// amax_part[row][part]; part 0 also applies the experts' gated unit.  Thread i of a workgroup owns vector i % 32 of its
// (i / 32)-th, (i / 32 + 8)-th, ... own group.
__global__ __launch_bounds__(256) void decode_ffn_amax_kernel(const uint16_t* __restrict__ UG, int B, int F, int r, int topk,
                                                              const float* __restrict__ hug, float* __restrict__ act,
                                                              float* __restrict__ amax_part) {
  __shared__ float red[4];
  const int row = blockIdx.x / FFN_MID_PARTS, part = blockIdx.x % FFN_MID_PARTS, tid = threadIdx.x;
  const int lay = row / B, tok = row - lay * B;
  const uint4* u4 = reinterpret_cast<const uint4*>(UG + ((size_t)(2 * lay) * B + tok) * F);
  const uint4* g4 = reinterpret_cast<const uint4*>(UG + ((size_t)(2 * lay + 1) * B + tok) * F);
  const int nvec = F / 8;
  float amax = 0.0f;
  for (int gi = tid >> 5; (part + FFN_MID_PARTS * gi) * 32 < nvec; gi += 8) {
    const int c = (part + FFN_MID_PARTS * gi) * 32 + (tid & 31);
    if (c < nvec) {
      float hd[8];
      ffn_hd8(u4[c], g4[c], hd);
#pragma unroll
      for (int t = 0; t < 8; ++t) amax = fmaxf(amax, fabsf(hd[t]));
    }
  }
  if (part == 0)
    for (int o = tid; o < topk * r; o += 256) {
      const int j = o / r, i = o - j * r;
      const float* hp = hug + ((size_t)row * topk + j) * 2 * r;
      act[(size_t)row * topk * r + o] = silu_f(hp[r + i]) * hp[i];
    }
  amax = wave_max(amax);
  if ((tid & 63) == 0) red[tid >> 6] = amax;
  __syncthreads();
  if (tid == 0) amax_part[(size_t)row * FFN_MID_PARTS + part] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// Pass 2: the row's maximum from the eight parts, then the part's own column groups again (from cache) through the
// quantiser: codes, bit planes, gamma by part 0, the row sum by integer atomics.
__global__ __launch_bounds__(256) void decode_ffn_mid_kernel(const uint16_t* __restrict__ UG, int B, int F,
                                                             const float* __restrict__ amax_part,
                                                             int8_t* __restrict__ xq, uint32_t* __restrict__ planes,
                                                             int* __restrict__ rowsum, float* __restrict__ gamma) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // this part's column groups of Hd as fp32
  __shared__ prep_shared sh;
  // row = (layer, token); U and G of a layer are two weight sets' outputs, [2 layer + {0, 1}][B][F]
  const int row = blockIdx.x / FFN_MID_PARTS, part = blockIdx.x % FFN_MID_PARTS, tid = threadIdx.x;
  const int lay = row / B, tok = row - lay * B;
  const uint4* u4 = reinterpret_cast<const uint4*>(UG + ((size_t)(2 * lay) * B + tok) * F);
  const uint4* g4 = reinterpret_cast<const uint4*>(UG + ((size_t)(2 * lay + 1) * B + tok) * F);
  const int nvec = F / 8;
  float amax = 0.0f;
#pragma unroll
  for (int q = 0; q < FFN_MID_PARTS; ++q) amax = fmaxf(amax, amax_part[(size_t)row * FFN_MID_PARTS + q]);
  for (int gi = tid >> 5; (part + FFN_MID_PARTS * gi) * 32 < nvec; gi += 8) {
    const int c = (part + FFN_MID_PARTS * gi) * 32 + (tid & 31);
    float hd[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (c < nvec) ffn_hd8(u4[c], g4[c], hd);
    float* dst = xs + gi * 256 + 8 * (tid & 31);
    *reinterpret_cast<float4*>(dst) = make_float4(hd[0], hd[1], hd[2], hd[3]);
    *reinterpret_cast<float4*>(dst + 4) = make_float4(hd[4], hd[5], hd[6], hd[7]);
  }
  __syncthreads();                                    // xs complete
  prep_quantise_own(amax, (size_t)row, F, xs, sh, xq, planes, rowsum, gamma, part, FFN_MID_PARTS);
}

}  // namespace

// The per-token kernels stage one token as fp32 (plus its codes for INT8 experts) in dynamic LDS next to a small
// static block: above 64 KB in total the launch needs the limit raised once per process.
// LDS of the row-interleaved small-batch kernel for the codes: the whole rows, or one block of them
static size_t g16_tiled_code_bytes(int toks, int K) {
  const size_t all = (size_t)toks * K;
  return all < (size_t)G16_LDS_CODE_BYTES ? all : (size_t)G16_LDS_CODE_BYTES;
}

static size_t ffn_mid_lds_bytes(int F) {
  const int groups = (F + 255) / 256;
  return (size_t)((groups + FFN_MID_PARTS - 1) / FFN_MID_PARTS) * 256 * sizeof(float);
}

static int decode_raise_lds_limits() {
  static std::once_flag once;
  static int rc = PQ_OK;
  std::call_once(once, [] {
    const int lim = 96 * 1024;
    auto set = [&](const void* f) {
      if (rc == PQ_OK && hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lim) != hipSuccess)
        rc = pq_set_error(PQ_ERR_HIP, "hipFuncSetAttribute failed for a decode kernel");
    };
    set((const void*)decode_prep_kernel);
    set((const void*)decode_prep_h_kernel<false>);
    set((const void*)decode_prep_h_kernel<true>);
    set((const void*)decode_ffn_mid_kernel);
  });
  return rc;
}

static int decode_set_gemm16_limits() {
  static std::once_flag once;
  static int rc = PQ_OK;
  std::call_once(once, [] {
    auto set = [&](const void* f) {
      if (rc == PQ_OK && hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
        rc = pq_set_error(PQ_ERR_HIP, "hipFuncSetAttribute failed for a decode kernel");
    };
    set((const void*)decode_gemm16_kernel<8>);
    set((const void*)decode_gemm16_kernel<16>);
    set((const void*)decode_gemm16_tiled_kernel<8>);
    set((const void*)decode_gemm16_tiled_kernel<16>);
    set((const void*)decode_gemm16_tiled_kernel<8, true>);
    set((const void*)decode_gemm16_tiled_kernel<16, true>);
  });
  return rc;
}

// Several tokens per layer (2..16): the same four stages on the small-batch kernels.  The up and gate products are
// 2 L weight sets that read their layer's token block (codes staged once per workgroup), the expert hidden pairs come
// from the per-slot kernel at rank 2 r, the gated unit and the quantiser of Hd run per (layer, token), and the down
// product carries the experts' down projections.
static int launch_decode_ffn_batch(int L, int B, int D, int F, int r, int E, int topk, float alpha, const void* X,
                                   const uint32_t* packed_upgate, const uint16_t* scale_upgate, const uint32_t* packed_down,
                                   const uint16_t* scale_down, const void* UpGate, const void* Down, const void* Wr, void* Y,
                                   int32_t* acc_upgate, void* UG, void* ws1, void* ws2, float* amax_part, hipStream_t s) {
  if (int e = decode_set_gemm16_limits()) return e;
  pq_decode_desc d1{B, D, F, 2 * r, E, topk, L, PQ_PACKED_TILED64, alpha};
  pq_decode_desc d2{B, F, D, r, E, topk, L, PQ_PACKED_TILED64, alpha};
  size_t o1[7], o2[7];
  pq_decode_ws_layout(d1, o1);
  pq_decode_ws_layout(d2, o2);
  char* w1 = (char*)ws1;
  char* w2 = (char*)ws2;
  int8_t* xq1 = (int8_t*)(w1 + o1[0]); uint32_t* pl1 = (uint32_t*)(w1 + o1[1]); int* rs1 = (int*)(w1 + o1[2]);
  float* gm1 = (float*)(w1 + o1[3]); int* idx = (int*)(w1 + o1[4]); float* gate = (float*)(w1 + o1[5]); float* hug = (float*)(w1 + o1[6]);
  int8_t* xq2 = (int8_t*)(w2 + o2[0]); uint32_t* pl2 = (uint32_t*)(w2 + o2[1]); int* rs2 = (int*)(w2 + o2[2]);
  float* gm2 = (float*)(w2 + o2[3]); float* act = (float*)(w2 + o2[6]);
  const int toks = B <= 8 ? 8 : 16;
  {
    pq_prof_scope prof(PQP_DECODE_PREP, s);
    decode_prep_kernel<<<L * B * 2, 256, (size_t)D * sizeof(float), s>>>((const uint16_t*)X, (const uint16_t*)Wr, B, D, E, topk, xq1, pl1, rs1,
                                                                        gm1, idx, gate, rs2);
    PQ_CHECK_LAUNCH("decode_prep_kernel");
  }
  {  // hidden pairs [Up_e x ; Gate_e x] of every (token, selected expert)
    pq_prof_scope prof(PQP_DECODE_H, s);
    const int total = L * B * topk * 2 * r;
    if (!launch_h_grouped((const uint16_t*)X, (const uint16_t*)UpGate, idx, L, B, D, E, 2 * r, topk, hug, s))
      decode_h_kernel<<<(total + 3) / 4, 256, 0, s>>>((const uint16_t*)X, (const uint16_t*)UpGate, idx, B, D, E, 2 * r, topk, total, hug);
    PQ_CHECK_LAUNCH("decode_h_kernel");
  }
  {  // U and G
    pq_prof_scope prof(PQP_DECODE_MAIN, s);
    gemm16_params p{packed_upgate, scale_upgate, xq1, rs1, gm1, nullptr, nullptr, nullptr, nullptr, (uint16_t*)UG, acc_upgate,
                    B, F, D, 0, 0, 0, alpha, nullptr, 2};
    const size_t lds = g16_tiled_code_bytes(toks, D) + 8192;
    dim3 grid(((F + 63) / 64 + 3) / 4, 2 * L);
    if (toks == 8) decode_gemm16_tiled_kernel<8><<<grid, 256, lds, s>>>(p);
    else decode_gemm16_tiled_kernel<16><<<grid, 256, lds, s>>>(p);
    PQ_CHECK_LAUNCH("decode_gemm16_tiled_kernel");
  }
  {
    pq_prof_scope prof(PQP_SWIGLU, s);
    decode_ffn_amax_kernel<<<L * B * FFN_MID_PARTS, 256, 0, s>>>((const uint16_t*)UG, B, F, r, topk, hug, act, amax_part);
    PQ_CHECK_LAUNCH("decode_ffn_amax_kernel");
    decode_ffn_mid_kernel<<<L * B * FFN_MID_PARTS, 256, ffn_mid_lds_bytes(F), s>>>((const uint16_t*)UG, B, F, amax_part, xq2, pl2, rs2, gm2);
    PQ_CHECK_LAUNCH("decode_ffn_mid_kernel");
  }
  {  // down product + experts' down projections
    pq_prof_scope prof(PQP_DECODE_MAIN, s);
    gemm16_params p{packed_down, scale_down, xq2, rs2, gm2, (const uint16_t*)Down, idx, gate, act, (uint16_t*)Y, nullptr,
                    B, D, F, E, r, topk, alpha, nullptr, 1};
    const size_t hm = 2 * (size_t)toks * E * r;
    const size_t lds = g16_tiled_code_bytes(toks, F) + (hm > 8192 ? hm : 8192);
    dim3 grid(((D + 63) / 64 + 3) / 4, L);
    if (toks == 8) decode_gemm16_tiled_kernel<8><<<grid, 256, lds, s>>>(p);
    else decode_gemm16_tiled_kernel<16><<<grid, 256, lds, s>>>(p);
    PQ_CHECK_LAUNCH("decode_gemm16_tiled_kernel");
  }
  return PQ_OK;
}

int pq_launch_decode_ffn(int L, int B, int D, int F, int r, int E, int topk, float alpha, const void* X, const uint32_t* packed_upgate,
                         const uint16_t* scale_upgate, const uint32_t* packed_down, const uint16_t* scale_down,
                         const void* UpGate, const void* Down, const void* Wr, void* Y, int32_t* acc_upgate, void* UG,
                         void* ws1, void* ws2, float* amax_part, hipStream_t s) {
  if (int e = decode_raise_lds_limits()) return e;
  if (B > 1)
    return launch_decode_ffn_batch(L, B, D, F, r, E, topk, alpha, X, packed_upgate, scale_upgate, packed_down, scale_down, UpGate, Down, Wr,
                                   Y, acc_upgate, UG, ws1, ws2, amax_part, s);
  pq_decode_desc d1{1, D, F, 2 * r, E, topk, L, PQ_PACKED_TILED64, alpha};
  pq_decode_desc d2{1, F, D, r, E, topk, L, PQ_PACKED_TILED64, alpha};
  size_t o1[7], o2[7];
  pq_decode_ws_layout(d1, o1);
  pq_decode_ws_layout(d2, o2);
  char* w1 = (char*)ws1;
  char* w2 = (char*)ws2;
  int8_t* xq1 = (int8_t*)(w1 + o1[0]); uint32_t* pl1 = (uint32_t*)(w1 + o1[1]); int* rs1 = (int*)(w1 + o1[2]);
  float* gm1 = (float*)(w1 + o1[3]); int* idx = (int*)(w1 + o1[4]); float* gate = (float*)(w1 + o1[5]); float* hug = (float*)(w1 + o1[6]);
  int8_t* xq2 = (int8_t*)(w2 + o2[0]); uint32_t* pl2 = (uint32_t*)(w2 + o2[1]); int* rs2 = (int*)(w2 + o2[2]);
  float* gm2 = (float*)(w2 + o2[3]); float* act = (float*)(w2 + o2[6]);
  {  // quantiser of x, router, expert hidden pairs [Up_e x ; Gate_e x]
    pq_prof_scope prof(PQP_DECODE_PREP, s);
    const int parts = 1 + (topk * 2 * r + PREP_H_ROWS - 1) / PREP_H_ROWS;
    decode_prep_h_kernel<false><<<L * parts, 256, (size_t)D * sizeof(float), s>>>((const uint16_t*)X, (const uint16_t*)Wr, UpGate, nullptr, D, E,
                                                                                 2 * r, topk, parts, xq1, pl1, rs1, gm1, idx, gate, hug, rs2);
    PQ_CHECK_LAUNCH("decode_prep_h_kernel");
  }
  {  // U and G: 2 L weight sets, each pair reading its layer's token once quantised
    pq_prof_scope prof(PQP_DECODE_MAIN, s);
    gemv_params p{packed_upgate, scale_upgate, pl1, rs1, gm1, nullptr, nullptr, nullptr, nullptr, (uint16_t*)UG, acc_upgate,
                  F, D, E, 0, 0, alpha, nullptr, 2};
    dim3 grid((F + 63) / 64, 2 * L);
    decode_gemv_tiled_kernel<1, false><<<grid, 256, 0, s>>>(p);
    PQ_CHECK_LAUNCH("decode_gemv_tiled_kernel");
  }
  {  // gated unit, quantiser of Hd, experts' gated unit
    pq_prof_scope prof(PQP_SWIGLU, s);
    decode_ffn_amax_kernel<<<L * FFN_MID_PARTS, 256, 0, s>>>((const uint16_t*)UG, 1, F, r, topk, hug, act, amax_part);
    PQ_CHECK_LAUNCH("decode_ffn_amax_kernel");
    decode_ffn_mid_kernel<<<L * FFN_MID_PARTS, 256, ffn_mid_lds_bytes(F), s>>>((const uint16_t*)UG, 1, F, amax_part, xq2, pl2, rs2, gm2);
    PQ_CHECK_LAUNCH("decode_ffn_mid_kernel");
  }
  {  // down product + experts' down projections
    pq_prof_scope prof(PQP_DECODE_MAIN, s);
    gemv_params p{packed_down, scale_down, pl2, rs2, gm2, (const uint16_t*)Down, idx, gate, act, (uint16_t*)Y, nullptr,
                  D, F, E, r, topk, alpha, nullptr, 1};
    dim3 grid((D + 63) / 64, L);
    decode_gemv_tiled_kernel<1, false><<<grid, 256, 0, s>>>(p);
    PQ_CHECK_LAUNCH("decode_gemv_tiled_kernel");
  }
  return PQ_OK;
}

// ------------------------------------------------------------------------------------------
size_t pq_decode_ws_layout(const pq_decode_desc& d, size_t* off /* [7]: xq planes rowsum gamma idx gate h */) {
  const size_t L = d.n_layers, B = d.batch, K = d.d_in;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = pq_align_up(o + bytes, 256); return r; };
  off[0] = take(L * B * K);
  off[1] = take(L * B * 8 * (K / 32) * sizeof(uint32_t));
  off[2] = take(L * B * sizeof(int));
  off[3] = take(L * B * sizeof(float));
  off[4] = take(L * B * (size_t)d.top_k * sizeof(int));
  off[5] = take(L * B * (size_t)d.top_k * sizeof(float));
  off[6] = take(L * B * (size_t)d.top_k * d.hp_rank * sizeof(float));
  return o;
}

int pq_launch_decode(const pq_decode_desc& d, const void* X, const uint32_t* packed, const uint16_t* scale_fp16,
                     const void* hpA, const void* hpB, const void* Wr, void* Y, int32_t* acc_out, void* workspace,
                     hipStream_t s, const float* gA, const float* gB) {
  const bool i8 = gA != nullptr;                      // INT8 experts (the caller has checked the limits)
  if (int e = decode_raise_lds_limits()) return e;
  size_t off[7];
  pq_decode_ws_layout(d, off);
  char* ws = (char*)workspace;
  int8_t* xq = (int8_t*)(ws + off[0]);
  uint32_t* planes = (uint32_t*)(ws + off[1]);
  int* rowsum = (int*)(ws + off[2]);
  float* gamma = (float*)(ws + off[3]);
  int* idx = (int*)(ws + off[4]);
  float* gate = (float*)(ws + off[5]);
  float* h = (float*)(ws + off[6]);
  const int L = d.n_layers, B = d.batch, K = d.d_in, N = d.d_out, r = d.hp_rank, E = r > 0 ? d.n_experts : 0;
  if (B == 1 && r > 0) {
    pq_prof_scope prof(PQP_DECODE_PREP, s);
    const int parts = 1 + (d.top_k * r + PREP_H_ROWS - 1) / PREP_H_ROWS;
    if (i8)
      decode_prep_h_kernel<true><<<L * parts, 256, (size_t)K * 5, s>>>((const uint16_t*)X, (const uint16_t*)Wr, hpA, gA, K, E, r, d.top_k,
                                                                      parts, xq, planes, rowsum, gamma, idx, gate, h, nullptr);
    else
      decode_prep_h_kernel<false><<<L * parts, 256, (size_t)K * sizeof(float), s>>>((const uint16_t*)X, (const uint16_t*)Wr, hpA, nullptr,
                                                                                   K, E, r, d.top_k, parts, xq, planes, rowsum, gamma,
                                                                                   idx, gate, h, nullptr);
    PQ_CHECK_LAUNCH("decode_prep_h_kernel");
  } else {
    {
      pq_prof_scope prof(PQP_DECODE_PREP, s);
      decode_prep_kernel<<<L * B * (E > 0 ? 2 : 1), 256, (size_t)K * sizeof(float), s>>>((const uint16_t*)X, (const uint16_t*)Wr, B, K, E, d.top_k, xq,
                                                                      planes, rowsum, gamma, idx, gate, nullptr);
      PQ_CHECK_LAUNCH("decode_prep_kernel");
    }
    if (r > 0) {
      pq_prof_scope prof(PQP_DECODE_H, s);
      const int total = L * B * d.top_k * r;
      if (i8) {
        decode_h_int8_kernel<<<L * d.n_experts * (r / H8_ROWS), 256, 0, s>>>((const uint16_t*)X, (const int8_t*)hpA, gA, gamma, idx, B, K,
                                                                           d.n_experts, r, d.top_k, h);
      } else
        if (!launch_h_grouped((const uint16_t*)X, (const uint16_t*)hpA, idx, L, B, K, d.n_experts, r, d.top_k, h, s))
          decode_h_kernel<<<(total + 3) / 4, 256, 0, s>>>((const uint16_t*)X, (const uint16_t*)hpA, idx, B, K, d.n_experts, r, d.top_k, total, h);
      PQ_CHECK_LAUNCH("decode_h_kernel");
    }
  }
  pq_prof_scope prof(PQP_DECODE_MAIN, s);
  if (B == 1) {
    gemv_params p{packed, scale_fp16, planes, rowsum, gamma, (const uint16_t*)hpB, idx, gate, h, (uint16_t*)Y, acc_out,
                  N, K, d.n_experts, r, d.top_k, d.alpha, gB};
    if (d.packed_layout == PQ_PACKED_TILED64) {
#ifndef PQ_GEMV_GPB
#define PQ_GEMV_GPB 1
#endif
      dim3 grid(((N + 63) / 64 + PQ_GEMV_GPB - 1) / PQ_GEMV_GPB, L);
      if (i8) decode_gemv_tiled_kernel<PQ_GEMV_GPB, true><<<grid, 256, 0, s>>>(p);
      else decode_gemv_tiled_kernel<PQ_GEMV_GPB, false><<<grid, 256, 0, s>>>(p);
      PQ_CHECK_LAUNCH("decode_gemv_tiled_kernel");
    } else {
      dim3 grid((N + GEMV_ROWS_PER_BLOCK - 1) / GEMV_ROWS_PER_BLOCK, L);
      if (i8) decode_gemv_b1_kernel<true><<<grid, 256, 0, s>>>(p);
      else decode_gemv_b1_kernel<false><<<grid, 256, 0, s>>>(p);
      PQ_CHECK_LAUNCH("decode_gemv_b1_kernel");
    }
  } else {
    gemm16_params p{packed, scale_fp16, xq, rowsum, gamma, (const uint16_t*)hpB, idx, gate, h, (uint16_t*)Y, acc_out,
                    B, N, K, d.n_experts, r, d.top_k, d.alpha, gB, 1};
    const int toks = B <= 8 ? 8 : 16;
    const bool tiled = d.packed_layout == PQ_PACKED_TILED64;
    const size_t hm_bytes = 2 * (size_t)toks * d.n_experts * r;
    const size_t lds = tiled ? g16_tiled_code_bytes(toks, K) + (hm_bytes > 8192 ? hm_bytes : 8192) : (size_t)toks * K + hm_bytes;
    if (int e = decode_set_gemm16_limits()) return e;
    if (tiled) {
      dim3 grid(((N + 63) / 64 + 3) / 4, L);
      if (i8) {
        if (toks == 8) decode_gemm16_tiled_kernel<8, true><<<grid, 256, lds, s>>>(p);
        else decode_gemm16_tiled_kernel<16, true><<<grid, 256, lds, s>>>(p);
      } else {
        if (toks == 8) decode_gemm16_tiled_kernel<8><<<grid, 256, lds, s>>>(p);
        else decode_gemm16_tiled_kernel<16><<<grid, 256, lds, s>>>(p);
      }
    } else {
      if (i8) return pq_set_error(PQ_ERR_SHAPE, "INT8 experts with batch > 1 need the row-interleaved packing");
      dim3 grid((N + G16_ROWS_PER_BLOCK - 1) / G16_ROWS_PER_BLOCK, L);
      if (toks == 8) decode_gemm16_kernel<8><<<grid, 256, lds, s>>>(p);
      else decode_gemm16_kernel<16><<<grid, 256, lds, s>>>(p);
    }
    PQ_CHECK_LAUNCH("decode_gemm16_kernel");
  }
  return PQ_OK;
}

int pq_launch_retile64(const uint32_t* packed, int N, int K, uint32_t* tiled, hipStream_t s) {
  const int nw = K / 32;
  const size_t total = (size_t)((N + 63) / 64) * 64 * nw;
  retile64_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(packed, N, nw, tiled, total);
  PQ_CHECK_LAUNCH("retile64_kernel");
  return PQ_OK;
}
