// Routing bookkeeping and element-wise kernels of the decoupled FFN (Sec. 3.2, 3.3): expert
// histogram and stable permutation, row gather, the gated unit with fused AbsMax re-quantisation,
// expert activation forward/backward, gate/alpha reductions, router backward, scatter-combine.
// All tensors here are bf16 unless noted; every reduction has a fixed order.
#include <mutex>

#include "pq_internal.h"

namespace {

__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xFFFF0000u);
  f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xFFFF0000u);
  f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xFFFF0000u);
  f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xFFFF0000u);
}
__device__ __forceinline__ uint4 pack8(const float* f) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}
// sigmoid through the hardware exponential and reciprocal (about 2 ulp each): with a correctly rounded expf and an IEEE
// division per element the element-wise kernels of the gated unit are bound by their instruction count, not by memory
__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float siluf_(float x) { return x * sigmoidf_(x); }
__device__ __forceinline__ float dsiluf_(float x) {
  const float s = sigmoidf_(x);
  return s * (1.0f + x * (1.0f - s));
}

// Stable counting sort of the slots (slot = token * k + j) by expert: perm[pos] = slot, inv[slot] = pos,
// offsets[e] = first position of expert e.  One workgroup of 16 wavefronts, each owning a contiguous range of whole
// 64-slot batches.  The expert ids (< 64) are first copied into LDS as bytes (LDS_IDS; otherwise both passes read them
// from global memory).  Pass 1: lane e of a wavefront counts expert e in the wavefront's range (one ballot per batch and
// expert).  The counts are scanned over (expert, wavefront), which gives every wavefront the first position of each
// expert's slots inside its range.  Pass 2: the same walk assigns positions in slot order (rank inside a batch by
// ballot prefix), lane e carrying expert e's running position.
template <bool LDS_IDS>
__global__ __launch_bounds__(1024) void route_kernel(const int* __restrict__ idx, int S, int E, int* __restrict__ counts,
                                                     int* __restrict__ offsets, int* __restrict__ perm,
                                                     int* __restrict__ inv) {
  extern __shared__ unsigned char s_ids[];
  __shared__ int s_cnt[16][64], s_off[65];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if constexpr (LDS_IDS) {
    // eight loads per thread in flight (indices clamped, the store conditional): one memory latency per 8192 slots
    for (int s0 = 0; s0 < S; s0 += 8192) {
      int v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = idx[min(s0 + q * 1024 + (int)threadIdx.x, S - 1)];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int s = s0 + q * 1024 + (int)threadIdx.x;
        if (s < S) s_ids[s] = (unsigned char)v[q];
      }
    }
    __syncthreads();
  }
  auto id_at = [&](int s) -> int {
    if (s >= S) return -1;
    if constexpr (LDS_IDS) return s_ids[s];
    else return idx[s];
  };
  const int nb = (S + 63) / 64, per = (nb + 15) / 16;
  const int b0 = min(nb, wave * per), b1 = min(nb, b0 + per);
  int cnt = 0;                                      // lane e: slots of expert e in this wavefront's range
  for (int b = b0; b < b1; ++b) {
    const int id = id_at(b * 64 + lane);
    for (int e = 0; e < E; ++e) {
      const int c = __builtin_popcountll(__ballot(id == e));
      if (lane == e) cnt += c;
    }
  }
  s_cnt[wave][lane] = cnt;
  __syncthreads();
  if (wave == 0) {                                  // lane e: expert e's total, then the exclusive prefix over the experts (E <= 64)
    int tot = 0;
    if (lane < E) {
#pragma unroll
      for (int w = 0; w < 16; ++w) tot += s_cnt[w][lane];
    }
    int incl = tot;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane < E) {
      s_off[lane] = incl - tot;
      offsets[lane] = incl - tot;
      counts[lane] = tot;
    }
    if (lane == E - 1) {
      s_off[E] = incl;
      offsets[E] = incl;
    }
  }
  __syncthreads();
  int running = 0;                                  // lane e: next position of expert e for this wavefront
  if (lane < E) {
    running = s_off[lane];
    for (int w = 0; w < wave; ++w) running += s_cnt[w][lane];
  }
  for (int b = b0; b < b1; ++b) {
    const int s = b * 64 + lane;
    const int id = id_at(s);
    int pos = 0;
    for (int e = 0; e < E; ++e) {
      const unsigned long long m = __ballot(id == e);
      const int base = __builtin_amdgcn_readlane(running, e);   // e is uniform: a scalar read, not a trip through LDS
      if (id == e) pos = base + __builtin_popcountll(m & ((1ull << lane) - 1ull));
      if (lane == e) running += __builtin_popcountll(m);
    }
    // one pair of stores per 64 slots (a store under each expert's branch made the single CU's memory pipe the bottleneck:
    // 2 E store instructions per block and wavefront)
    if (id >= 0) {
      perm[pos] = s;
      inv[s] = pos;
    }
  }
}

// One expert (a single high-precision branch, top-1): what the router and the counting sort produce is known beforehand:
// expert 0 with gate softmax([logit]) = 1 for every token, the identity permutation, one segment of all slots.
__global__ __launch_bounds__(256) void route_single_kernel(int S, int* __restrict__ idx, float* __restrict__ gate, float* __restrict__ probs,
                                                           int* __restrict__ counts, int* __restrict__ offsets, int* __restrict__ perm,
                                                           int* __restrict__ inv) {
  const int s = blockIdx.x * 256 + threadIdx.x;
  if (s == 0) {
    counts[0] = S;
    offsets[0] = 0;
    offsets[1] = S;
  }
  if (s >= S) return;
  idx[s] = 0;
  gate[s] = 1.0f;
  probs[s] = 1.0f;
  perm[s] = s;
  inv[s] = s;
}
__global__ __launch_bounds__(256) void zero_f32_kernel(float* __restrict__ p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.0f;
}

// dst[pos][:] = src[perm[pos] / k][:]   (rows of d bf16, d % 8 == 0), one wavefront per row
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint16_t* __restrict__ src, const int* __restrict__ perm, int k,
                                                          int S, int d, uint16_t* __restrict__ dst) {
  const int pos = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (pos >= S) return;
  const int t = perm[pos] / k;
  const uint4* s4 = reinterpret_cast<const uint4*>(src + (size_t)t * d);
  uint4* d4 = reinterpret_cast<uint4*>(dst + (size_t)pos * d);
  for (int c = lane; c < d / 8; c += 64) d4[c] = s4[c];
}

__global__ __launch_bounds__(256) void gather_f32_kernel(const float* __restrict__ src, const int* __restrict__ perm, int k, int S,
                                                         float* __restrict__ dst) {
  const int pos = blockIdx.x * 256 + threadIdx.x;
  if (pos < S) dst[pos] = src[perm[pos] / k];
}

// ---- the gated unit with fused AbsMax re-quantisation (one wavefront per token) -------------
//   Hd = silu(G) * U in fp32; gamma_h = 128 / max(|Hd|, 1e-5); Hq = codes; Ht = bf16(Hq / gamma_h)
// Rows are F elements apart; only the first Fv columns exist (Fv % 4 == 0): the others are written as zero codes,
// whatever U and G hold there (a width that is not a multiple of 32 is padded, Table 1: 5076 -> 5088).
// All of a row's vectors are requested before the first is used, so a token costs one memory latency.
template <int NV>
__global__ __launch_bounds__(256) void swiglu_quant_kernel(const uint16_t* __restrict__ U, const uint16_t* __restrict__ G,
                                                           int T, int F, int Fv, int8_t* __restrict__ Hq, float* __restrict__ gamma,
                                                           uint16_t* __restrict__ Ht) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  const uint4* u4 = reinterpret_cast<const uint4*>(U + (size_t)t * F);
  const uint4* g4 = reinterpret_cast<const uint4*>(G + (size_t)t * F);
  const int nvec = F / 8;
  float hd[NV > 0 ? NV : 1][8];
  float amax = 0.0f;
  auto gated = [&](const uint4& u, const uint4& g, int c, float* h) {
    float uf[8], gf[8];
    unpack8(u, uf);
    unpack8(g, gf);
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = (c * 8 + j < Fv) ? siluf_(gf[j]) * uf[j] : 0.0f;
  };
  if constexpr (NV > 0) {
    uint4 ur[NV], gr[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      // unconditional (lanes past the end repeat the last vector, which cannot change the maximum): loads under
      // a branch would each get a wait of their own
      const int c = min(i * 64 + lane, nvec - 1);
      ur[i] = u4[c];
      gr[i] = g4[c];
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      gated(ur[i], gr[i], min(i * 64 + lane, nvec - 1), hd[i]);
#pragma unroll
      for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(hd[i][j]));
    }
  } else {
    for (int c = lane; c < nvec; c += 64) {
      float h[8];
      gated(u4[c], g4[c], c, h);
#pragma unroll
      for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(h[j]));
    }
  }
  amax = wave_max(amax);
  const float g = 128.0f / fmaxf(amax, 1e-5f);
  const float ginv = 1.0f / g;                       // q / gamma as q * (1 / gamma): one division per token
  if (lane == 0) gamma[t] = g;
  auto emit = [&](int c, const float* h) {
    int q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = (int)fminf(fmaxf(rintf(__fmul_rn(h[j], g)), -128.0f), 127.0f);
    const uint32_t w0 = (uint32_t)(q[0] & 0xFF) | ((uint32_t)(q[1] & 0xFF) << 8) | ((uint32_t)(q[2] & 0xFF) << 16) | ((uint32_t)(q[3] & 0xFF) << 24);
    const uint32_t w1 = (uint32_t)(q[4] & 0xFF) | ((uint32_t)(q[5] & 0xFF) << 8) | ((uint32_t)(q[6] & 0xFF) << 16) | ((uint32_t)(q[7] & 0xFF) << 24);
    *reinterpret_cast<uint2*>(Hq + (size_t)t * F + (size_t)c * 8) = make_uint2(w0, w1);
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = __fmul_rn((float)q[j], ginv);
    *reinterpret_cast<uint4*>(Ht + (size_t)t * F + (size_t)c * 8) = pack8(o);
  };
  if constexpr (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * 64 + lane;
      if (c < nvec) emit(c, hd[i]);
    }
  } else {
    for (int c = lane; c < nvec; c += 64) {
      float h[8];
      gated(u4[c], g4[c], c, h);
      emit(c, h);
    }
  }
}

// dU = dHd * silu(G), dG = dHd * U * silu'(G)   (element-wise over rows of F elements of which the first Fv exist; the
// others are written as zeros; two vectors of 8 per thread and pass)
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const uint16_t* __restrict__ dHd, const uint16_t* __restrict__ U,
                                                         const uint16_t* __restrict__ G, size_t nvec, int F, int Fv,
                                                         uint16_t* __restrict__ dU, uint16_t* __restrict__ dG) {
  const size_t stride = (size_t)gridDim.x * 256;
  const int vpr = F / 8;                             // vectors per row
  for (size_t c0 = (size_t)blockIdx.x * 256 + threadIdx.x; c0 < nvec; c0 += 2 * stride) {
    const size_t c1 = c0 + stride;
    const bool two = c1 < nvec;
    const size_t cb = two ? c1 : c0;
    const uint4 r0[3] = {reinterpret_cast<const uint4*>(dHd)[c0], reinterpret_cast<const uint4*>(U)[c0], reinterpret_cast<const uint4*>(G)[c0]};
    const uint4 r1[3] = {reinterpret_cast<const uint4*>(dHd)[cb], reinterpret_cast<const uint4*>(U)[cb], reinterpret_cast<const uint4*>(G)[cb]};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (q == 1 && !two) break;
      const size_t c = q ? c1 : c0;
      const int col = (int)(c % (size_t)vpr) * 8;
      float dh[8], uf[8], gf[8], du[8], dg[8];
      unpack8(q ? r1[0] : r0[0], dh);
      unpack8(q ? r1[1] : r0[1], uf);
      unpack8(q ? r1[2] : r0[2], gf);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float sg = sigmoidf_(gf[j]);
        const bool ok = col + j < Fv;
        du[j] = ok ? dh[j] * (gf[j] * sg) : 0.0f;
        dg[j] = ok ? dh[j] * uf[j] * (sg * (1.0f + gf[j] * (1.0f - sg))) : 0.0f;
      }
      reinterpret_cast<uint4*>(dU)[c] = pack8(du);
      reinterpret_cast<uint4*>(dG)[c] = pack8(dg);
    }
  }
}

// ---- expert activation ----------------------------------------------------------------------
// a = silu(ge) * ue  over S rows of r elements (slot order); ue and ge have a row stride of ld elements (r, or 2 r when
// both lie side by side in one [S][2 r] product)
__global__ __launch_bounds__(256) void expert_act_kernel(const uint16_t* __restrict__ ue, const uint16_t* __restrict__ ge,
                                                         int ld, int r, size_t nvec, uint16_t* __restrict__ a) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= nvec) return;
  const size_t pos = c / (size_t)(r / 8), in = pos * ld + (c - pos * (size_t)(r / 8)) * 8;
  float uf[8], gf[8], o[8];
  unpack8(*reinterpret_cast<const uint4*>(ue + in), uf);
  unpack8(*reinterpret_cast<const uint4*>(ge + in), gf);
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = siluf_(gf[j]) * uf[j];
  reinterpret_cast<uint4*>(a)[c] = pack8(o);
}

// with s = alpha * gate[slot]:  du = s da silu(ge), dg = s da ue silu'(ge), as = s a   (r % 8 == 0)
__global__ __launch_bounds__(256) void expert_act_bwd_kernel(const uint16_t* __restrict__ da, const uint16_t* __restrict__ ue,
                                                             const uint16_t* __restrict__ ge, const uint16_t* __restrict__ a,
                                                             const int* __restrict__ perm, const float* __restrict__ gate,
                                                             float alpha, int r, int ld, size_t nvec, uint16_t* __restrict__ du,
                                                             uint16_t* __restrict__ dg, uint16_t* __restrict__ as) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= nvec) return;
  const int pos = (int)(c / (size_t)(r / 8));
  const size_t in = (size_t)pos * ld + (c - (size_t)pos * (r / 8)) * 8;   // ue, ge, du, dg: row stride ld (r or 2 r)
  const float sc = alpha * gate[perm[pos]];
  float d[8], uf[8], gf[8], af[8], o1[8], o2[8], o3[8];
  unpack8(reinterpret_cast<const uint4*>(da)[c], d);
  unpack8(*reinterpret_cast<const uint4*>(ue + in), uf);
  unpack8(*reinterpret_cast<const uint4*>(ge + in), gf);
  unpack8(reinterpret_cast<const uint4*>(a)[c], af);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float dj = sc * d[j];           // upstream of the expert output is alpha * gate * dY
    o1[j] = dj * siluf_(gf[j]);
    o2[j] = dj * uf[j] * dsiluf_(gf[j]);
    o3[j] = sc * af[j];
  }
  *reinterpret_cast<uint4*>(du + in) = pack8(o1);
  *reinterpret_cast<uint4*>(dg + in) = pack8(o2);
  reinterpret_cast<uint4*>(as)[c] = pack8(o3);
}

// Up and Gate of every expert as one matrix: UG[e][j][:] = Up[e][j][:] for j < r, Gate[e][j - r][:] for r <= j < 2 r
// (bf16 rows of d elements, d % 8 == 0), so that both projections are one product with 2 r outputs
__global__ __launch_bounds__(256) void concat_expert_rows_kernel(const uint16_t* __restrict__ up, const uint16_t* __restrict__ gate_w,
                                                                 int r, int d, size_t nvec, uint16_t* __restrict__ ug) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= nvec) return;
  const size_t row = c / (size_t)(d / 8), ch = c - row * (size_t)(d / 8);
  const size_t e = row / (size_t)(2 * r), j = row - e * (size_t)(2 * r);
  const uint16_t* src = j < (size_t)r ? up + (e * r + j) * (size_t)d : gate_w + (e * r + (j - r)) * (size_t)d;
  reinterpret_cast<uint4*>(ug)[c] = reinterpret_cast<const uint4*>(src)[ch];
}
// and back for the gradients (fp32 rows of d elements, d % 4 == 0)
__global__ __launch_bounds__(256) void split_expert_rows_kernel(const float* __restrict__ dug, int r, int d, size_t nvec,
                                                                float* __restrict__ dup, float* __restrict__ dgate) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= nvec) return;
  const size_t row = c / (size_t)(d / 4), ch = c - row * (size_t)(d / 4);
  const size_t e = row / (size_t)(2 * r), j = row - e * (size_t)(2 * r);
  float* dst = j < (size_t)r ? dup + (e * r + j) * (size_t)d : dgate + (e * r + (j - r)) * (size_t)d;
  reinterpret_cast<uint4*>(dst)[ch] = reinterpret_cast<const uint4*>(dug)[c];
}

// rd[pos] = <A[pos,:], B[pos,:]> (fp32), partial[block] = sum gate[perm[pos]] * rd[pos]  (for d alpha)
__global__ __launch_bounds__(256) void rowdot_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Bm,
                                                     const int* __restrict__ perm, const float* __restrict__ gate, int S, int d,
                                                     float* __restrict__ rd, double* __restrict__ partial) {
  __shared__ double red[4];
  const int pos = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  double contrib = 0.0;
  if (pos < S) {
    const uint4* a4 = reinterpret_cast<const uint4*>(A + (size_t)pos * d);
    const uint4* b4 = reinterpret_cast<const uint4*>(Bm + (size_t)pos * d);
    float acc = 0.0f;
    for (int c = lane; c < d / 8; c += 64) {
      float x[8], y[8];
      unpack8(a4[c], x);
      unpack8(b4[c], y);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += x[j] * y[j];
    }
    acc = wave_sum(acc);
    if (lane == 0) {
      rd[pos] = acc;
      contrib = (double)gate[perm[pos]] * (double)acc;
    }
  }
  const double t = block_sum_d<256>(contrib, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

// A[pos,:] *= alpha * gate[perm[pos]]  (rows of d bf16 in slot order, one wavefront per row): the upstream gradient of
// an expert's output for slot (t, j) is alpha * gate[t][j] * dY[t]
__global__ __launch_bounds__(256) void scale_rows_kernel(uint16_t* __restrict__ A, const int* __restrict__ perm,
                                                         const float* __restrict__ gate, float alpha, int S, int d) {
  const int pos = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (pos >= S) return;
  const float sc = alpha * gate[perm[pos]];
  uint4* a4 = reinterpret_cast<uint4*>(A + (size_t)pos * d);
  for (int c = lane; c < d / 8; c += 64) {
    float v[8];
    unpack8(a4[c], v);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= sc;
    a4[c] = pack8(v);
  }
}

// Y[t,:] += alpha * sum_j gate[t,j] * Ys[inv[t*k+j], :]   (one wavefront per token)
__global__ __launch_bounds__(256) void combine_fwd_kernel(uint16_t* __restrict__ Y, const uint16_t* __restrict__ Ys,
                                                          const int* __restrict__ inv, const float* __restrict__ gate, float alpha,
                                                          int T, int k, int d) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  uint4* y4 = reinterpret_cast<uint4*>(Y + (size_t)t * d);
  for (int c = lane; c < d / 8; c += 64) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = 0; j < k; ++j) {
      const float gt = gate[t * k + j];
      float v[8];
      unpack8(reinterpret_cast<const uint4*>(Ys + (size_t)inv[t * k + j] * d)[c], v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += gt * v[i];
    }
    float y[8];
    unpack8(y4[c], y);
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] += alpha * acc[i];
    y4[c] = pack8(y);
  }
}

// dlogit[t,e] = sum_j dgate[t,j] * p[idx_j] * (1[e == idx_j] - p[e]),  dgate[t,j] = alpha * rd[inv[t*k+j]]
__global__ __launch_bounds__(256) void router_bwd_kernel(const float* __restrict__ rd, const int* __restrict__ inv,
                                                         const int* __restrict__ idx, const float* __restrict__ probs, float alpha,
                                                         int T, int k, int E, float* __restrict__ dlogit) {
  const int i = blockIdx.x * 256 + threadIdx.x;   // t * E + e
  if (i >= T * E) return;
  const int t = i / E, e = i % E;
  const float pe = probs[i];
  float acc = 0.0f;
  for (int j = 0; j < k; ++j) {
    const int ej = idx[t * k + j];
    const float dgt = alpha * rd[inv[t * k + j]];
    acc += dgt * probs[t * E + ej] * ((e == ej ? 1.0f : 0.0f) - pe);
  }
  dlogit[i] = acc;
}

// dWr partials: part[tc][e][c] = sum_{t in chunk tc} dlogit[t,e] * X[t,c]   (chunks of 256 tokens).
// A workgroup covers 256 columns of one chunk: thread = (token subgroup sg, column group cg); it walks the
// 32 tokens t0 + sg, t0 + sg + 8, ... with 16-byte loads of 8 columns, then the 8 subgroups are summed in LDS
// in a fixed order.
constexpr int DWR_CHUNK = 128;                      // tokens per workgroup (a multiple of 64)
__global__ __launch_bounds__(256) void dwr_partial_kernel(const float* __restrict__ dlogit, const uint16_t* __restrict__ X, int T,
                                                          int d, int E, float* __restrict__ part) {
  __shared__ float red[8][4][8][32];                 // [subgroup][expert % 4][column % 8][column group]
  __shared__ __attribute__((aligned(16))) float sdl[DWR_CHUNK][8];   // the chunk's dlogit for the eight experts of a pass (zero past E and past T)
  const int tid = threadIdx.x, cg = tid & 31, sg = tid >> 5;
  const int c0 = blockIdx.x * 256 + cg * 8;
  const int t0 = blockIdx.y * DWR_CHUNK;
  const bool okc = c0 < d;                            // d % 8 == 0
  for (int e0 = 0; e0 < E; e0 += 8) {
    // every load below is unconditional (indices clamped into the arrays, the value masked afterwards): a load under
    // a branch waits for its own latency, and the loop over tokens becomes a chain of them
    for (int o = tid; o < DWR_CHUNK * 8; o += 256) {
      const int tt = o >> 3, u = o & 7;
      const float g = dlogit[(size_t)min(t0 + tt, T - 1) * E + min(e0 + u, E - 1)];
      sdl[tt][u] = (t0 + tt < T && e0 + u < E) ? g : 0.0f;
    }
    __syncthreads();
    float acc[8][8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[u][j] = 0.0f;
    if (okc) {
      for (int grp = 0; grp < DWR_CHUNK / 64; ++grp) {   // eight of the subgroup's tokens at a time, their loads issued together
        uint4 xv[8];
#pragma unroll
        for (int q = 0; q < 8; ++q)
          xv[q] = *reinterpret_cast<const uint4*>(X + (size_t)min(t0 + sg + 8 * (8 * grp + q), T - 1) * d + c0);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int tt = sg + 8 * (8 * grp + q);
          const float4 ga = *reinterpret_cast<const float4*>(&sdl[tt][0]), gb = *reinterpret_cast<const float4*>(&sdl[tt][4]);
          const float g[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
          float x[8];
          unpack8(xv[q], x);
#pragma unroll
          for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[u][j] += g[u] * x[j];
        }
      }
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {           // four experts per round through LDS
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j) red[sg][u][j][cg] = acc[4 * half + u][j];
      __syncthreads();
      for (int o = tid; o < 4 * 256; o += 256) {
        const int u = o >> 8, c = o & 255, e = e0 + 4 * half + u;
        if (e < E && blockIdx.x * 256 + c < d) {
          float v = 0.0f;
#pragma unroll
          for (int q = 0; q < 8; ++q) v += red[q][u][c & 7][c >> 3];
          part[((size_t)blockIdx.y * E + e) * d + blockIdx.x * 256 + c] = v;
        }
      }
      __syncthreads();
    }
  }
}
// dWr = the chunks' partial sums added in chunk order (eight loads in flight per thread)
__global__ __launch_bounds__(256) void dwr_final_kernel(const float* __restrict__ part, int nchunks, int n, float* __restrict__ dWr) {
  const int i = blockIdx.x * 256 + threadIdx.x;   // e * d + c
  if (i >= n) return;
  float acc = 0.0f;
  for (int tc = 0; tc < nchunks; tc += 8) {
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = part[(size_t)min(tc + q, nchunks - 1) * n + i];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc += (tc + q < nchunks) ? v[q] : 0.0f;
  }
  dWr[i] = acc;
}

// dX[t,:] += sum_j dXs[inv[t*k+j], :] + sum_e dlogit[t,e] * Wr[e,:]
__global__ __launch_bounds__(256) void combine_bwd_kernel(uint16_t* __restrict__ dX, const uint16_t* __restrict__ dXs,
                                                          const int* __restrict__ inv, const float* __restrict__ dlogit,
                                                          const uint16_t* __restrict__ Wr, int T, int k, int d, int E) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= T) return;
  uint4* x4 = reinterpret_cast<uint4*>(dX + (size_t)t * d);
  for (int c = lane; c < d / 8; c += 64) {
    float acc[8];
    unpack8(x4[c], acc);
    for (int j = 0; j < k; ++j) {
      float v[8];
      unpack8(reinterpret_cast<const uint4*>(dXs + (size_t)inv[t * k + j] * d)[c], v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += v[i];
    }
    for (int e = 0; e < E; ++e) {
      const float dl = dlogit[(size_t)t * E + e];
      float w[8];
      unpack8(reinterpret_cast<const uint4*>(Wr + (size_t)e * d)[c], w);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += dl * w[i];
    }
    x4[c] = pack8(acc);
  }
}

// The same with the router matrix in LDS (E * d bf16 <= 64 KB, E <= 64) and a token's pieces requested together: NC
// 16-byte pieces per lane (d = 512 NC), up to KMAX slots per token; lane e fetches dlogit[t][e] once and hands it round.
// (In the loop above every dlogit and router piece is a load of its own with a wait behind it: 32 cache round trips
// per lane and token at 8 experts.)  A workgroup takes CB_TOK tokens per wavefront, so the router matrix is staged once
// per 4 * CB_TOK tokens.  Same sums in the same order as above.
constexpr int CB_TOK = 4;
template <int NC, int KMAX>
__global__ __launch_bounds__(256) void combine_bwd_lds_kernel(uint16_t* __restrict__ dX, const uint16_t* __restrict__ dXs,
                                                              const int* __restrict__ inv, const float* __restrict__ dlogit,
                                                              const uint16_t* __restrict__ Wr, int T, int k, int E) {
  extern __shared__ __attribute__((aligned(16))) unsigned char wr_s[];   // [E][d] bf16
  constexpr int d = 512 * NC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  {
    const int nvec = E * d / 8;
    for (int c = threadIdx.x; c < nvec; c += 256) reinterpret_cast<uint4*>(wr_s)[c] = reinterpret_cast<const uint4*>(Wr)[c];
  }
  __syncthreads();
  for (int q = 0; q < CB_TOK; ++q) {
    const int t = (blockIdx.x * 4 + wave) * CB_TOK + q;
    if (t >= T) break;                                // wave-uniform
    int pos[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) pos[j] = inv[t * k + min(j, k - 1)];
    const float dlv = lane < E ? dlogit[(size_t)t * E + lane] : 0.0f;
    uint4* x4 = reinterpret_cast<uint4*>(dX + (size_t)t * d) + lane;
    uint4 xv[NC], sv[KMAX][NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) xv[i] = x4[64 * i];
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
#pragma unroll
      for (int i = 0; i < NC; ++i) sv[j][i] = reinterpret_cast<const uint4*>(dXs + (size_t)pos[j] * d)[lane + 64 * i];
    float acc[NC][8];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      unpack8(xv[i], acc[i]);
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {
        if (j < k) {
          float v[8];
          unpack8(sv[j][i], v);
#pragma unroll
          for (int u = 0; u < 8; ++u) acc[i][u] += v[u];
        }
      }
    }
    for (int e = 0; e < E; ++e) {
      const float dl = __shfl(dlv, e);
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        float w[8];
        unpack8(reinterpret_cast<const uint4*>(wr_s + (size_t)e * d * 2)[lane + 64 * i], w);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[i][u] += dl * w[u];
      }
    }
#pragma unroll
    for (int i = 0; i < NC; ++i) x4[64 * i] = pack8(acc[i]);
  }
}

// out = sum_i c[i] * x[i]  (up to 4 bf16 tensors, fp32 arithmetic, one rounding): the glue between
// the linears of a layer stack (residual adds, the stand-in for the attention core)
__global__ __launch_bounds__(256) void lincomb_kernel(uint16_t* __restrict__ out, const uint16_t* x0, const uint16_t* x1,
                                                      const uint16_t* x2, const uint16_t* x3, float c0, float c1, float c2,
                                                      float c3, size_t nvec) {
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < nvec; c += (size_t)gridDim.x * 256) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, v[8];
    unpack8(reinterpret_cast<const uint4*>(x0)[c], v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = c0 * v[j];
    if (x1) {
      unpack8(reinterpret_cast<const uint4*>(x1)[c], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += c1 * v[j];
    }
    if (x2) {
      unpack8(reinterpret_cast<const uint4*>(x2)[c], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += c2 * v[j];
    }
    if (x3) {
      unpack8(reinterpret_cast<const uint4*>(x3)[c], v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += c3 * v[j];
    }
    reinterpret_cast<uint4*>(out)[c] = pack8(acc);
  }
}

}  // namespace

int pq_launch_lincomb(void* out, const void* x0, const void* x1, const void* x2, const void* x3, float c0, float c1, float c2,
                      float c3, size_t n, hipStream_t s) {
  if (n == 0) return PQ_OK;
  pq_prof_scope prof(PQP_GLUE, s);
  const size_t nvec = n / 8;
  size_t blocks = (nvec + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  lincomb_kernel<<<(unsigned)blocks, 256, 0, s>>>((uint16_t*)out, (const uint16_t*)x0, (const uint16_t*)x1, (const uint16_t*)x2,
                                                 (const uint16_t*)x3, c0, c1, c2, c3, nvec);
  PQ_CHECK_LAUNCH("lincomb_kernel");
  return PQ_OK;
}

// ---------------------------------------------------------------------------------------------
int pq_launch_route(const int* idx, int S, int E, int* counts, int* offsets, int* perm, int* inv, hipStream_t s) {
  pq_prof_scope prof(PQP_MOE_ROUTE, s);
  if (S <= 96 * 1024) {
    static std::once_flag once;
    static int rc = PQ_OK;
    std::call_once(once, [] {
      if (hipFuncSetAttribute((const void*)route_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024) != hipSuccess)
        rc = pq_set_error(PQ_ERR_HIP, "hipFuncSetAttribute failed for route_kernel");
    });
    if (rc != PQ_OK) return rc;
    route_kernel<true><<<1, 1024, (size_t)((S + 15) / 16 * 16), s>>>(idx, S, E, counts, offsets, perm, inv);
  } else {
    route_kernel<false><<<1, 1024, 0, s>>>(idx, S, E, counts, offsets, perm, inv);
  }
  PQ_CHECK_LAUNCH("route_kernel");
  return PQ_OK;
}

int pq_launch_route_single(int S, int* idx, float* gate, float* probs, int* counts, int* offsets, int* perm, int* inv, hipStream_t s) {
  pq_prof_scope prof(PQP_MOE_ROUTE, s);
  route_single_kernel<<<(S + 256) / 256, 256, 0, s>>>(S, idx, gate, probs, counts, offsets, perm, inv);
  PQ_CHECK_LAUNCH("route_single_kernel");
  return PQ_OK;
}

int pq_launch_zero_f32(float* p, size_t n, hipStream_t s) {
  if (n == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  zero_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(p, n);
  PQ_CHECK_LAUNCH("zero_f32_kernel");
  return PQ_OK;
}

int pq_launch_gather_rows(const void* src, const int* perm, int k, int S, int d, void* dst, hipStream_t s) {
  if (S == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  gather_rows_kernel<<<(S + 3) / 4, 256, 0, s>>>((const uint16_t*)src, perm, k, S, d, (uint16_t*)dst);
  PQ_CHECK_LAUNCH("gather_rows_kernel");
  return PQ_OK;
}

int pq_launch_gather_f32(const float* src, const int* perm, int k, int S, float* dst, hipStream_t s) {
  if (S == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  gather_f32_kernel<<<(S + 255) / 256, 256, 0, s>>>(src, perm, k, S, dst);
  PQ_CHECK_LAUNCH("gather_f32_kernel");
  return PQ_OK;
}

int pq_launch_swiglu_quant(const void* U, const void* G, int T, int F, int Fv, int8_t* Hq, float* gamma, void* Ht, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_SWIGLU, s);
  const int per_lane = (F / 8 + 63) / 64;
  dim3 grid((T + 3) / 4), block(256);
  const uint16_t* u = (const uint16_t*)U;
  const uint16_t* g = (const uint16_t*)G;
  if (per_lane <= 4) swiglu_quant_kernel<4><<<grid, block, 0, s>>>(u, g, T, F, Fv, Hq, gamma, (uint16_t*)Ht);
  else if (per_lane <= 12) swiglu_quant_kernel<12><<<grid, block, 0, s>>>(u, g, T, F, Fv, Hq, gamma, (uint16_t*)Ht);
  else swiglu_quant_kernel<0><<<grid, block, 0, s>>>(u, g, T, F, Fv, Hq, gamma, (uint16_t*)Ht);
  PQ_CHECK_LAUNCH("swiglu_quant_kernel");
  return PQ_OK;
}

int pq_launch_swiglu_bwd(const void* dHd, const void* U, const void* G, int T, int F, int Fv, void* dU, void* dG, hipStream_t s) {
  const size_t n = (size_t)T * F;
  if (n == 0) return PQ_OK;
  pq_prof_scope prof(PQP_SWIGLU, s);
  const size_t nvec = n / 8;
  size_t blocks = (nvec + 511) / 512;                // two vectors per thread and pass
  if (blocks > 8192) blocks = 8192;
  swiglu_bwd_kernel<<<(unsigned)blocks, 256, 0, s>>>((const uint16_t*)dHd, (const uint16_t*)U, (const uint16_t*)G, nvec, F, Fv,
                                                    (uint16_t*)dU, (uint16_t*)dG);
  PQ_CHECK_LAUNCH("swiglu_bwd_kernel");
  return PQ_OK;
}

int pq_launch_expert_act(const void* ue, const void* ge, int ld, int S, int r, void* a, hipStream_t s) {
  const size_t n = (size_t)S * r;
  if (n == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  expert_act_kernel<<<(unsigned)((n / 8 + 255) / 256), 256, 0, s>>>((const uint16_t*)ue, (const uint16_t*)ge, ld, r, n / 8, (uint16_t*)a);
  PQ_CHECK_LAUNCH("expert_act_kernel");
  return PQ_OK;
}

int pq_launch_concat_expert_rows(const void* up, const void* gate_w, int E, int r, int d, void* ug, hipStream_t s) {
  const size_t nvec = (size_t)E * 2 * r * (d / 8);
  if (nvec == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  concat_expert_rows_kernel<<<(unsigned)((nvec + 255) / 256), 256, 0, s>>>((const uint16_t*)up, (const uint16_t*)gate_w, r, d, nvec, (uint16_t*)ug);
  PQ_CHECK_LAUNCH("concat_expert_rows_kernel");
  return PQ_OK;
}

int pq_launch_split_expert_rows(const float* dug, int E, int r, int d, float* dup, float* dgate, hipStream_t s) {
  const size_t nvec = (size_t)E * 2 * r * (d / 4);
  if (nvec == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  split_expert_rows_kernel<<<(unsigned)((nvec + 255) / 256), 256, 0, s>>>(dug, r, d, nvec, dup, dgate);
  PQ_CHECK_LAUNCH("split_expert_rows_kernel");
  return PQ_OK;
}

int pq_launch_expert_act_bwd(const void* da, const void* ue, const void* ge, const void* a, const int* perm, const float* gate,
                             float alpha, int S, int r, int ld, void* du, void* dg, void* as, hipStream_t s) {
  if (S == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  const size_t nvec = (size_t)S * r / 8;
  expert_act_bwd_kernel<<<(unsigned)((nvec + 255) / 256), 256, 0, s>>>((const uint16_t*)da, (const uint16_t*)ue, (const uint16_t*)ge,
                                                                      (const uint16_t*)a, perm, gate, alpha, r, ld, nvec, (uint16_t*)du,
                                                                      (uint16_t*)dg, (uint16_t*)as);
  PQ_CHECK_LAUNCH("expert_act_bwd_kernel");
  return PQ_OK;
}

int pq_launch_scale_rows(void* A, const int* perm, const float* gate, float alpha, int S, int d, hipStream_t s) {
  if (S <= 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  scale_rows_kernel<<<(S + 3) / 4, 256, 0, s>>>((uint16_t*)A, perm, gate, alpha, S, d);
  PQ_CHECK_LAUNCH("scale_rows_kernel");
  return PQ_OK;
}

int pq_rowdot_blocks(int S) { return (S + 3) / 4; }
int pq_launch_rowdot(const void* A, const void* B, const int* perm, const float* gate, int S, int d, float* rd, double* partial,
                     hipStream_t s) {
  if (S == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  rowdot_kernel<<<(S + 3) / 4, 256, 0, s>>>((const uint16_t*)A, (const uint16_t*)B, perm, gate, S, d, rd, partial);
  PQ_CHECK_LAUNCH("rowdot_kernel");
  return PQ_OK;
}

int pq_launch_combine_fwd(void* Y, const void* Ys, const int* inv, const float* gate, float alpha, int T, int k, int d, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  combine_fwd_kernel<<<(T + 3) / 4, 256, 0, s>>>((uint16_t*)Y, (const uint16_t*)Ys, inv, gate, alpha, T, k, d);
  PQ_CHECK_LAUNCH("combine_fwd_kernel");
  return PQ_OK;
}

int pq_launch_router_bwd(const float* rd, const int* inv, const int* idx, const float* probs, float alpha, int T, int k, int E,
                         float* dlogit, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  router_bwd_kernel<<<(T * E + 255) / 256, 256, 0, s>>>(rd, inv, idx, probs, alpha, T, k, E, dlogit);
  PQ_CHECK_LAUNCH("router_bwd_kernel");
  return PQ_OK;
}

size_t pq_dwr_scratch_bytes(int T, int d, int E) { return (size_t)((T + DWR_CHUNK - 1) / DWR_CHUNK) * E * d * sizeof(float); }
int pq_launch_dwr(const float* dlogit, const void* X, int T, int d, int E, float* part, float* dWr, hipStream_t s) {
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  const int nchunks = (T + DWR_CHUNK - 1) / DWR_CHUNK;
  if (nchunks > 0) {
    dim3 grid((d + 255) / 256, nchunks);
    dwr_partial_kernel<<<grid, 256, 0, s>>>(dlogit, (const uint16_t*)X, T, d, E, part);
    PQ_CHECK_LAUNCH("dwr_partial_kernel");
  }
  dwr_final_kernel<<<(E * d + 255) / 256, 256, 0, s>>>(part, nchunks, E * d, dWr);
  PQ_CHECK_LAUNCH("dwr_final_kernel");
  return PQ_OK;
}

int pq_launch_combine_bwd(void* dX, const void* dXs, const int* inv, const float* dlogit, const void* Wr, int T, int k, int d, int E,
                          hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_MOE_ELEMENTWISE, s);
  const size_t wr_bytes = (size_t)E * d * 2;
  const int grid_l = (T + 4 * CB_TOK - 1) / (4 * CB_TOK);
  if (E > 0 && E <= 64 && k <= 2 && wr_bytes <= 64 * 1024 && d == 2048)
    combine_bwd_lds_kernel<4, 2><<<grid_l, 256, wr_bytes, s>>>((uint16_t*)dX, (const uint16_t*)dXs, inv, dlogit, (const uint16_t*)Wr, T, k, E);
  else if (E > 0 && E <= 64 && k <= 2 && wr_bytes <= 64 * 1024 && d == 4096)
    combine_bwd_lds_kernel<8, 2><<<grid_l, 256, wr_bytes, s>>>((uint16_t*)dX, (const uint16_t*)dXs, inv, dlogit, (const uint16_t*)Wr, T, k, E);
  else
    combine_bwd_kernel<<<(T + 3) / 4, 256, 0, s>>>((uint16_t*)dX, (const uint16_t*)dXs, inv, dlogit, (const uint16_t*)Wr, T, k, d, E);
  PQ_CHECK_LAUNCH("combine_bwd_kernel");
  return PQ_OK;
}
