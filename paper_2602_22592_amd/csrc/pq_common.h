// Shared device/host helpers of libpquant (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/pquant.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) int i32x16_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;

#define PQ_WAVE 64

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even float -> bf16 bits (finite inputs; NaN stays NaN through the hardware cast)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Stores with an optional non-temporal hint, for results that are written once and not re-read before they
// would have left the caches anyway.  Measured on a stream of fresh buffers the hint raises the write rate by
// about 40 %; inside a training step, where the next kernel re-reads a result out of the last-level cache,
// plain stores are the better choice, so the hint is a per-call-site decision.
typedef uint32_t pq_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t pq_u32x2_t __attribute__((ext_vector_type(2)));
template <bool NT>
__device__ __forceinline__ void pq_st16(void* p, const uint4& v) {
  if constexpr (NT) __builtin_nontemporal_store(pq_u32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<pq_u32x4_t*>(p));
  else *reinterpret_cast<uint4*>(p) = v;
}
template <bool NT>
__device__ __forceinline__ void pq_st8(void* p, const uint2& v) {
  if constexpr (NT) __builtin_nontemporal_store(pq_u32x2_t{v.x, v.y}, reinterpret_cast<pq_u32x2_t*>(p));
  else *reinterpret_cast<uint2*>(p) = v;
}

template <typename T> struct io_traits;
template <> struct io_traits<float> {
  static __device__ __forceinline__ float load(const float* p, size_t i) { return p[i]; }
  static __device__ __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct io_traits<uint16_t> {  // bf16 bit patterns
  static __device__ __forceinline__ float load(const uint16_t* p, size_t i) { return bf16_to_f32(p[i]); }
  static __device__ __forceinline__ void store(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Block-wide sum in a fixed order (deterministic): wave sums, then wave 0 adds them in index order.
template <int NT>
__device__ __forceinline__ double block_sum_d(double v, double* smem /* NT/64 doubles */) {
  v = wave_sum_d(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  if (l == 0) smem[w] = v;
  __syncthreads();
  double s = 0.0;
  if (threadIdx.x == 0) {
    for (int i = 0; i < NT / 64; ++i) s += smem[i];
  }
  __syncthreads();
  return s;  // valid in thread 0 only
}

// Host-side error plumbing (defined in pq_api.hip)
int pq_set_error(int code, const char* fmt, ...);
#define PQ_CHECK_HIP(expr)                                                              \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) return pq_set_error(PQ_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)
#define PQ_CHECK_LAUNCH(name)                                                           \
  do {                                                                                  \
    hipError_t e_ = hipGetLastError();                                                  \
    if (e_ != hipSuccess) return pq_set_error(PQ_ERR_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
  } while (0)

static inline size_t pq_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Sum of the fp32 slabs of a split contraction in slab order, rounded to bf16: C[m][n .. n+7] for the idx-th group of
// eight columns (the plain epilogue C = acc of the GEMM engine's own reduction, bit for bit).
__device__ __forceinline__ void pq_slab_sum_bf16_body(const float* __restrict__ part, int splits, int M, int N, uint16_t* __restrict__ C,
                                                      int ldc, size_t idx) {
  const size_t n8 = (size_t)N / 8, total = (size_t)M * n8;
  if (idx >= total) return;
  const int m = (int)(idx / n8), n = (int)(idx % n8) * 8;
  const size_t slab = (size_t)M * N;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
  for (int z = 0; z < splits; z += 4) {
    float4 x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* p = part + (size_t)min(z + u, splits - 1) * slab + (size_t)m * N + n;
      x[u] = *reinterpret_cast<const float4*>(p);
      y[u] = *reinterpret_cast<const float4*>(p + 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (z + u < splits) {
        a.x += x[u].x; a.y += x[u].y; a.z += x[u].z; a.w += x[u].w;
        b.x += y[u].x; b.y += y[u].y; b.z += y[u].z; b.w += y[u].w;
      }
  }
  *reinterpret_cast<uint4*>(C + (size_t)m * ldc + n) =
      make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y), pack_bf16x2(b.z, b.w));
}

// Fixed-order final reduction of per-block fp64 partial sums to one fp32 value: out = (sum partials) * factor [* *dev_factor].
// One workgroup of 256 threads per job.
struct pq_reduce_job { const double* partials; int n; float factor; const float* dev_factor; float* out; };
__device__ __forceinline__ void pq_reduce_job_body(const pq_reduce_job& j) {
  __shared__ double red[4];
  double s = 0.0;
  for (int i = threadIdx.x; i < j.n; i += 256) s += j.partials[i];
  double t = block_sum_d<256>(s, red);
  if (threadIdx.x == 0) {
    double f = (double)j.factor;
    if (j.dev_factor) f *= (double)(*j.dev_factor);
    j.out[0] = (float)(t * f);
  }
}
