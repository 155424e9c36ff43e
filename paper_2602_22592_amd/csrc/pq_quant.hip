// Bandwidth-bound element kernels: AbsMax INT8 activation quantiser (Sec. 3.1), weight statistics
// mu/lambda and the sign binariser/packer (Sec. 3.1, App. A), the router (Sec. 3.3).
#include <mutex>
#include "pq_internal.h"

// ------------------------------------------------------------------------------------------
// Activation quantiser: one wavefront per token.  The row is read once from HBM into registers
// (16 B per lane per step), the wave reduces |x| with cross-lane shuffles, then each lane
// quantises what it holds.  Rows too long for the register cache are re-read (second read hits L2).
// ------------------------------------------------------------------------------------------
template <typename T> struct vec16;  // 16 bytes of T
template <> struct vec16<float> {
  static constexpr int V = 4;
  static __device__ __forceinline__ void unpack(const uint4& u, float* f) {
    f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
    f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
  }
};
template <> struct vec16<uint16_t> {
  static constexpr int V = 8;
  static __device__ __forceinline__ void unpack(const uint4& u, float* f) {
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xFFFF0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xFFFF0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xFFFF0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xFFFF0000u);
  }
};

__device__ __forceinline__ int quant_code(float x, float g) {
  float y = __fmul_rn(x, g);                       // one fp32 product, no contraction
  float r = rintf(y);                              // round half to even
  r = fminf(fmaxf(r, -128.0f), 127.0f);
  return (int)r;
}

template <typename T, bool NT = false>
__device__ __forceinline__ void quant_store(const uint4& u, float g, int8_t* qrow, uint16_t* xtrow,
                                            int c) {
  constexpr int V = vec16<T>::V;
  float f[V];
  vec16<T>::unpack(u, f);
  int q[V];
#pragma unroll
  for (int j = 0; j < V; ++j) q[j] = quant_code(f[j], g);
  uint32_t w[V / 4];
#pragma unroll
  for (int j = 0; j < V / 4; ++j)
    w[j] = (uint32_t)(q[4 * j] & 0xFF) | ((uint32_t)(q[4 * j + 1] & 0xFF) << 8) |
           ((uint32_t)(q[4 * j + 2] & 0xFF) << 16) | ((uint32_t)(q[4 * j + 3] & 0xFF) << 24);
  if constexpr (V == 8) {
    pq_st8<NT>(qrow + (size_t)c * 8, make_uint2(w[0], w[1]));
  } else {
    *reinterpret_cast<uint32_t*>(qrow + (size_t)c * 4) = w[0];
  }
  if (xtrow) {
    uint32_t o[V / 2];
#pragma unroll
    for (int j = 0; j < V / 2; ++j)
      o[j] = pack_bf16x2((float)q[2 * j] / g, (float)q[2 * j + 1] / g);
    if constexpr (V == 8) {
      pq_st16<NT>(xtrow + (size_t)c * 8, make_uint4(o[0], o[1], o[2], o[3]));
    } else {
      pq_st8<NT>(xtrow + (size_t)c * 4, make_uint2(o[0], o[1]));
    }
  }
}

template <typename T, int NV>
__device__ __forceinline__ void quant_act_body(const T* __restrict__ X, int Tn, int K, int8_t* __restrict__ Xq,
                                               float* __restrict__ gamma, uint16_t* __restrict__ Xt, int block) {
  constexpr int V = vec16<T>::V;
  const int lane = threadIdx.x & 63;
  const int row = block * 4 + (threadIdx.x >> 6);
  if (row >= Tn) return;
  const uint4* xr = reinterpret_cast<const uint4*>(X + (size_t)row * K);
  const int nvec = K / V;
  float amax = 0.0f;
  uint4 cache[NV > 0 ? NV : 1];
  if constexpr (NV > 0) {
    // unconditional loads (lanes past the end re-read the last vector, which cannot change the maximum): a load
    // under a branch gets a wait of its own and the row would arrive one memory latency per vector
#pragma unroll
    for (int i = 0; i < NV; ++i) cache[i] = xr[min(i * 64 + lane, nvec - 1)];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float f[V];
      vec16<T>::unpack(cache[i], f);
#pragma unroll
      for (int j = 0; j < V; ++j) amax = fmaxf(amax, fabsf(f[j]));
    }
  } else {
    for (int c = lane; c < nvec; c += 64) {
      uint4 u = xr[c];
      float f[V];
      vec16<T>::unpack(u, f);
#pragma unroll
      for (int j = 0; j < V; ++j) amax = fmaxf(amax, fabsf(f[j]));
    }
  }
  amax = wave_max(amax);
  const float g = 128.0f / fmaxf(amax, 1e-5f);     // IEEE fp32 division (no fast-math in this build)
  if (lane == 0) gamma[row] = g;
  int8_t* qrow = Xq + (size_t)row * K;
  uint16_t* xtrow = Xt ? Xt + (size_t)row * K : nullptr;
  if constexpr (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int c = i * 64 + lane;
      if (c < nvec) quant_store<T>(cache[i], g, qrow, xtrow, c);
    }
  } else {
    for (int c = lane; c < nvec; c += 64) quant_store<T>(xr[c], g, qrow, xtrow, c);
  }
}

template <typename T, int NV>
__global__ __launch_bounds__(256) void quant_act_kernel(const T* __restrict__ X, int Tn, int K,
                                                        int8_t* __restrict__ Xq,
                                                        float* __restrict__ gamma,
                                                        uint16_t* __restrict__ Xt) {
  quant_act_body<T, NV>(X, Tn, K, Xq, gamma, Xt, blockIdx.x);
}

template <typename T>
static int launch_quant_t(const T* X, int Tn, int K, int8_t* Xq, float* gamma, uint16_t* Xt,
                          hipStream_t s) {
  constexpr int V = vec16<T>::V;
  const int per_lane = (K / V + 63) / 64;
  dim3 grid((Tn + 3) / 4), block(256);
  if (per_lane <= 4) quant_act_kernel<T, 4><<<grid, block, 0, s>>>(X, Tn, K, Xq, gamma, Xt);
  else if (per_lane <= 8) quant_act_kernel<T, 8><<<grid, block, 0, s>>>(X, Tn, K, Xq, gamma, Xt);
  else if (per_lane <= 16) quant_act_kernel<T, 16><<<grid, block, 0, s>>>(X, Tn, K, Xq, gamma, Xt);
  else quant_act_kernel<T, 0><<<grid, block, 0, s>>>(X, Tn, K, Xq, gamma, Xt);
  PQ_CHECK_LAUNCH("quant_act_kernel");
  return PQ_OK;
}

int pq_launch_quant_act(const void* X, int dtype, int T, int K, int8_t* Xq, float* gamma,
                        uint16_t* Xt, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_QUANT, s);
  if (dtype == PQ_F32) return launch_quant_t<float>((const float*)X, T, K, Xq, gamma, Xt, s);
  return launch_quant_t<uint16_t>((const uint16_t*)X, T, K, Xq, gamma, Xt, s);
}

// ------------------------------------------------------------------------------------------
// RMSNorm fused with the AbsMax quantiser (Sec. 3.1: Q(Norm(X)); App. A: both are element-wise per token
// and merge; App. B: RMSNorm).  One wavefront per token, the row stays in registers between the three
// steps: sum of squares (fp64, so that rstd does not depend on the order of the sum beyond its last fp64
// bit), x_hat = fl(fl(x rstd) g) rounded to the I/O type, then the quantiser of the stored x_hat.
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ uint4 pack_io(const float* f);
template <>
__device__ __forceinline__ uint4 pack_io<float>(const float* f) {
  return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
template <>
__device__ __forceinline__ uint4 pack_io<uint16_t>(const float* f) {
  return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_quant_kernel(const T* __restrict__ X, const T* __restrict__ gain, int Tn, int K,
                                                            float eps, T* __restrict__ Xn, int8_t* __restrict__ Xq,
                                                            float* __restrict__ gamma, uint16_t* __restrict__ Xt,
                                                            float* __restrict__ rstd_out) {
  constexpr int V = vec16<T>::V;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Tn) return;
  const uint4* xr = reinterpret_cast<const uint4*>(X + (size_t)row * K);
  const uint4* gr = reinterpret_cast<const uint4*>(gain);
  const int nvec = K / V;
  uint4 cache[NV], gc[NV];
  double ss = 0.0;
  // unconditional loads (clamped index) so that all of them are in flight together
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int cc = min(i * 64 + lane, nvec - 1);
    cache[i] = xr[cc];
    gc[i] = gr[cc];
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if (i * 64 + lane < nvec) {
      float f[V];
      vec16<T>::unpack(cache[i], f);
#pragma unroll
      for (int j = 0; j < V; ++j) ss += (double)f[j] * (double)f[j];
    }
  }
  ss = wave_sum_d(ss);
  const float r = (float)(1.0 / sqrt(ss / (double)K + (double)eps));
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) {
      float f[V], g[V];
      vec16<T>::unpack(cache[i], f);
      vec16<T>::unpack(gc[i], g);
#pragma unroll
      for (int j = 0; j < V; ++j) f[j] = __fmul_rn(__fmul_rn(f[j], r), g[j]);
      cache[i] = pack_io<T>(f);                      // the stored x_hat; everything below reads it back
      vec16<T>::unpack(cache[i], f);
#pragma unroll
      for (int j = 0; j < V; ++j) amax = fmaxf(amax, fabsf(f[j]));
      if (Xn) pq_st16<true>(reinterpret_cast<uint4*>(Xn + (size_t)row * K) + c, cache[i]);
    }
  }
  amax = wave_max(amax);
  const float g = 128.0f / fmaxf(amax, 1e-5f);
  if (lane == 0) {
    gamma[row] = g;
    if (rstd_out) rstd_out[row] = r;
  }
  int8_t* qrow = Xq + (size_t)row * K;
  uint16_t* xtrow = Xt ? Xt + (size_t)row * K : nullptr;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) quant_store<T, true>(cache[i], g, qrow, xtrow, c);
  }
}

template <typename T>
static int launch_rmsnorm_quant_t(const T* X, const T* gain, int Tn, int K, float eps, T* Xn, int8_t* Xq, float* gamma,
                                  uint16_t* Xt, float* rstd, hipStream_t s) {
  constexpr int V = vec16<T>::V;
  const int per_lane = (K / V + 63) / 64;
  dim3 grid((Tn + 3) / 4), block(256);
  if (per_lane <= 4) rmsnorm_quant_kernel<T, 4><<<grid, block, 0, s>>>(X, gain, Tn, K, eps, Xn, Xq, gamma, Xt, rstd);
  else if (per_lane <= 8) rmsnorm_quant_kernel<T, 8><<<grid, block, 0, s>>>(X, gain, Tn, K, eps, Xn, Xq, gamma, Xt, rstd);
  else if (per_lane <= 16) rmsnorm_quant_kernel<T, 16><<<grid, block, 0, s>>>(X, gain, Tn, K, eps, Xn, Xq, gamma, Xt, rstd);
  else return pq_set_error(PQ_ERR_SHAPE, "row of %d elements does not fit the register cache of the fused normalising quantiser", K);
  PQ_CHECK_LAUNCH("rmsnorm_quant_kernel");
  return PQ_OK;
}

int pq_launch_rmsnorm_quant(const void* X, const void* gain, int dtype, int T, int K, float eps, void* Xn, int8_t* Xq,
                            float* gamma, uint16_t* Xt, float* rstd, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_NORM_QUANT, s);
  if (dtype == PQ_F32)
    return launch_rmsnorm_quant_t<float>((const float*)X, (const float*)gain, T, K, eps, (float*)Xn, Xq, gamma, Xt, rstd, s);
  return launch_rmsnorm_quant_t<uint16_t>((const uint16_t*)X, (const uint16_t*)gain, T, K, eps, (uint16_t*)Xn, Xq, gamma, Xt, rstd, s);
}

// Backward of the normalisation (the quantiser is passed straight through, App. B.1): with u = x rstd,
//   dx = rstd (g dxn - u mean_k(g dxn u)),   dg[k] = sum_t dxn[t][k] u[t][k].
// A wavefront walks NORM_BWD_TPW tokens and keeps its share of dg in registers; the four wavefronts of a
// workgroup add their shares through LDS into one partial row, and a second kernel adds the partial rows in a
// fixed order (fp64), so the result is the same on every run.
constexpr int NORM_BWD_TPW = 4;                    // tokens per wavefront
constexpr int NORM_BWD_TPB = 4 * NORM_BWD_TPW;     // tokens per workgroup = per partial row of dgain

template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ dXn, const T* __restrict__ X,
                                                          const T* __restrict__ gain, const float* __restrict__ rstd, int Tn,
                                                          int K, T* __restrict__ dX, float* __restrict__ part) {
  constexpr int V = vec16<T>::V;
  extern __shared__ __attribute__((aligned(16))) float dsh[];   // [3][K]: the dgain shares of wavefronts 1..3
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * NORM_BWD_TPB + wave * NORM_BWD_TPW;
  const int nvec = K / V;
  const uint4* gr = reinterpret_cast<const uint4*>(gain);
  uint4 gp[NV];
  float dga[NV][V];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    gp[i] = gr[min(i * 64 + lane, nvec - 1)];
#pragma unroll
    for (int j = 0; j < V; ++j) dga[i][j] = 0.0f;
  }
  const int t1 = min(t0 + NORM_BWD_TPW, Tn);
  for (int t = t0; t < t1; t += 2) {                  // two tokens per pass: sixteen row loads in flight
    const bool two = t + 1 < t1;
    const int tb = two ? t + 1 : t;
    uint4 dc[2][NV], xc[2][NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = min(i * 64 + lane, nvec - 1);
      dc[0][i] = reinterpret_cast<const uint4*>(dXn + (size_t)t * K)[c];
      xc[0][i] = reinterpret_cast<const uint4*>(X + (size_t)t * K)[c];
      dc[1][i] = reinterpret_cast<const uint4*>(dXn + (size_t)tb * K)[c];
      xc[1][i] = reinterpret_cast<const uint4*>(X + (size_t)tb * K)[c];
    }
    const float s2[2] = {rstd[t], rstd[tb]};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (q == 1 && !two) break;
      const float s = s2[q];
      double dot = 0.0;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        if (i * 64 + lane < nvec) {
          float d[V], x[V], g[V];
          vec16<T>::unpack(dc[q][i], d);
          vec16<T>::unpack(xc[q][i], x);
          vec16<T>::unpack(gp[i], g);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float u = __fmul_rn(x[j], s);
            dot += (double)__fmul_rn(g[j], d[j]) * (double)u;
            dga[i][j] = __fadd_rn(dga[i][j], __fmul_rn(d[j], u));
          }
        }
      }
      const float cm = (float)(wave_sum_d(dot) / (double)K);
      T* orow = dX + (size_t)(q ? tb : t) * K;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        if (c < nvec) {
          float d[V], x[V], g[V], o[V];
          vec16<T>::unpack(dc[q][i], d);
          vec16<T>::unpack(xc[q][i], x);
          vec16<T>::unpack(gp[i], g);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float u = __fmul_rn(x[j], s);
            o[j] = __fmul_rn(s, __fsub_rn(__fmul_rn(g[j], d[j]), __fmul_rn(u, cm)));
          }
          pq_st16<true>(reinterpret_cast<uint4*>(orow) + c, pack_io<T>(o));
        }
      }
    }
  }
  // the four wavefronts' shares are added in wavefront order and leave as one partial row
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * 64 + lane;
      if (c < nvec) {
#pragma unroll
        for (int j = 0; j < V; j += 4)
          *reinterpret_cast<float4*>(dsh + (size_t)(wave - 1) * K + (size_t)c * V + j) =
              make_float4(dga[i][j], dga[i][j + 1], dga[i][j + 2], dga[i][j + 3]);
      }
    }
  }
  __syncthreads();
  if (wave == 0) {
    float* prow = part + (size_t)blockIdx.x * K;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * 64 + lane;
      if (c < nvec) {
#pragma unroll
        for (int j = 0; j < V; j += 4) {
          float4 a = make_float4(dga[i][j], dga[i][j + 1], dga[i][j + 2], dga[i][j + 3]);
#pragma unroll
          for (int w = 0; w < 3; ++w) {
            const float4 b = *reinterpret_cast<const float4*>(dsh + (size_t)w * K + (size_t)c * V + j);
            a.x = __fadd_rn(a.x, b.x); a.y = __fadd_rn(a.y, b.y); a.z = __fadd_rn(a.z, b.z); a.w = __fadd_rn(a.w, b.w);
          }
          *reinterpret_cast<float4*>(prow + (size_t)c * V + j) = a;
        }
      }
    }
  }
}

// 8 columns x 32 row slices per workgroup: slice r adds rows r, r + 32, ... (sixteen independent loads in
// flight), the slices are then added in slice order.
__global__ __launch_bounds__(256) void rmsnorm_dgain_kernel(const float* __restrict__ part, int nrows, int K, float* __restrict__ dgain) {
  __shared__ double red[32][9];
  const int col = threadIdx.x & 7, slice = threadIdx.x >> 3;
  const int k = blockIdx.x * 8 + col;
  double a = 0.0;
  if (k < K) {
    int w = slice;
    for (; w + 15 * 32 < nrows; w += 16 * 32) {
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = part[(size_t)(w + 32 * i) * K + k];
#pragma unroll
      for (int i = 0; i < 16; ++i) a += (double)v[i];
    }
    for (; w < nrows; w += 32) a += (double)part[(size_t)w * K + k];
  }
  red[slice][col] = a;
  __syncthreads();
  if (slice == 0 && k < K) {
    double t = 0.0;
#pragma unroll
    for (int r = 0; r < 32; ++r) t += red[r][col];
    dgain[k] = (float)t;
  }
}

size_t pq_rmsnorm_bwd_scratch_bytes(int T, int K) {
  return (size_t)((T + NORM_BWD_TPB - 1) / NORM_BWD_TPB) * K * sizeof(float);
}

template <typename T>
static int launch_rmsnorm_bwd_t(const T* dXn, const T* X, const T* gain, const float* rstd, int Tn, int K, T* dX, float* part,
                                hipStream_t s) {
  constexpr int V = vec16<T>::V;
  const int per_lane = (K / V + 63) / 64;
  dim3 grid((Tn + NORM_BWD_TPB - 1) / NORM_BWD_TPB), block(256);
  const size_t lds = (size_t)3 * K * sizeof(float);
  if (per_lane <= 4) rmsnorm_bwd_kernel<T, 4><<<grid, block, lds, s>>>(dXn, X, gain, rstd, Tn, K, dX, part);
  else if (per_lane <= 8) rmsnorm_bwd_kernel<T, 8><<<grid, block, lds, s>>>(dXn, X, gain, rstd, Tn, K, dX, part);
  else return pq_set_error(PQ_ERR_SHAPE, "row of %d elements does not fit the register cache of the normalisation backward", K);
  PQ_CHECK_LAUNCH("rmsnorm_bwd_kernel");
  return PQ_OK;
}

int pq_launch_rmsnorm_bwd(const void* dXn, const void* X, const void* gain, const float* rstd, int dtype, int T, int K, void* dX,
                          float* dgain, float* part, hipStream_t s) {
  if (T > 0) {
    pq_prof_scope prof(PQP_NORM_BWD, s);
    int e;
    if (dtype == PQ_F32)
      e = launch_rmsnorm_bwd_t<float>((const float*)dXn, (const float*)X, (const float*)gain, rstd, T, K, (float*)dX, part, s);
    else
      e = launch_rmsnorm_bwd_t<uint16_t>((const uint16_t*)dXn, (const uint16_t*)X, (const uint16_t*)gain, rstd, T, K, (uint16_t*)dX, part, s);
    if (e) return e;
  }
  pq_prof_scope prof(PQP_NORM_BWD, s);
  rmsnorm_dgain_kernel<<<(K + 7) / 8, 256, 0, s>>>(part, (T + NORM_BWD_TPB - 1) / NORM_BWD_TPB, K, dgain);
  PQ_CHECK_LAUNCH("rmsnorm_dgain_kernel");
  return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Scratch for callers that cannot allocate (code under graph capture, serving loops): a file-scope device array
// that every GPU the library runs on holds until the process ends.  Its name is a host-side stand-in, not a
// device address: the address is looked up once per device and only that pointer is handed to kernels.
// ------------------------------------------------------------------------------------------
constexpr size_t PQ_STATIC_SCRATCH_BYTES = (size_t)4 << 20;
constexpr int PQ_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[PQ_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[PQ_MAX_DEVICES];

size_t pq_static_scratch_bytes() { return PQ_STATIC_SCRATCH_BYTES; }

int pq_static_scratch(void** out) {
  int dev = -1;
  PQ_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= PQ_MAX_DEVICES) return pq_set_error(PQ_ERR_HIP, "device ordinal %d is outside 0..%d", dev, PQ_MAX_DEVICES - 1);
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    PQ_CHECK_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return pq_set_error(PQ_ERR_HIP, "hipGetSymbolAddress returned a NULL address for the static scratch");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Weight statistics, stage 1: grid-stride fp64 sums of W and |W|, one pair per block.
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void wstats_partial_body(const T* __restrict__ W, size_t nvec, double* __restrict__ partials, int block,
                                                    int nblocks) {
  constexpr int V = vec16<T>::V;
  __shared__ double red[4];
  const uint4* w4 = reinterpret_cast<const uint4*>(W);
  double s = 0.0, a = 0.0;
  for (size_t c = (size_t)block * 256 + threadIdx.x; c < nvec; c += (size_t)nblocks * 256) {
    float f[V];
    vec16<T>::unpack(w4[c], f);
#pragma unroll
    for (int j = 0; j < V; ++j) {
      s += (double)f[j];
      a += (double)fabsf(f[j]);
    }
  }
  double bs = block_sum_d<256>(s, red);
  double ba = block_sum_d<256>(a, red);
  if (threadIdx.x == 0) {
    partials[2 * block] = bs;
    partials[2 * block + 1] = ba;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void wstats_partial_kernel(const T* __restrict__ W, size_t nvec,
                                                             double* __restrict__ partials) {
  wstats_partial_body<T>(W, nvec, partials, blockIdx.x, gridDim.x);
}

// The first stage of the weight statistics and the activation quantiser of one forward call are independent and
// each too short to fill its own launch well: one launch, the first nw workgroups take the weights.
struct slab_sum_job { const float* part; int splits, M, N; uint16_t* C; int ldc; };
template <int NV>
__global__ __launch_bounds__(256) void wstats_quant_kernel(const uint16_t* __restrict__ W, size_t nvec, double* __restrict__ partials,
                                                           int nw, const uint16_t* __restrict__ X, int Tn, int K,
                                                           int8_t* __restrict__ Xq, float* __restrict__ gamma,
                                                           uint16_t* __restrict__ Xt, int nq, slab_sum_job sj) {
  const int b = blockIdx.x;
  if (b < nw) wstats_partial_body<uint16_t>(W, nvec, partials, b, nw);
  else if (b < nw + nq) quant_act_body<uint16_t, NV>(X, Tn, K, Xq, gamma, Xt, b - nw);
  else pq_slab_sum_bf16_body(sj.part, sj.splits, sj.M, sj.N, sj.C, sj.ldc, (size_t)(b - nw - nq) * 256 + threadIdx.x);
}

// bf16 only; rows too long for the register-cached quantiser (more than 16 vectors per lane) take two launches
int pq_launch_wstats_quant(const void* W, size_t n_elems, double* partials, int nblocks, const void* X, int T, int K,
                           int8_t* Xq, float* gamma, uint16_t* Xt, hipStream_t s, const float* slabs, int splits, int M, int N,
                           void* C, int ldc) {
  const int per_lane = (K / 8 + 63) / 64;
  if (T <= 0 || per_lane > 16) return pq_set_error(PQ_ERR_SHAPE, "combined statistics/quantiser launch: bad shape T=%d K=%d", T, K);
  pq_prof_scope prof(PQP_QUANT, s);
  const int nq = (T + 3) / 4;
  const int ns = slabs ? (int)(((size_t)M * (N / 8) + 255) / 256) : 0;
  dim3 grid(nblocks + nq + ns), block(256);
  const uint16_t* w = (const uint16_t*)W;
  const uint16_t* x = (const uint16_t*)X;
  const slab_sum_job sj{slabs, splits, M, N, (uint16_t*)C, ldc};
  if (per_lane <= 4) wstats_quant_kernel<4><<<grid, block, 0, s>>>(w, n_elems / 8, partials, nblocks, x, T, K, Xq, gamma, Xt, nq, sj);
  else if (per_lane <= 8) wstats_quant_kernel<8><<<grid, block, 0, s>>>(w, n_elems / 8, partials, nblocks, x, T, K, Xq, gamma, Xt, nq, sj);
  else wstats_quant_kernel<16><<<grid, block, 0, s>>>(w, n_elems / 8, partials, nblocks, x, T, K, Xq, gamma, Xt, nq, sj);
  PQ_CHECK_LAUNCH("wstats_quant_kernel");
  return PQ_OK;
}

int pq_stats_blocks(size_t n_elems) {
  size_t b = (n_elems / 8 + 256 * 8 - 1) / (256 * 8);
  if (b < 1) b = 1;
  if (b > 1024) b = 1024;
  return (int)b;
}

int pq_launch_wstats_partial(const void* W, int dtype, size_t n_elems, double* partials, int nblocks,
                             hipStream_t s) {
  pq_prof_scope prof(PQP_WSTATS, s);
  if (dtype == PQ_F32)
    wstats_partial_kernel<float><<<nblocks, 256, 0, s>>>((const float*)W, n_elems / 4, partials);
  else
    wstats_partial_kernel<uint16_t><<<nblocks, 256, 0, s>>>((const uint16_t*)W, n_elems / 8, partials);
  PQ_CHECK_LAUNCH("wstats_partial_kernel");
  return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Stage 2 + binarise + pack.  A block owns a 32-row x 512-column tile of W: every lane turns 8
// consecutive weights into one byte of the row-packed stream (LSB = lowest column), the bytes
// also go to LDS, from which the column-packed orientation (32 rows per word) is assembled.
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ uint32_t sign_byte(const T* p, float mu);
template <>
__device__ __forceinline__ uint32_t sign_byte<uint16_t>(const uint16_t* p, float mu) {
  float f[8];
  vec16<uint16_t>::unpack(*reinterpret_cast<const uint4*>(p), f);
  uint32_t b = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) b |= (f[j] >= mu ? 1u : 0u) << j;
  return b;
}
template <>
__device__ __forceinline__ uint32_t sign_byte<float>(const float* p, float mu) {
  float f[8];
  vec16<float>::unpack(*reinterpret_cast<const uint4*>(p), f);
  vec16<float>::unpack(*reinterpret_cast<const uint4*>(p + 4), f + 4);
  uint32_t b = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) b |= (f[j] >= mu ? 1u : 0u) << j;
  return b;
}

// RAGGED: K is a multiple of 4 but not of 32, or N is not a multiple of 32 (Table 1: D_ff - r = 5076).  Rows may then start
// on 8-byte (bf16) boundaries only and end inside a lane's 8 weights, so the weights are fetched as two halves of four, each
// wholly inside or wholly outside its row; everything outside (columns K..Kp-1 of a packed row, Kp = K rounded up to whole
// words, and rows N.. of the last word of the transposed packing) is packed as +1: a padded position only ever meets an
// activation code (or gradient) of zero.
template <typename T, bool RAGGED>
__global__ __launch_bounds__(256) void pack_sign_kernel(const T* __restrict__ W, int N, int K,
                                                        const double* __restrict__ partials, int G,
                                                        uint8_t* __restrict__ Pbytes,
                                                        uint32_t* __restrict__ Pt,
                                                        float* __restrict__ mu_lambda) {
  __shared__ double red[4];
  __shared__ float s_mu;
  __shared__ uint8_t tileb[32][64];
  // the weights do not depend on the statistics: their eight chunks are requested first, so that their latency and
  // the reduction of the partial sums overlap instead of standing in a row
  constexpr int NU = sizeof(T) == 2 ? 1 : 2;          // 16-byte loads per 8 weights
  const int Kp = (K + 31) & ~31;
  const int n0 = blockIdx.y * 32, k0 = blockIdx.x * 512;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int k = k0 + lane * 8;
  uint4 wv[8][NU];
#pragma unroll
  for (int rr = 0; rr < 8; ++rr) {
    const int row = n0 + w * 8 + rr;
    if constexpr (RAGGED) {
      // halves of four weights: 8 bytes (bf16) or 16 bytes (fp32), aligned because K % 4 == 0
      const bool in0 = row < N && k + 4 <= K, in1 = row < N && k + 8 <= K;
      const T* p0 = W + (in0 ? (size_t)row * K + k : (size_t)0);
      const T* p1 = W + (in1 ? (size_t)row * K + k + 4 : (size_t)0);
      if constexpr (sizeof(T) == 2) {
        const uint2 a = *reinterpret_cast<const uint2*>(p0), b = *reinterpret_cast<const uint2*>(p1);
        wv[rr][0] = make_uint4(a.x, a.y, b.x, b.y);
      } else {
        wv[rr][0] = *reinterpret_cast<const uint4*>(p0);
        wv[rr][1] = *reinterpret_cast<const uint4*>(p1);
      }
    } else {
      const bool in = row < N && k < K;
      const uint4* src = reinterpret_cast<const uint4*>(W + (in ? (size_t)row * K + k : (size_t)0));   // element (0, 0) always exists
#pragma unroll
      for (int u = 0; u < NU; ++u) wv[rr][u] = src[u];
    }
  }
  double s = 0.0, a = 0.0;
  for (int i = threadIdx.x; i < G; i += 256) {
    s += partials[2 * i];
    a += partials[2 * i + 1];
  }
  double ts = block_sum_d<256>(s, red);
  double ta = block_sum_d<256>(a, red);
  if (threadIdx.x == 0) {
    const double cnt = (double)N * (double)K;
    float mu = (float)(ts / cnt);
    s_mu = mu;
    if (blockIdx.x == 0 && blockIdx.y == 0) {
      mu_lambda[0] = mu;
      mu_lambda[1] = (float)(ta / cnt);
    }
  }
  __syncthreads();
  const float mu = s_mu;
  const size_t kb = (size_t)Kp / 8;
#pragma unroll
  for (int rr = 0; rr < 8; ++rr) {
    const int rl = w * 8 + rr, row = n0 + rl;
    uint32_t b = RAGGED ? 0xFFu : 0u;
    if (row < N && k < Kp) {
      b = sign_byte<T>(reinterpret_cast<const T*>(wv[rr]), mu);
      if constexpr (RAGGED) {
        if (k + 4 > K) b |= 0x0Fu;
        if (k + 8 > K) b |= 0xF0u;
      }
      Pbytes[(size_t)row * kb + (k >> 3)] = (uint8_t)b;
    }
    tileb[rl][lane] = (uint8_t)b;
  }
  if (Pt == nullptr) return;
  __syncthreads();
  const size_t nw = ((size_t)N + 31) / 32;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int kk = threadIdx.x + h * 256;
    if (k0 + kk < K) {
      uint32_t word = 0;
#pragma unroll
      for (int j = 0; j < 32; ++j) word |= (((uint32_t)tileb[j][kk >> 3] >> (kk & 7)) & 1u) << j;
      Pt[(size_t)(k0 + kk) * nw + blockIdx.y] = word;
    }
  }
}

int pq_launch_pack(const void* W, int dtype, int N, int K, const double* partials, int nblocks,
                   uint32_t* P, uint32_t* Pt, float* mu_lambda, hipStream_t s) {
  pq_prof_scope prof(PQP_PACK, s);
  const int Kp = (K + 31) & ~31;
  dim3 grid((Kp + 511) / 512, (N + 31) / 32), block(256);
  const bool ragged = (K % 32 != 0) || (N % 32 != 0);
  if (dtype == PQ_F32) {
    if (ragged) pack_sign_kernel<float, true><<<grid, block, 0, s>>>((const float*)W, N, K, partials, nblocks, (uint8_t*)P, Pt, mu_lambda);
    else pack_sign_kernel<float, false><<<grid, block, 0, s>>>((const float*)W, N, K, partials, nblocks, (uint8_t*)P, Pt, mu_lambda);
  } else {
    if (ragged) pack_sign_kernel<uint16_t, true><<<grid, block, 0, s>>>((const uint16_t*)W, N, K, partials, nblocks, (uint8_t*)P, Pt, mu_lambda);
    else pack_sign_kernel<uint16_t, false><<<grid, block, 0, s>>>((const uint16_t*)W, N, K, partials, nblocks, (uint8_t*)P, Pt, mu_lambda);
  }
  PQ_CHECK_LAUNCH("pack_sign_kernel");
  return PQ_OK;
}

// N values per lane summed over the wavefront, transposed: every exchange step halves the values a lane carries (the
// lane with the step's bit set keeps the upper half and hands over the lower), so that after log2(N) steps a lane holds
// one value -- lane l the one with index l / (64 / N) -- and the remaining steps are plain exchanges.  The additions
// are those of the butterfly sum (same pairs, same order), at a quarter of the instructions.  Every index is static.
template <int N, int OFF>
__device__ __forceinline__ void wave_sum_transposed(double* v, int lane) {
  if constexpr (N > 1) {
    const bool up = (lane & OFF) != 0;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      const double send = up ? v[i] : v[i + N / 2];
      const double keep = up ? v[i + N / 2] : v[i];
      v[i] = keep + __shfl_xor(send, OFF, 64);
    }
    if constexpr (OFF > 1) wave_sum_transposed<N / 2, OFF / 2>(v, lane);
  } else {
    v[0] += __shfl_xor(v[0], OFF, 64);
    if constexpr (OFF > 1) wave_sum_transposed<1, OFF / 2>(v, lane);
  }
}

// ------------------------------------------------------------------------------------------
// Router: a wavefront takes TB tokens at once (a router row converted to fp64 serves all of them): fp64 dot products
// against all E router rows, lane l accumulating the 16-byte chunks l, l + 64, ... of a token row in order, then the
// wave sums, which leave one (token, expert) pair per lane; that lane rounds the logit to fp32 and evaluates its term
// of the softmax in fp64; the first lane of a token's group selects the top-k (ties to the lower index).
// ------------------------------------------------------------------------------------------
template <typename T, int EMAX, int TB>
__global__ __launch_bounds__(256) void router_kernel(const T* __restrict__ X, const T* __restrict__ Wr,
                                                     int Tn, int K, int E, int k, int* __restrict__ idx,
                                                     float* __restrict__ gate, float* __restrict__ probs) {
  constexpr int V = vec16<T>::V;
  const int lane = threadIdx.x & 63;
  const int t0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * TB;
  if (t0 >= Tn) return;
  const int nvec = K / V;
  double acc[TB][EMAX];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int e = 0; e < EMAX; ++e) acc[tb][e] = 0.0;
  // Router rows are requested unconditionally, eight at a time (rows past E repeat the last one and their sums
  // are never used; tokens past the end repeat the last token): a load under a branch gets a wait of its own, which
  // made this loop a chain of latencies.
  for (int c = lane; c < nvec; c += 64) {
    double xd[TB][V];
    uint4 xv[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) xv[tb] = reinterpret_cast<const uint4*>(X + (size_t)min(t0 + tb, Tn - 1) * K)[c];
#pragma unroll
    for (int e0 = 0; e0 < EMAX; e0 += 8) {
      uint4 wv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) wv[u] = reinterpret_cast<const uint4*>(Wr + (size_t)min(e0 + u, E - 1) * K)[c];
      if (e0 == 0) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
          float xf[V];
          vec16<T>::unpack(xv[tb], xf);
#pragma unroll
          for (int j = 0; j < V; ++j) xd[tb][j] = (double)xf[j];
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float wf[V];
        vec16<T>::unpack(wv[u], wf);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const double wd = (double)wf[j];
#pragma unroll
          for (int tb = 0; tb < TB; ++tb) acc[tb][e0 + u] += xd[tb][j] * wd;
        }
      }
    }
  }
  // Sums over the wavefront, transposed (see wave_sum_transposed): lane l ends with the sum of value l / ST.
  constexpr int NV = TB * EMAX, ST = 64 / NV;
  static_assert(NV == 32 || NV == 64, "a wavefront carries 32 or 64 (token, expert) sums");
  double v[NV];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int e = 0; e < EMAX; ++e) v[tb * EMAX + e] = acc[tb][e];
  wave_sum_transposed<NV, 32>(v, lane);
  // lane l: pair (token tb, expert e); one exponential and one division per lane
  const int vi = lane / ST, tb = vi / EMAX, e = vi % EMAX;
  const double lg = (double)(float)v[0];              // one rounding to fp32
  const bool live = e < E;
  double mx = live ? lg : -1e300;
#pragma unroll
  for (int off = ST; off < ST * EMAX; off <<= 1) mx = fmax(mx, __shfl_xor(mx, off, 64));
  double pr = live ? exp(lg - mx) : 0.0;
  double den = pr;
#pragma unroll
  for (int off = ST; off < ST * EMAX; off <<= 1) den += __shfl_xor(den, off, 64);
  pr /= den;
  const int t = t0 + tb;
  if (probs && live && t < Tn && lane % ST == 0) probs[(size_t)t * E + e] = (float)pr;
  // the token's logits and probabilities into every lane of its group, then the top-k (ties to the lower index)
  double logit[EMAX], p[EMAX];
#pragma unroll
  for (int ee = 0; ee < EMAX; ++ee) {
    logit[ee] = __shfl(lg, (tb * EMAX + ee) * ST, 64);
    p[ee] = __shfl(pr, (tb * EMAX + ee) * ST, 64);
  }
  if (lane % (ST * EMAX) != 0 || t >= Tn) return;     // the group's first lane writes the token's choice
  unsigned long long taken = 0ull;
  for (int j = 0; j < k; ++j) {
    int best = -1;
    double bv = 0.0, bp = 0.0;
#pragma unroll
    for (int ee = 0; ee < EMAX; ++ee) {
      if (ee < E && !((taken >> ee) & 1ull) && (best < 0 || logit[ee] > bv)) {
        best = ee; bv = logit[ee]; bp = p[ee];
      }
    }
    taken |= 1ull << best;
    idx[(size_t)t * k + j] = best;
    gate[(size_t)t * k + j] = (float)bp;
  }
}

template <typename T>
static int launch_router_t(const T* X, const T* Wr, int Tn, int K, int E, int k, int* idx, float* gate,
                           float* probs, hipStream_t s) {
  dim3 block(256);
  if (E <= 8) router_kernel<T, 8, 4><<<dim3((Tn + 15) / 16), block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
  else if (E <= 16) router_kernel<T, 16, 2><<<dim3((Tn + 7) / 8), block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
  else router_kernel<T, 64, 1><<<dim3((Tn + 3) / 4), block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
  PQ_CHECK_LAUNCH("router_kernel");
  return PQ_OK;
}

int pq_launch_router(const void* X, const void* Wr, int dtype, int T, int K, int E, int k, int* idx,
                     float* gate, float* probs, hipStream_t s) {
  if (T == 0) return PQ_OK;
  pq_prof_scope prof(PQP_ROUTER, s);
  if (dtype == PQ_F32)
    return launch_router_t<float>((const float*)X, (const float*)Wr, T, K, E, k, idx, gate, probs, s);
  return launch_router_t<uint16_t>((const uint16_t*)X, (const uint16_t*)Wr, T, K, E, k, idx, gate, probs, s);
}

// ------------------------------------------------------------------------------------------
// Fixed-order final reduction of per-block partial sums.
// ------------------------------------------------------------------------------------------
typedef pq_reduce_job reduce_job;

__global__ __launch_bounds__(256) void reduce_partials_kernel(reduce_job j0, reduce_job j1) {   // one workgroup per job
  pq_reduce_job_body(blockIdx.x == 0 ? j0 : j1);
}

int pq_launch_reduce_partials(const double* partials, int n, float factor, const float* dev_factor,
                              float* out, hipStream_t s) {
  pq_prof_scope prof(PQP_REDUCE, s);
  const reduce_job j{partials, n, factor, dev_factor, out};
  reduce_partials_kernel<<<1, 256, 0, s>>>(j, j);
  PQ_CHECK_LAUNCH("reduce_partials_kernel");
  return PQ_OK;
}

// two independent reductions in one launch
int pq_launch_reduce_partials2(const double* pa, int na, float fa, const float* dfa, float* oa, const double* pb, int nb, float fb,
                               const float* dfb, float* ob, hipStream_t s) {
  pq_prof_scope prof(PQP_REDUCE, s);
  reduce_partials_kernel<<<2, 256, 0, s>>>(reduce_job{pa, na, fa, dfa, oa}, reduce_job{pb, nb, fb, dfb, ob});
  PQ_CHECK_LAUNCH("reduce_partials_kernel");
  return PQ_OK;
}
