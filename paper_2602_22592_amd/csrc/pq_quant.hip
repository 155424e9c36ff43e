// Bandwidth-bound element kernels: AbsMax INT8 activation quantiser (Sec. 3.1), weight statistics
// mu/lambda and the sign binariser/packer (Sec. 3.1, App. A), the router (Sec. 3.3).
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

template <typename T>
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
    *reinterpret_cast<uint2*>(qrow + (size_t)c * 8) = make_uint2(w[0], w[1]);
  } else {
    *reinterpret_cast<uint32_t*>(qrow + (size_t)c * 4) = w[0];
  }
  if (xtrow) {
    uint32_t o[V / 2];
#pragma unroll
    for (int j = 0; j < V / 2; ++j)
      o[j] = pack_bf16x2((float)q[2 * j] / g, (float)q[2 * j + 1] / g);
    if constexpr (V == 8) {
      *reinterpret_cast<uint4*>(xtrow + (size_t)c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      *reinterpret_cast<uint2*>(xtrow + (size_t)c * 4) = make_uint2(o[0], o[1]);
    }
  }
}

template <typename T, int NV>
__global__ __launch_bounds__(256) void quant_act_kernel(const T* __restrict__ X, int Tn, int K,
                                                        int8_t* __restrict__ Xq,
                                                        float* __restrict__ gamma,
                                                        uint16_t* __restrict__ Xt) {
  constexpr int V = vec16<T>::V;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Tn) return;
  const uint4* xr = reinterpret_cast<const uint4*>(X + (size_t)row * K);
  const int nvec = K / V;
  float amax = 0.0f;
  uint4 cache[NV > 0 ? NV : 1];
  if constexpr (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int c = i * 64 + lane;
      if (c < nvec) {
        cache[i] = xr[c];
        float f[V];
        vec16<T>::unpack(cache[i], f);
#pragma unroll
        for (int j = 0; j < V; ++j) amax = fmaxf(amax, fabsf(f[j]));
      }
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
// Weight statistics, stage 1: grid-stride fp64 sums of W and |W|, one pair per block.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void wstats_partial_kernel(const T* __restrict__ W, size_t nvec,
                                                             double* __restrict__ partials) {
  constexpr int V = vec16<T>::V;
  __shared__ double red[4];
  const uint4* w4 = reinterpret_cast<const uint4*>(W);
  double s = 0.0, a = 0.0;
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < nvec; c += (size_t)gridDim.x * 256) {
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
    partials[2 * blockIdx.x] = bs;
    partials[2 * blockIdx.x + 1] = ba;
  }
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

template <typename T>
__global__ __launch_bounds__(256) void pack_sign_kernel(const T* __restrict__ W, int N, int K,
                                                        const double* __restrict__ partials, int G,
                                                        uint8_t* __restrict__ Pbytes,
                                                        uint32_t* __restrict__ Pt,
                                                        float* __restrict__ mu_lambda) {
  __shared__ double red[4];
  __shared__ float s_mu;
  __shared__ uint8_t tileb[32][64];
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
  const int n0 = blockIdx.y * 32, k0 = blockIdx.x * 512;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int k = k0 + lane * 8;
  const size_t kb = (size_t)K / 8;
#pragma unroll
  for (int rr = 0; rr < 8; ++rr) {
    const int rl = w * 8 + rr, row = n0 + rl;
    uint32_t b = 0;
    if (row < N && k < K) {
      b = sign_byte<T>(W + (size_t)row * K + k, mu);
      Pbytes[(size_t)row * kb + (k >> 3)] = (uint8_t)b;
    }
    tileb[rl][lane] = (uint8_t)b;
  }
  if (Pt == nullptr) return;
  __syncthreads();
  const size_t nw = (size_t)N / 32;
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
  dim3 grid((K + 511) / 512, (N + 31) / 32), block(256);
  if (dtype == PQ_F32)
    pack_sign_kernel<float><<<grid, block, 0, s>>>((const float*)W, N, K, partials, nblocks,
                                                   (uint8_t*)P, Pt, mu_lambda);
  else
    pack_sign_kernel<uint16_t><<<grid, block, 0, s>>>((const uint16_t*)W, N, K, partials, nblocks,
                                                      (uint8_t*)P, Pt, mu_lambda);
  PQ_CHECK_LAUNCH("pack_sign_kernel");
  return PQ_OK;
}

// ------------------------------------------------------------------------------------------
// Router: one wavefront per token, fp64 dot products against all E router rows, then lane 0
// rounds the logits to fp32, selects the top-k (ties to the lower index) and evaluates the
// softmax in fp64.
// ------------------------------------------------------------------------------------------
template <typename T, int EMAX>
__global__ __launch_bounds__(256) void router_kernel(const T* __restrict__ X, const T* __restrict__ Wr,
                                                     int Tn, int K, int E, int k, int* __restrict__ idx,
                                                     float* __restrict__ gate, float* __restrict__ probs) {
  constexpr int V = vec16<T>::V;
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  const uint4* xr = reinterpret_cast<const uint4*>(X + (size_t)t * K);
  const int nvec = K / V;
  double acc[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) acc[e] = 0.0;
  for (int c = lane; c < nvec; c += 64) {
    float xf[V];
    vec16<T>::unpack(xr[c], xf);
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      if (e < E) {
        float wf[V];
        vec16<T>::unpack(reinterpret_cast<const uint4*>(Wr + (size_t)e * K)[c], wf);
#pragma unroll
        for (int j = 0; j < V; ++j) acc[e] += (double)xf[j] * (double)wf[j];
      }
    }
  }
  double logit[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) logit[e] = (double)(float)wave_sum_d(acc[e]);  // one rounding to fp32
  if (lane != 0) return;
  double mx = -1e300;
#pragma unroll
  for (int e = 0; e < EMAX; ++e)
    if (e < E) mx = fmax(mx, logit[e]);
  double p[EMAX];
  double den = 0.0;
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    p[e] = (e < E) ? exp(logit[e] - mx) : 0.0;
    den += p[e];
  }
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    p[e] /= den;
    if (probs && e < E) probs[(size_t)t * E + e] = (float)p[e];
  }
  unsigned long long taken = 0ull;
  for (int j = 0; j < k; ++j) {
    int best = -1;
    double bv = 0.0, bp = 0.0;
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      if (e < E && !((taken >> e) & 1ull) && (best < 0 || logit[e] > bv)) {
        best = e; bv = logit[e]; bp = p[e];
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
  dim3 grid((Tn + 3) / 4), block(256);
  if (E <= 8) router_kernel<T, 8><<<grid, block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
  else if (E <= 16) router_kernel<T, 16><<<grid, block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
  else router_kernel<T, 64><<<grid, block, 0, s>>>(X, Wr, Tn, K, E, k, idx, gate, probs);
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
__global__ __launch_bounds__(256) void reduce_partials_kernel(const double* __restrict__ partials, int n,
                                                              float factor, const float* dev_factor,
                                                              float* __restrict__ out) {
  __shared__ double red[4];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += partials[i];
  double t = block_sum_d<256>(s, red);
  if (threadIdx.x == 0) {
    double f = (double)factor;
    if (dev_factor) f *= (double)(*dev_factor);
    out[0] = (float)(t * f);
  }
}

int pq_launch_reduce_partials(const double* partials, int n, float factor, const float* dev_factor,
                              float* out, hipStream_t s) {
  pq_prof_scope prof(PQP_REDUCE, s);
  reduce_partials_kernel<<<1, 256, 0, s>>>(partials, n, factor, dev_factor, out);
  PQ_CHECK_LAUNCH("reduce_partials_kernel");
  return PQ_OK;
}
