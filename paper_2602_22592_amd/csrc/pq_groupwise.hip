// Group-wise scales of the 1-bit weights (Sec. 4.6 ablation), built as a measured contrast to the per-tensor form:
//   Y[t][n] = beta / gamma_t * sum_g lambda[n][g] * sum_{k in group g} S[n][k] q[t][k],   groups of 64 input columns,
// lambda[n][g] = mean |W[n][k in g]| held in fp16 (one 16-bit scale per 64 one-bit weights), mu and S = Sign(W - mu)
// as in the per-tensor form (Sec. 3.1).  The same kernel also runs the per-tensor product (group = 0: int32 accumulation
// over the whole contraction, one scale in the epilogue), so that the two timings differ by the group scales alone:
// a flush of the int32 accumulators into fp32 ones every 64 contraction indices (16 conversions and 16 multiply-adds per
// 32x32 block behind two int8 MFMAs) and the scale loads.
#include <hip/hip_fp16.h>

#include "pq_internal.h"

namespace {

#define PQ_REQUIRE(cond, code, ...) \
  do { if (!(cond)) return pq_set_error(code, __VA_ARGS__); } while (0)

constexpr int GW_GROUP = 64;
constexpr int GW_LDA = 80;   // bytes between rows of the activation tile in LDS (64 codes + 16: 16-byte reads of 32 rows fall on distinct banks)

// lam16[n][g] = fp16(fp32(mean |W[n][64 g .. 64 g + 63]|)): the sum of 64 bf16 magnitudes is exact in fp64
__global__ __launch_bounds__(256) void groupwise_scales_kernel(const uint16_t* __restrict__ W, int N, int K, uint16_t* __restrict__ lam16) {
  const size_t gi = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t ng = (size_t)N * (K / GW_GROUP);
  if (gi >= ng) return;
  const uint4* p = reinterpret_cast<const uint4*>(W + gi * GW_GROUP);
  double sum = 0.0;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const uint4 v = p[c];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      sum += (double)fabsf(__uint_as_float(w[d] << 16));
      sum += (double)fabsf(__uint_as_float(w[d] & 0xFFFF0000u));
    }
  }
  const float m32 = (float)(sum / 64.0);
  lam16[gi] = __half_as_ushort(__float2half_rn(m32));
}

__device__ __forceinline__ i32x4_t gw_bits_to_i8(uint32_t b) {   // 16 bits -> 16 int8 of +/-1 (bit set = +1, Eq. 4)
  i32x4_t o;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t m = __umul24((b >> (4 * d)) & 0xFu, 0x00204081u) & 0x01010101u;
    o[d] = (int)__builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, m);
  }
  return o;
}

// 128 tokens x 128 outputs per workgroup, four wavefronts of 64 x 64 (2 x 2 blocks of 32 x 32), one group (64 contraction
// indices) per step: activation codes [128][64] and packed signs [128][8 B] through two LDS stages filled from registers.
// Accumulator block: lane l holds output column n = l % 32, register v token row 8 (v / 4) + 4 (l / 32) + v % 4, so a
// group's scale is one value per lane and block.
template <bool GROUPWISE>
__global__ __launch_bounds__(256) void groupwise_gemm_kernel(const int8_t* __restrict__ Xq, const float* __restrict__ gamma,
                                                             const uint8_t* __restrict__ P, const uint16_t* __restrict__ lam16,
                                                             const float* __restrict__ mu_lambda, int T, int K, int N, float beta,
                                                             float* __restrict__ Y) {
  __shared__ __attribute__((aligned(16))) unsigned char sA[2][128 * GW_LDA];
  __shared__ __attribute__((aligned(16))) unsigned char sB[2][128 * 8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  const int G = K / GW_GROUP;

  // staging: thread -> rows tid / 4 and tid / 4 + 64 of the activation tile, 16-byte chunk tid % 4; threads 0..127 -> the
  // 8 sign bytes of weight row tid.  Rows past the end repeat the last valid one (never stored).
  const int ar = tid >> 2, ac = tid & 3;
  const int8_t* a_src0 = Xq + (size_t)min(m0 + ar, T - 1) * K + ac * 16;
  const int8_t* a_src1 = Xq + (size_t)min(m0 + ar + 64, T - 1) * K + ac * 16;
  const uint8_t* b_src = P + (size_t)min(n0 + (tid & 127), N - 1) * (K / 8);
  uint4 ra0, ra1;
  uint2 rb = make_uint2(0u, 0u);
  auto gload = [&](int g) {
    ra0 = *reinterpret_cast<const uint4*>(a_src0 + (size_t)g * 64);
    ra1 = *reinterpret_cast<const uint4*>(a_src1 + (size_t)g * 64);
    if (tid < 128) rb = *reinterpret_cast<const uint2*>(b_src + (size_t)g * 8);
  };
  auto sstore = [&](int st) {
    *reinterpret_cast<uint4*>(&sA[st][ar * GW_LDA + ac * 16]) = ra0;
    *reinterpret_cast<uint4*>(&sA[st][(ar + 64) * GW_LDA + ac * 16]) = ra1;
    if (tid < 128) *reinterpret_cast<uint2*>(&sB[st][tid * 8]) = rb;
  };
  // the group scales of this lane's two columns, one group ahead
  const uint16_t* lam_src[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) lam_src[j] = lam16 + (size_t)min(n0 + wn0 + 32 * j + (lane & 31), N - 1) * G;

  f32x16_t accf[2][2];
  i32x16_t acci[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        accf[i][j][v] = 0.f;
        acci[i][j][v] = 0;
      }

  if (G > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  for (int g = 0; g < G; ++g) {
    const int st = g & 1;
    if (g + 1 < G) gload(g + 1);
    float lam[2] = {0.f, 0.f};
    if constexpr (GROUPWISE) {
#pragma unroll
      for (int j = 0; j < 2; ++j) lam[j] = __half2float(__ushort_as_half(lam_src[j][g]));
    }
    i32x4_t fa[2][2], fb[2][2];   // [block][half of the group]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
        fa[i][kk] = *reinterpret_cast<const i32x4_t*>(&sA[st][(wm0 + 32 * i + (lane & 31)) * GW_LDA + kk * 32 + (lane >> 5) * 16]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint2 w = *reinterpret_cast<const uint2*>(&sB[st][(wn0 + 32 * j + (lane & 31)) * 8]);
      fb[j][0] = gw_bits_to_i8(w.x >> (16 * (lane >> 5)));
      fb[j][1] = gw_bits_to_i8(w.y >> (16 * (lane >> 5)));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (GROUPWISE) {
          i32x16_t p;
#pragma unroll
          for (int v = 0; v < 16; ++v) p[v] = 0;
          p = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][0], fb[j][0], p, 0, 0, 0);
          p = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][1], fb[j][1], p, 0, 0, 0);
#pragma unroll
          for (int v = 0; v < 16; ++v) accf[i][j][v] = fmaf(lam[j], (float)p[v], accf[i][j][v]);
        } else {
          acci[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][0], fb[j][0], acci[i][j], 0, 0, 0);
          acci[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][1], fb[j][1], acci[i][j], 0, 0, 0);
        }
      }
    if (g + 1 < G) sstore(st ^ 1);
    __syncthreads();
  }

  const float lam_t = GROUPWISE ? 1.0f : mu_lambda[1];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (m >= T) continue;
      const float gm = gamma[m];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn0 + 32 * j + (lane & 31);
        if (n >= N) continue;
        const float a = GROUPWISE ? accf[i][j][v] : __fmul_rn(lam_t, (float)acci[i][j][v]);
        Y[(size_t)m * N + n] = __fmul_rn(beta, a) / gm;
      }
    }
}

struct gw_layout {
  size_t Xq, gamma, stat, ml, P, lam16, total;
};
gw_layout gw_make_layout(int T, int K, int N) {
  gw_layout L;
  size_t off = 0;
  auto take = [&](size_t b) { size_t o = off; off = pq_align_up(off + (b ? b : 1), 256); return o; };
  L.Xq = take((size_t)T * K);
  L.gamma = take((size_t)T * 4);
  L.stat = take(2 * sizeof(double) * 1024);
  L.ml = take(8);
  L.P = take((size_t)N * K / 8);
  L.lam16 = take((size_t)N * (K / GW_GROUP) * 2);
  L.total = off;
  return L;
}
int gw_check(int dtype, int T, int K, int N, int group) {
  PQ_REQUIRE(T >= 0 && K > 0 && N > 0, PQ_ERR_BAD_ARG, "bad dimension");
  PQ_REQUIRE(dtype == PQ_BF16, PQ_ERR_DTYPE, "the group-wise contrast runs on bf16 inputs only");
  PQ_REQUIRE(group == 0 || group == GW_GROUP, PQ_ERR_BAD_ARG, "group must be 64 (group-wise scales) or 0 (per-tensor scale), got %d", group);
  PQ_REQUIRE(K % 64 == 0 && N % 32 == 0, PQ_ERR_SHAPE, "d_in=%d must be a multiple of 64 and d_out=%d of 32", K, N);
  return PQ_OK;
}

}  // namespace

extern "C" size_t pq_groupwise_workspace_bytes(int32_t T, int32_t K, int32_t N) {
  if (T < 0 || K <= 0 || N <= 0 || K % 64 != 0) return 0;
  return gw_make_layout(T, K, N).total;
}

extern "C" int pq_groupwise_fwd(const void* X, const void* W, int32_t dtype, int32_t T, int32_t K, int32_t N, int32_t group,
                                float beta, float* Y, void* workspace, size_t workspace_bytes, void* stream) {
  if (int e = gw_check(dtype, T, K, N, group)) return e;
  if (T == 0) return PQ_OK;                          // no tokens: nothing is read or written
  PQ_REQUIRE(X && W && Y && workspace, PQ_ERR_BAD_ARG, "NULL buffer");
  PQ_REQUIRE(((uintptr_t)X % 16) == 0 && ((uintptr_t)W % 16) == 0 && ((uintptr_t)Y % 16) == 0 && ((uintptr_t)workspace % 16) == 0,
             PQ_ERR_SHAPE, "buffers must be 16-byte aligned");
  const gw_layout L = gw_make_layout(T, K, N);
  PQ_REQUIRE(workspace_bytes >= L.total, PQ_ERR_WORKSPACE, "workspace %zu < %zu", workspace_bytes, L.total);
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  int8_t* Xq = (int8_t*)(ws + L.Xq);
  float* gamma = (float*)(ws + L.gamma);
  double* part = (double*)(ws + L.stat);
  float* ml = (float*)(ws + L.ml);
  if (int e = pq_launch_quant_act(X, PQ_BF16, T, K, Xq, gamma, nullptr, s)) return e;
  const size_t n = (size_t)N * K;
  const int nb = pq_stats_blocks(n);
  if (int e = pq_launch_wstats_partial(W, PQ_BF16, n, part, nb, s)) return e;
  if (int e = pq_launch_pack(W, PQ_BF16, N, K, part, nb, (uint32_t*)(ws + L.P), nullptr, ml, s)) return e;
  uint16_t* lam16 = (uint16_t*)(ws + L.lam16);
  if (group) {
    pq_prof_scope prof(PQP_WSTATS, s);
    const size_t ng = (size_t)N * (K / GW_GROUP);
    groupwise_scales_kernel<<<(unsigned)((ng + 255) / 256), 256, 0, s>>>((const uint16_t*)W, N, K, lam16);
    PQ_CHECK_LAUNCH("groupwise_scales_kernel");
  }
  pq_prof_scope prof(PQP_GEMM_ONEBIT, s);
  dim3 grid((N + 127) / 128, (T + 127) / 128), block(256);
  if (group) groupwise_gemm_kernel<true><<<grid, block, 0, s>>>(Xq, gamma, (const uint8_t*)(ws + L.P), lam16, ml, T, K, N, beta, Y);
  else groupwise_gemm_kernel<false><<<grid, block, 0, s>>>(Xq, gamma, (const uint8_t*)(ws + L.P), lam16, ml, T, K, N, beta, Y);
  PQ_CHECK_LAUNCH("groupwise_gemm_kernel");
  return PQ_OK;
}
