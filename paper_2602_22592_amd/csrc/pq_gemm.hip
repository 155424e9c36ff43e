// Tiled MFMA GEMM for gfx950 with pluggable operand sources and epilogues, plus a
// reference-precision engine (fp64 accumulate) used for fp32 I/O.
//
//   C[m][n] (+)= epilogue( sum_k A(m,k) * B(n,k) )
//
// Both operands are staged through LDS as tiles of ROWS x 128 bytes with the contraction index
// contiguous (64 bf16 or 128 int8 per row), whatever their layout in HBM:
//   KC16 / KC8   contraction-contiguous rows are copied 16 bytes at a time;
//   KS16         contraction-strided sources (the transposed operands of the weight-gradient
//                GEMMs) are read as 8x8 blocks of 16-bit elements, transposed in registers with
//                byte permutes and written as 16-byte chunks;
//   BITS8/BITS16 packed sign bits are expanded to +/-1 (int8 or bf16) on the way into LDS, so the
//                1-bit weights cross HBM and L2 as bits (Sec. 3.1 W^INT1; App. A packing).
// A wavefront owns a (BM/WGM) x (BN/WGN) sub-tile as 32x32 MFMA blocks:
//   v_mfma_f32_32x32x16_bf16 / v_mfma_i32_32x32x32_i8, 16 bytes of operand per lane per issue.
// LDS rows are 128 bytes with the 16-byte chunk index XOR-swizzled by the row so that the MFMA
// operand reads, the row-wise stores and the transposed stores are all free of bank conflicts.
#include <string.h>
#include <type_traits>
#include "pq_internal.h"

namespace {

__device__ __forceinline__ uint4 mask4(const uint4& t, bool keep) {
  const uint32_t m = keep ? 0xFFFFFFFFu : 0u;
  return make_uint4(t.x & m, t.y & m, t.z & m, t.w & m);
}

__device__ __forceinline__ int lds_off(int r, int c) { return r * 128 + (((c ^ r ^ (r >> 3)) & 7) << 4); }

// ---------------------------------------------------------------------------------------------
// Operand tile staging: global -> registers (load) and registers -> LDS (store)
// ---------------------------------------------------------------------------------------------
template <int KIND, int ROWS, int NT>
struct tile_stage {
  static constexpr int NCH = (ROWS * 8 + NT - 1) / NT;  // 16-byte LDS chunks per thread
  static constexpr bool kBits = (KIND == PQ_SRC_BITS8 || KIND == PQ_SRC_BITS16);
  static constexpr bool kStrided = (KIND == PQ_SRC_KS16);
  static constexpr int EPC = (KIND == PQ_SRC_KC8 || KIND == PQ_SRC_BITS8) ? 16 : 8;  // elements per chunk
  // KS16: a unit is 8 rows x KQ contraction indices (KQ 16-byte loads, transposed in registers)
  static constexpr int KQ = (ROWS >= NT) ? 8 : 4;
  static constexpr int UPR = 64 / KQ;                     // units per 8-row group
  static constexpr int NU = (ROWS / 8 * UPR + NT - 1) / NT;  // units per thread
  uint4 v[kBits ? 1 : (kStrided ? NU * KQ : NCH)];
  uint32_t raw[kBits ? NCH : 1];
  uint32_t okbits;  // validity of each loaded chunk, applied when the tile is written to LDS

  // Loads are unconditional (an out-of-range chunk reads element (0,0), which always exists, and is
  // then replaced by zeros) so that all of a thread's loads are in flight together.
  __device__ __forceinline__ void load(const pq_operand& op, int row0, int rows, int k0, int K, int tid) {
    okbits = 0u;
    if constexpr (kStrided) {
      const uint16_t* p = (const uint16_t*)op.p;
#pragma unroll
      for (int i = 0; i < NU; ++i) {
        const int u = tid + i * NT;
        const int r8 = u / UPR, kq = u % UPR;
        const int col = row0 + r8 * 8;
        const bool okc = (u < ROWS / 8 * UPR) && (col < rows);
#pragma unroll
        for (int j = 0; j < KQ; ++j) {
          const int kk = k0 + kq * KQ + j;
          const bool ok = okc && (kk < K);
          const size_t off = ok ? (size_t)kk * op.ld + col : 0;
          v[i * KQ + j] = *reinterpret_cast<const uint4*>(p + off);
          okbits |= (ok ? 1u : 0u) << (i * KQ + j);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * NT;
        const int r = c >> 3, kc = c & 7;
        const int grow = row0 + r, k = k0 + kc * EPC;
        const bool ok = (c < ROWS * 8) && (grow < rows) && (k < K);
        if constexpr (KIND == PQ_SRC_KC16) {
          const size_t off = ok ? (size_t)grow * op.ld + k : 0;
          v[i] = *reinterpret_cast<const uint4*>((const uint16_t*)op.p + off);
          okbits |= (ok ? 1u : 0u) << i;
        } else if constexpr (KIND == PQ_SRC_KC8) {
          const size_t off = ok ? (size_t)grow * op.ld + k : 0;
          v[i] = *reinterpret_cast<const uint4*>((const int8_t*)op.p + off);
          okbits |= (ok ? 1u : 0u) << i;
        } else if constexpr (KIND == PQ_SRC_BITS8) {
          const size_t off = ok ? (size_t)grow * op.ld + (k >> 3) : 0;
          raw[i] = *reinterpret_cast<const uint16_t*>((const uint8_t*)op.p + off);
          okbits |= (ok ? 1u : 0u) << i;
        } else {  // BITS16
          const size_t off = ok ? (size_t)grow * op.ld + (k >> 3) : 0;
          raw[i] = ((const uint8_t*)op.p)[off];
          okbits |= (ok ? 1u : 0u) << i;
        }
      }
    }
  }

  __device__ __forceinline__ void store(unsigned char* lds, int tid) const {
    if constexpr (kStrided) {
#pragma unroll
      for (int i = 0; i < NU; ++i) {
        const int u = tid + i * NT;
        if (u < ROWS / 8 * UPR) {
          const int r8 = u / UPR, kq = u % UPR;
          // transpose of 16-bit elements: v[i*KQ+j] holds rows r8*8..+7 at contraction index j
#pragma unroll
          for (int rr = 0; rr < 8; ++rr) {
            uint32_t o[KQ / 2];
#pragma unroll
            for (int p = 0; p < KQ / 2; ++p) {
              const uint4 lo4 = mask4(v[i * KQ + 2 * p], (okbits >> (i * KQ + 2 * p)) & 1u);
              const uint4 hi4 = mask4(v[i * KQ + 2 * p + 1], (okbits >> (i * KQ + 2 * p + 1)) & 1u);
              const uint32_t lo = (rr >> 1) == 0 ? lo4.x : (rr >> 1) == 1 ? lo4.y : (rr >> 1) == 2 ? lo4.z : lo4.w;
              const uint32_t hi = (rr >> 1) == 0 ? hi4.x : (rr >> 1) == 1 ? hi4.y : (rr >> 1) == 2 ? hi4.z : hi4.w;
              // result = [lo.half, hi.half]; v_perm selects bytes 0-3 from the 2nd operand, 4-7 from the 1st
              o[p] = (rr & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                              : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            if constexpr (KQ == 8) {
              *reinterpret_cast<uint4*>(lds + lds_off(r8 * 8 + rr, kq)) = make_uint4(o[0], o[1], o[2], o[3]);
            } else {
              *reinterpret_cast<uint2*>(lds + lds_off(r8 * 8 + rr, kq >> 1) + (kq & 1) * 8) = make_uint2(o[0], o[1]);
            }
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * NT;
        if (c < ROWS * 8) {
          const int r = c >> 3, kc = c & 7;
          uint4 out;
          if constexpr (KIND == PQ_SRC_BITS8) {
            // 16 bits -> 16 bytes of +1 (0x01) / -1 (0xFF): spread a nibble to one bit per byte with a
            // 24-bit multiply, then map byte values {0,1} through a byte permute.
            const uint32_t b = raw[i];
            uint32_t o[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const uint32_t nib = (b >> (4 * d)) & 0xFu;
              const uint32_t m = __umul24(nib, 0x00204081u) & 0x01010101u;
              o[d] = __builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, m);
            }
            out = mask4(make_uint4(o[0], o[1], o[2], o[3]), (okbits >> i) & 1u);
          } else if constexpr (KIND == PQ_SRC_BITS16) {
            // 8 bits -> 8 bf16 of +1 (0x3F80) / -1 (0xBF80)
            const uint32_t b = raw[i];
            uint32_t o[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const uint32_t x = (b >> (2 * d)) & 3u;
              o[d] = 0xBF80BF80u ^ (((x & 1u) << 15) | ((x & 2u) << 30));
            }
            out = mask4(make_uint4(o[0], o[1], o[2], o[3]), (okbits >> i) & 1u);
          } else {
            out = mask4(v[i], (okbits >> i) & 1u);
          }
          *reinterpret_cast<uint4*>(lds + lds_off(r, kc)) = out;
        }
      }
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Epilogue shared by both engines
// ---------------------------------------------------------------------------------------------
struct epi_state {
  float sc0;
  float mu;
  double psum;
};

__device__ __forceinline__ void epi_begin(const pq_epilogue& e, epi_state& st) {
  st.sc0 = e.dev_scale ? __fmul_rn(e.scale, *e.dev_scale) : e.scale;
  st.mu = e.mu_dev ? *e.mu_dev : 0.0f;
  st.psum = 0.0;
}

__device__ __forceinline__ float load_io(const void* p, int kind, size_t i) {
  return kind == PQ_OUT_BF16 ? bf16_to_f32(((const uint16_t*)p)[i]) : ((const float*)p)[i];
}

// acc_f: the accumulator as a real number; acc_i: as an integer (int8 engine / I32 output only)
template <typename AccT>
__device__ __forceinline__ void epi_elem(const pq_epilogue& e, epi_state& st, int m, int n, AccT acc, int acc_i) {
  const size_t ci = (size_t)m * e.ldc + n;
  if (e.out_kind == PQ_OUT_I32) {
    ((int*)e.C)[ci] = acc_i;
    return;
  }
  if (e.dot_comp) st.psum += (double)load_io(e.dot_comp, e.comp_kind, (size_t)m * e.ld_comp + n) * (double)acc;
  if (e.sign_bytes) {
    const uint32_t bit = (e.sign_bytes[(size_t)m * e.ld_sign + (n >> 3)] >> (n & 7)) & 1u;
    st.psum += bit ? (double)acc : -(double)acc;
  }
  float sc = st.sc0;
  if (e.row_div) sc = sc / e.row_div[m];
  AccT val = (AccT)sc * acc;
  if (e.maskW) {
    const double w = (double)load_io(e.maskW, e.mask_kind, ci);
    if (fabs(w - (double)st.mu) > (double)e.tau) val = (AccT)0;
  }
  if (e.accumulate) val += (AccT)load_io(e.C, e.out_kind, ci);
  if (e.out_kind == PQ_OUT_BF16) ((uint16_t*)e.C)[ci] = f32_to_bf16((float)val);
  else ((float*)e.C)[ci] = (float)val;
}

template <int NT>
__device__ __forceinline__ void epi_end(const pq_epilogue& e, epi_state& st, double* red, int block_linear) {
  if (e.partials) {
    double t = block_sum_d<NT>(st.psum, red);
    if (threadIdx.x == 0) e.partials[block_linear] = t;
  }
}

// Eight consecutive columns of one output row (MFMA engine; widths and leading dimensions are
// multiples of 8, so every group is either fully inside or fully outside the matrix).
__device__ __forceinline__ void load_io8(const void* p, int kind, size_t i, float* f) {
  if (kind == PQ_OUT_BF16) {
    const uint4 u = *reinterpret_cast<const uint4*>((const uint16_t*)p + i);
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xFFFF0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xFFFF0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xFFFF0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xFFFF0000u);
  } else {
    const float4 a = *reinterpret_cast<const float4*>((const float*)p + i);
    const float4 b = *reinterpret_cast<const float4*>((const float*)p + i + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
}

template <bool INT8>
__device__ __forceinline__ void epi_vec8(const pq_epilogue& e, epi_state& st, int m, int n, const uint4& r0,
                                         const uint4& r1) {
  const size_t ci = (size_t)m * e.ldc + n;
  if (e.out_kind == PQ_OUT_I32) {
    *reinterpret_cast<uint4*>((int*)e.C + ci) = r0;
    *reinterpret_cast<uint4*>((int*)e.C + ci + 4) = r1;
    return;
  }
  float acc[8];
  if constexpr (INT8) {
    acc[0] = (float)(int)r0.x; acc[1] = (float)(int)r0.y; acc[2] = (float)(int)r0.z; acc[3] = (float)(int)r0.w;
    acc[4] = (float)(int)r1.x; acc[5] = (float)(int)r1.y; acc[6] = (float)(int)r1.z; acc[7] = (float)(int)r1.w;
  } else {
    acc[0] = __uint_as_float(r0.x); acc[1] = __uint_as_float(r0.y); acc[2] = __uint_as_float(r0.z); acc[3] = __uint_as_float(r0.w);
    acc[4] = __uint_as_float(r1.x); acc[5] = __uint_as_float(r1.y); acc[6] = __uint_as_float(r1.z); acc[7] = __uint_as_float(r1.w);
  }
  if (e.dot_comp) {
    float c[8];
    load_io8(e.dot_comp, e.comp_kind, (size_t)m * e.ld_comp + n, c);
#pragma unroll
    for (int j = 0; j < 8; ++j) st.psum += (double)c[j] * (double)acc[j];
  }
  if (e.sign_bytes) {
    const uint32_t byte = e.sign_bytes[(size_t)m * e.ld_sign + (n >> 3)];
#pragma unroll
    for (int j = 0; j < 8; ++j) st.psum += ((byte >> j) & 1u) ? (double)acc[j] : -(double)acc[j];
  }
  float sc = st.sc0;
  if (e.row_div) sc = sc / e.row_div[m];
  float val[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) val[j] = __fmul_rn(sc, acc[j]);
  if (e.maskW) {
    float w[8];
    load_io8(e.maskW, e.mask_kind, ci, w);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (fabs((double)w[j] - (double)st.mu) > (double)e.tau) val[j] = 0.0f;
  }
  if (e.accumulate) {
    float c[8];
    load_io8(e.C, e.out_kind, ci, c);
#pragma unroll
    for (int j = 0; j < 8; ++j) val[j] += c[j];
  }
  if (e.out_kind == PQ_OUT_BF16) {
    *reinterpret_cast<uint4*>((uint16_t*)e.C + ci) =
        make_uint4(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]), pack_bf16x2(val[4], val[5]),
                   pack_bf16x2(val[6], val[7]));
  } else {
    *reinterpret_cast<float4*>((float*)e.C + ci) = make_float4(val[0], val[1], val[2], val[3]);
    *reinterpret_cast<float4*>((float*)e.C + ci + 4) = make_float4(val[4], val[5], val[6], val[7]);
  }
}

// ---------------------------------------------------------------------------------------------
// MFMA engine
// ---------------------------------------------------------------------------------------------
// One workgroup computes a BM x BN tile over the contraction range [z*kchunk, (z+1)*kchunk), z =
// blockIdx.y.  LDS holds two stages of both operand tiles; per 128-byte step there is a single
// barrier: after it, the registers prefetched during the previous step are written to the idle
// stage, the loads of the step after next are issued, and the MFMAs run on the ready stage.
template <int BM, int BN, int WGM, int WGN, bool INT8, int AK, int BKIND>
__global__ __launch_bounds__(WGM * WGN * 64) void mfma_gemm_kernel(int M, int N, int K, pq_operand A,
                                                                     pq_operand B, pq_epilogue epi,
                                                                     int nbn, int total_tiles, int kchunk,
                                                                     float* splitk_part, pq_gemm_group grp) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int EPB = INT8 ? 128 : 64;  // contraction elements per 128-byte LDS row
  constexpr int STAGE = (BM + BN) * 128;
  using acc_t = typename std::conditional<INT8, i32x16_t, f32x16_t>::type;

  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];
  __shared__ double red[NT / 64];

  // XCD-aware tile order: consecutive workgroups go to different XCDs, so give each XCD a
  // contiguous range of tiles (its L2 then sees the same A row-panel for a run of tiles).
  int pid = blockIdx.x;
  if ((total_tiles & 7) == 0) pid = (pid & 7) * (total_tiles >> 3) + (pid >> 3);
  const int bm = pid / nbn, bn = pid % nbn;
  int m0 = bm * BM;
  const int n0 = bn * BN;
  int kb = blockIdx.y * kchunk;
  int ke = min(K, kb + kchunk);
  if (grp.mode == 1) {          // rows of group z: [offsets[z], offsets[z+1])
    const int z = blockIdx.z;
    m0 += grp.offsets[z];
    M = grp.offsets[z + 1];
    if (m0 >= M) return;        // uniform for the workgroup
    B.p = (const char*)B.p + (size_t)z * grp.b_stride * (BKIND == PQ_SRC_KC8 ? 1 : 2);
  } else if (grp.mode == 2) {   // contraction range of group z, own output slab
    const int z = blockIdx.z;
    kb = grp.offsets[z];
    ke = grp.offsets[z + 1];
    epi.C = (char*)epi.C + (size_t)z * grp.c_stride * (epi.out_kind == PQ_OUT_BF16 ? 2 : 4);
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

  acc_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  tile_stage<AK, BM, NT> sa;
  tile_stage<BKIND, BN, NT> sb;
  const int nkt = ke > kb ? (ke - kb + EPB - 1) / EPB : 0;
  if (nkt > 0) {
    sa.load(A, m0, M, kb, ke, tid);
    sb.load(B, n0, N, kb, ke, tid);
    sa.store(smem, tid);
    sb.store(smem + BM * 128, tid);
    if (nkt > 1) {
      sa.load(A, m0, M, kb + EPB, ke, tid);
      sb.load(B, n0, N, kb + EPB, ke, tid);
    }
  }

  for (int kt = 0; kt < nkt; ++kt) {
    __syncthreads();  // stage kt&1 is complete; nobody still reads the other stage
    unsigned char* cur = smem + (kt & 1) * STAGE;
    unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
    if (kt + 1 < nkt) {
      sa.store(nxt, tid);
      sb.store(nxt + BM * 128, tid);
    }
    if (kt + 2 < nkt) {
      sa.load(A, m0, M, kb + (kt + 2) * EPB, ke, tid);
      sb.load(B, n0, N, kb + (kt + 2) * EPB, ke, tid);
    }
    const unsigned char* As = cur;
    const unsigned char* Bs = cur + BM * 128;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 af[TM], bf[TN];
      const int ch = 2 * ks + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const uint4*>(As + lds_off(wm0 + i * 32 + (lane & 31), ch));
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[j] = *reinterpret_cast<const uint4*>(Bs + lds_off(wn0 + j * 32 + (lane & 31), ch));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if constexpr (INT8)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4_t, af[i]),
                                                              __builtin_bit_cast(i32x4_t, bf[j]), acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                                __builtin_bit_cast(bf16x8_t, bf[j]), acc[i][j], 0, 0, 0);
        }
    }
  }
  __syncthreads();  // all MFMA operand reads are done: LDS is reused below

  // Epilogue: each wavefront passes its 32x32 accumulator blocks through a private LDS patch
  // (row stride 36 words: conflict-free both ways) so that a lane ends up with 8 consecutive
  // columns of one row and global loads/stores are 16 bytes wide.  With a split contraction the
  // raw fp32 accumulators go to this split's slab instead; splitk_reduce_kernel finishes the job.
  epi_state st;
  epi_begin(epi, st);
  float* slab = splitk_part ? splitk_part + (size_t)blockIdx.y * M * N : nullptr;
  uint32_t* stg = reinterpret_cast<uint32_t*>(smem) + wave * (32 * 36);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rr = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const auto elem = acc[i][j][v];  // copy out first: a vector element is not a bit_cast-able lvalue
        stg[rr * 36 + (lane & 31)] = __builtin_bit_cast(uint32_t, elem);
      }
      // wave-private patch: order this wave's LDS writes before its reads (other lanes' data)
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        const int rr = pass * 16 + (lane >> 2), c0 = (lane & 3) * 8;
        const int m = m0 + wm0 + i * 32 + rr, n = n0 + wn0 + j * 32 + c0;
        const uint4 r0 = *reinterpret_cast<const uint4*>(stg + rr * 36 + c0);
        const uint4 r1 = *reinterpret_cast<const uint4*>(stg + rr * 36 + c0 + 4);
        if (m < M && n < N) {
          if (slab) {
            *reinterpret_cast<uint4*>(slab + (size_t)m * N + n) = r0;
            *reinterpret_cast<uint4*>(slab + (size_t)m * N + n + 4) = r1;
          } else {
            epi_vec8<INT8>(epi, st, m, n, r0, r1);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  if (!slab) epi_end<NT>(epi, st, red, blockIdx.x);
}

// Second stage of a split contraction: sum the slabs in index order (deterministic), then apply
// the caller's epilogue.  One thread per 8 consecutive columns.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(int M, int N, int splits, const float* __restrict__ part,
                                                            pq_epilogue epi) {
  __shared__ double red[4];
  const size_t n8 = (size_t)N / 8, total = (size_t)M * n8;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  epi_state st;
  epi_begin(epi, st);
  if (idx < total) {
    const int m = (int)(idx / n8), n = (int)(idx % n8) * 8;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
    const size_t slab = (size_t)M * N;
    for (int z = 0; z < splits; ++z) {
      const float* p = part + z * slab + (size_t)m * N + n;
      const float4 x = *reinterpret_cast<const float4*>(p);
      const float4 y = *reinterpret_cast<const float4*>(p + 4);
      a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w;
      b.x += y.x; b.y += y.y; b.z += y.z; b.w += y.w;
    }
    const uint4 r0 = make_uint4(__float_as_uint(a.x), __float_as_uint(a.y), __float_as_uint(a.z), __float_as_uint(a.w));
    const uint4 r1 = make_uint4(__float_as_uint(b.x), __float_as_uint(b.y), __float_as_uint(b.z), __float_as_uint(b.w));
    epi_vec8<false>(epi, st, m, n, r0, r1);
  }
  epi_end<256>(epi, st, red, blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// Reference-precision engine: one thread per output element, fp64 accumulation, any source kind.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ double ref_elem(const pq_operand& op, int row, int k) {
  double v;
  switch (op.kind) {
    case PQ_SRC_KC32: v = ((const float*)op.p)[(size_t)row * op.ld + k]; break;
    case PQ_SRC_KS32: v = ((const float*)op.p)[(size_t)k * op.ld + row]; break;
    case PQ_SRC_KC16: v = bf16_to_f32(((const uint16_t*)op.p)[(size_t)row * op.ld + k]); break;
    case PQ_SRC_KS16: v = bf16_to_f32(((const uint16_t*)op.p)[(size_t)k * op.ld + row]); break;
    case PQ_SRC_KC8: v = ((const int8_t*)op.p)[(size_t)row * op.ld + k]; break;
    case PQ_SRC_KS8: v = ((const int8_t*)op.p)[(size_t)k * op.ld + row]; break;
    default: {
      const uint32_t byte = ((const uint8_t*)op.p)[(size_t)row * op.ld + (k >> 3)];
      v = ((byte >> (k & 7)) & 1u) ? 1.0 : -1.0;
    }
  }
  if (op.kdiv) v /= (double)op.kdiv[k];
  return v;
}

__global__ __launch_bounds__(256) void ref_gemm_kernel(int M, int N, int K, pq_operand A, pq_operand B,
                                                       pq_epilogue epi) {
  __shared__ double red[4];
  const int n = blockIdx.x * 16 + (threadIdx.x & 15);
  const int m = blockIdx.y * 16 + (threadIdx.x >> 4);
  epi_state st;
  epi_begin(epi, st);
  if (m < M && n < N) {
    double acc = 0.0;
    for (int k = 0; k < K; ++k) acc += ref_elem(A, m, k) * ref_elem(B, n, k);
    epi_elem<double>(epi, st, m, n, acc, (int)acc);
  }
  epi_end<256>(epi, st, red, blockIdx.y * gridDim.x + blockIdx.x);
}

template <int BM, int BN, int WGM, int WGN, bool INT8, int AK, int BKIND>
int launch_mfma(const pq_gemm_plan& pl, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                const pq_epilogue& epi, hipStream_t s, float* part, const pq_gemm_group& grp) {
  const int Mrows = grp.mode == 1 ? grp.max_rows : M;
  const int nbm = (Mrows + BM - 1) / BM, nbn = (N + BN - 1) / BN;
  const int tiles = nbm * nbn;
  dim3 grid(tiles, pl.splits, grp.mode ? grp.n_groups : 1), block(WGM * WGN * 64);
  mfma_gemm_kernel<BM, BN, WGM, WGN, INT8, AK, BKIND><<<grid, block, 0, s>>>(M, N, K, A, B, epi, nbn, tiles, pl.kchunk,
                                                                               pl.splits > 1 ? part : nullptr, grp);
  PQ_CHECK_LAUNCH("mfma_gemm_kernel");
  return PQ_OK;
}

template <bool INT8, int AK, int BKIND>
int launch_mfma_cfg(const pq_gemm_plan& pl, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                    const pq_epilogue& epi, hipStream_t s, float* part, const pq_gemm_group& grp) {
  if (pl.bm == 256) return launch_mfma<256, 256, 2, 4, INT8, AK, BKIND>(pl, M, N, K, A, B, epi, s, part, grp);
  return launch_mfma<128, 128, 2, 2, INT8, AK, BKIND>(pl, M, N, K, A, B, epi, s, part, grp);
}

}  // namespace

// Tile shape and contraction split for one GEMM.  A 256x256 tile (8 wavefronts, 128x64 each) when
// the output is large enough, else 128x128 (4 wavefronts); when the tiles alone cannot occupy the
// 256 compute units the contraction is split and reduced in a second, fixed-order pass.
pq_gemm_plan pq_plan_gemm(int engine, int M, int N, int K, bool int8) {
  pq_gemm_plan pl;
  memset(&pl, 0, sizeof(pl));
  pl.splits = 1;
  if (engine == 1) {
    pl.bm = pl.bn = 16;
    pl.kchunk = K;
    pl.red_blocks = ((M + 15) / 16) * ((N + 15) / 16);
    return pl;
  }
  const bool big = (M >= 256 && N >= 256);
  pl.bm = pl.bn = big ? 256 : 128;
  const long tiles = (long)((M + pl.bm - 1) / pl.bm) * ((N + pl.bn - 1) / pl.bn);
  pl.kchunk = K > 0 ? K : 1;
  if (!int8 && tiles > 0 && tiles <= 128 && K >= 512) {
    long want = 256 / tiles;
    if (want > 16) want = 16;
    long chunk = (K + want - 1) / want;
    chunk = (chunk + 255) / 256 * 256;          // whole 128-byte steps, at least four of them
    pl.kchunk = (int)chunk;
    pl.splits = (int)((K + chunk - 1) / chunk);
  }
  pl.red_blocks = pl.splits > 1 ? (int)(((size_t)M * (N / 8) + 255) / 256) : (int)tiles;
  pl.ws_bytes = pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
  return pl;
}

int pq_launch_gemm(int engine, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                   const pq_epilogue& epi, hipStream_t s, int prof_label, void* splitk_ws,
                   const pq_gemm_group* group) {
  if (M <= 0 || N <= 0) return PQ_OK;
  pq_gemm_group grp;
  memset(&grp, 0, sizeof(grp));
  if (group) grp = *group;
  if (grp.mode && engine == 1) return pq_set_error(PQ_ERR_DTYPE, "grouped GEMMs run on the MFMA engine only (bf16 I/O)");
  pq_prof_scope prof(prof_label, s);
  if (engine == 1) {
    dim3 grid((N + 15) / 16, (M + 15) / 16), block(256);
    ref_gemm_kernel<<<grid, block, 0, s>>>(M, N, K, A, B, epi);
    PQ_CHECK_LAUNCH("ref_gemm_kernel");
    return PQ_OK;
  }
  const int ak = A.kind, bk = B.kind;
  const bool int8 = (ak == PQ_SRC_KC8);
  pq_gemm_plan pl = pq_plan_gemm(0, M, N, K, int8);
  if (grp.mode) {               // groups already give parallelism; no contraction split
    pl.splits = 1;
    pl.kchunk = K > 0 ? K : 1;
    pl.bm = pl.bn = 128;
  }
  if (pl.splits > 1 && !splitk_ws) return pq_set_error(PQ_ERR_WORKSPACE, "split contraction needs scratch");
  float* part = (float*)splitk_ws;
  int rc;
  if (ak == PQ_SRC_KC8 && bk == PQ_SRC_BITS8) rc = launch_mfma_cfg<true, PQ_SRC_KC8, PQ_SRC_BITS8>(pl, M, N, K, A, B, epi, s, part, grp);
  else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_KC16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_KC16>(pl, M, N, K, A, B, epi, s, part, grp);
  else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_KS16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_KS16>(pl, M, N, K, A, B, epi, s, part, grp);
  else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_BITS16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_BITS16>(pl, M, N, K, A, B, epi, s, part, grp);
  else if (ak == PQ_SRC_KS16 && bk == PQ_SRC_KS16) rc = launch_mfma_cfg<false, PQ_SRC_KS16, PQ_SRC_KS16>(pl, M, N, K, A, B, epi, s, part, grp);
  else return pq_set_error(PQ_ERR_BAD_ARG, "no MFMA kernel for operand kinds (%d, %d)", ak, bk);
  if (rc != PQ_OK) return rc;
  if (pl.splits > 1) {
    splitk_reduce_kernel<<<pl.red_blocks, 256, 0, s>>>(M, N, pl.splits, part, epi);
    PQ_CHECK_LAUNCH("splitk_reduce_kernel");
  }
  return PQ_OK;
}
