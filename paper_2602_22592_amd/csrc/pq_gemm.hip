// Tiled MFMA GEMM for gfx950 with pluggable operand sources and epilogues, plus a
// reference-precision engine (fp64 products and sums on the fp64 matrix instruction) used for fp32 I/O.
//
//   C[m][n] (+)= epilogue( sum_k A(m,k) * B(n,k) )
//
// Operand sources (the 1-bit weights cross HBM and L2 as bits in every case: Sec. 3.1 W^INT1; App. A packing):
//   KC16 / KC8   contraction-contiguous rows, 16 bytes at a time;
//   KS16         contraction-strided sources (the transposed operands of the weight-gradient GEMMs);
//   BITS8/BITS16 packed sign bits, expanded to +/-1 (int8 or bf16).
// Two main loops share the kernel.  The streaming loop (256x256 tiles, whole contraction steps) sends operands from
// global memory straight into LDS: KC tiles as ROWS x 128 bytes, KS16 tiles as they lie in memory (read back with the
// transposing LDS read), and packed bits stay packed in LDS and are expanded in registers next to the MFMAs that consume
// them.  The register-staged loop (ragged contraction steps, 128x128 tiles, grouped contraction ranges) stages every
// operand as ROWS x 128 bytes with the contraction index contiguous: KS16 blocks are transposed in registers with byte
// permutes, bits are expanded on the way into LDS.
// A wavefront owns a (BM/WGM) x (BN/WGN) sub-tile as 32x32 MFMA blocks:
//   v_mfma_f32_32x32x16_bf16 / v_mfma_i32_32x32x32_i8, 16 bytes of operand per lane per issue.
// LDS rows are 128 bytes with the 16-byte chunk index XOR-swizzled by the row so that the MFMA
// operand reads, the row-wise stores and the transposed stores are all free of bank conflicts.
#include <stdlib.h>
#include <string.h>
#include <type_traits>
#include "pq_internal.h"

#ifdef PQ_TRACE
// Instrumented builds only (never the shipped library): cycle stamps of two workgroups of the streaming loops, taken at
// points where no LDS read is outstanding (the stamp is a scalar-memory read and shares the counter LDS reads use).
__device__ unsigned long long pq_trace_buf[6][8][64][2];   // [3 kernel kinds x 2 workgroups][wave][step][before/after the barrier]
extern "C" int pq_debug_read_trace(unsigned long long* host_out) {
  return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(pq_trace_buf), sizeof(unsigned long long) * 6 * 8 * 64 * 2) == hipSuccess ? 0 : -5;
}
#define PQ_STAMP(wg_slot, wave, step, which)                                                          \
  do {                                                                                                \
    if ((wg_slot) >= 0 && (step) < 64) {                                                              \
      const unsigned long long t_ = __builtin_readcyclecounter();                                     \
      if ((threadIdx.x & 63) == 0) pq_trace_buf[wg_slot][wave][step][which] = t_;                     \
    }                                                                                                 \
  } while (0)
#else
#define PQ_STAMP(wg_slot, wave, step, which) do { } while (0)
#endif

namespace {

__device__ __forceinline__ uint4 mask4(const uint4& t, bool keep) {
  const uint32_t m = keep ? 0xFFFFFFFFu : 0u;
  return make_uint4(t.x & m, t.y & m, t.z & m, t.w & m);
}

// Byte offset of 16-byte chunk c of row r in a tile whose rows are KB bytes (128 or 64).  The chunk
// index is XOR-swizzled by the row so that 8 consecutive rows at one logical chunk, and rows 8 apart
// at consecutive chunks (the transposing stores), fall into distinct 16-byte bank groups.
template <int KB>
__device__ __forceinline__ int lds_off(int r, int c) {
  if constexpr (KB == 128) return r * 128 + (((c ^ r ^ (r >> 3)) & 7) << 4);
  else return r * 64 + (((c ^ (r >> 1) ^ (r >> 3)) & 3) << 4);
}

// ---------------------------------------------------------------------------------------------
// Operand tile staging: global -> registers (load) and registers -> LDS (store)
// ---------------------------------------------------------------------------------------------
// Everything that does not change from one contraction step to the next (which rows and LDS slots a
// thread serves, their byte offsets) is computed once in setup(); a step then costs one load per
// 16 bytes with a uniform base pointer.  FAST instantiations are for shapes made of whole tiles:
// they carry no validity masks at all.  Otherwise loads stay unconditional (an out-of-range chunk
// reads element (0,0), which always exists, and is replaced by zeros on the way into LDS) so that
// all of a thread's loads are in flight together.
template <int KIND, int ROWS, int NT, int KB, bool FAST>
struct tile_stage {
  static constexpr int CPR = KB / 16;                        // 16-byte chunks per LDS row
  static constexpr int NCH = (ROWS * CPR + NT - 1) / NT;     // chunks per thread
  static constexpr bool kBits = (KIND == PQ_SRC_BITS8 || KIND == PQ_SRC_BITS16);
  static constexpr bool kStrided = (KIND == PQ_SRC_KS16);
  static constexpr int EPC = (KIND == PQ_SRC_KC8 || KIND == PQ_SRC_BITS8) ? 16 : 8;  // elements per chunk
  // KS16: a unit is 8 rows x KQ contraction indices (KQ 16-byte loads, transposed in registers);
  // KQ is the largest of 8, 4, 2 that still gives every thread a unit
  static constexpr int KQ = (ROWS * KB / 128 >= NT) ? 8 : (ROWS * KB / 64 >= NT) ? 4 : 2;
  static constexpr int UPR = (KB / 2) / KQ;                  // units per 8-row group
  static constexpr int UPC = 8 / KQ;                         // units per 16-byte chunk
  static constexpr int NU = (ROWS / 8 * UPR + NT - 1) / NT;  // units per thread
  static_assert(NT % CPR == 0 && NT % UPR == 0, "a thread keeps its contraction position across chunks");
  uint4 v[kBits ? 1 : (kStrided ? NU * KQ : NCH)];
  uint32_t raw[kBits ? NCH : 1];
  uint32_t boff[kStrided ? NU : NCH];      // byte offset of each load at contraction index 0
  uint32_t ldst[kStrided ? NU * 8 : NCH];  // LDS byte offset of each store
  uint32_t rowok;                          // bit i: chunk / unit i lies in a valid row
  uint32_t okbits;                         // validity of each load of the step in flight
  uint32_t jstride;                        // KS16: bytes between consecutive contraction indices
  int kpos;                                // this thread's contraction offset inside a tile (elements)

  // bytes of the source advanced per contraction element, times 8 (bits kinds advance 1/8 byte)
  static constexpr int ES8 = (KIND == PQ_SRC_KC16) ? 16 : (KIND == PQ_SRC_KC8) ? 8 : 1;

  __device__ __forceinline__ void setup(const pq_operand& op, int row0, int rows, int tid) {
    rowok = 0u;
    okbits = 0u;
    if constexpr (kStrided) {
      jstride = (uint32_t)op.ld * 2u;
      kpos = (tid % UPR) * KQ;
#pragma unroll
      for (int i = 0; i < NU; ++i) {
        const int u = tid + i * NT;
        const int r8 = u / UPR, kq = u % UPR;
        const int col = row0 + r8 * 8;
        const bool ok = (u < ROWS / 8 * UPR) && (col < rows);
        rowok |= (ok ? 1u : 0u) << i;
        boff[i] = ((uint32_t)(kq * KQ) * (uint32_t)op.ld + (uint32_t)(ok ? col : 0)) * 2u;
#pragma unroll
        for (int rr = 0; rr < 8; ++rr)
          ldst[i * 8 + rr] = (uint32_t)(lds_off<KB>(r8 * 8 + rr, kq / UPC) + (kq % UPC) * (KQ * 2));
      }
    } else {
      jstride = 0u;
      kpos = (tid % CPR) * EPC;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * NT;
        const int r = c / CPR, kc = c % CPR;
        const int grow = row0 + r;
        const bool ok = (c < ROWS * CPR) && (grow < rows);
        rowok |= (ok ? 1u : 0u) << i;
        const uint32_t rowb = (uint32_t)(ok ? grow : 0) * (uint32_t)op.ld;   // ld is in bytes for the bits kinds
        boff[i] = (kBits ? rowb : rowb * (uint32_t)(ES8 / 8)) + (uint32_t)(kc * EPC * ES8 / 8);
        ldst[i] = (uint32_t)lds_off<KB>(r, kc);
      }
    }
  }

  // k0: contraction index of the tile's first element; K: end of the valid contraction range.  The loads of
  // a step can be issued in `np` pieces (piece = 0..np-1, both compile-time constants after unrolling) so
  // that the caller can spread them between its MFMA groups.
  __device__ __forceinline__ void load(const pq_operand& op, int k0, int K, int piece = 0, int np = 1) {
    if constexpr (kStrided) {
      constexpr int NL = NU * KQ;
      const char* base = FAST ? (const char*)op.p + (size_t)k0 * jstride : (const char*)op.p;
      const uint32_t kbyte = FAST ? 0u : (uint32_t)k0 * jstride;
      if (piece == 0) okbits = 0u;
#pragma unroll
      for (int i = 0; i < NU; ++i) {
#pragma unroll
        for (int j = 0; j < KQ; ++j) {
          if (((i * KQ + j) * np) / NL != piece) continue;
          uint32_t off = boff[i] + (uint32_t)j * jstride;
          if constexpr (!FAST) {
            const bool ok = ((rowok >> i) & 1u) && (k0 + kpos + j < K);
            off = ok ? off + kbyte : 0u;
            okbits |= (ok ? 1u : 0u) << (i * KQ + j);
          }
          v[i * KQ + j] = *reinterpret_cast<const uint4*>(base + off);
        }
      }
    } else {
      const size_t kb8 = (size_t)k0 * ES8 / 8;
      const char* base = FAST ? (const char*)op.p + kb8 : (const char*)op.p;
      const bool kv = FAST ? true : (k0 + kpos < K);
      okbits = kv ? rowok : 0u;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        if ((i * np) / NCH != piece) continue;
        uint32_t off = boff[i];
        if constexpr (!FAST) off = ((okbits >> i) & 1u) ? off + (uint32_t)kb8 : 0u;
        if constexpr (KIND == PQ_SRC_BITS8) raw[i] = *reinterpret_cast<const uint16_t*>(base + off);
        else if constexpr (KIND == PQ_SRC_BITS16) raw[i] = *reinterpret_cast<const uint8_t*>(base + off);
        else v[i] = *reinterpret_cast<const uint4*>(base + off);
      }
    }
  }

  __device__ __forceinline__ uint4 valid(const uint4& t, int bit) const {
    if constexpr (FAST) return t;
    else return mask4(t, (okbits >> bit) & 1u);
  }

  // np > 1: only the chunks of piece `piece` (contraction-contiguous and bit kinds)
  __device__ __forceinline__ void store(unsigned char* lds, int tid, int piece = 0, int np = 1) const {
    if constexpr (kStrided) {
#pragma unroll
      for (int i = 0; i < NU; ++i) {
        const int u = tid + i * NT;
        if (u < ROWS / 8 * UPR) {
          // transpose of 16-bit elements: v[i*KQ+j] holds rows r8*8..+7 at contraction index j
#pragma unroll
          for (int rr = 0; rr < 8; ++rr) {
            uint32_t o[KQ / 2];
#pragma unroll
            for (int p = 0; p < KQ / 2; ++p) {
              const uint4 lo4 = valid(v[i * KQ + 2 * p], i * KQ + 2 * p);
              const uint4 hi4 = valid(v[i * KQ + 2 * p + 1], i * KQ + 2 * p + 1);
              const uint32_t lo = (rr >> 1) == 0 ? lo4.x : (rr >> 1) == 1 ? lo4.y : (rr >> 1) == 2 ? lo4.z : lo4.w;
              const uint32_t hi = (rr >> 1) == 0 ? hi4.x : (rr >> 1) == 1 ? hi4.y : (rr >> 1) == 2 ? hi4.z : hi4.w;
              // result = [lo.half, hi.half]; v_perm selects bytes 0-3 from the 2nd operand, 4-7 from the 1st
              o[p] = (rr & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                              : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            unsigned char* dst = lds + ldst[i * 8 + rr];
            if constexpr (KQ == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
            else if constexpr (KQ == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
            else *reinterpret_cast<uint32_t*>(dst) = o[0];
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        if ((i * np) / NCH != piece) continue;
        const int c = tid + i * NT;
        if (c < ROWS * CPR) {
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
            out = valid(make_uint4(o[0], o[1], o[2], o[3]), i);
          } else if constexpr (KIND == PQ_SRC_BITS16) {
            // 8 bits -> 8 bf16 of +1 (0x3F80) / -1 (0xBF80): move each (inverted) bit to a sign position
            const uint32_t nb = ~raw[i];
            uint32_t o[4];
#pragma unroll
            for (int d = 0; d < 4; ++d)
              o[d] = 0x3F803F80u | ((nb << (15 - 2 * d)) & 0x00008000u) | ((nb << (30 - 2 * d)) & 0x80000000u);
            out = valid(make_uint4(o[0], o[1], o[2], o[3]), i);
          } else {
            out = valid(v[i], i);
          }
          *reinterpret_cast<uint4*>(lds + ldst[i]) = out;
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
  if ((e.m_limit > 0 && m >= e.m_limit) || (e.n_limit > 0 && n >= e.n_limit)) return;
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
  if (e.col_div) val = val / (AccT)e.col_div[n];
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
// row_scale: sc0 / row_div[m] when the caller has it at hand (NaN = not given, it is formed here)
__device__ __forceinline__ void epi_vec8(const pq_epilogue& e, epi_state& st, int m, int n, const uint4& r0,
                                         const uint4& r1, float row_scale = __builtin_nanf("")) {
  const size_t ci = (size_t)m * e.ldc + n;
  if ((e.m_limit > 0 && m >= e.m_limit) || (e.n_limit > 0 && n >= e.n_limit)) return;
  const bool half = e.n_limit > 0 && n + 8 > e.n_limit;   // only the first four columns exist
  if (e.out_kind == PQ_OUT_I32) {
    *reinterpret_cast<uint4*>((int*)e.C + ci) = r0;
    if (!half) *reinterpret_cast<uint4*>((int*)e.C + ci + 4) = r1;
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
  if (e.row_div) sc = (row_scale == row_scale) ? row_scale : sc / e.row_div[m];
  float val[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) val[j] = __fmul_rn(sc, acc[j]);
  if (e.col_div) {
    const float4 c0 = *reinterpret_cast<const float4*>(e.col_div + n), c1 = *reinterpret_cast<const float4*>(e.col_div + n + 4);
    const float cd[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) val[j] = val[j] / cd[j];
  }
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
    if (half)
      *reinterpret_cast<uint2*>((uint16_t*)e.C + ci) = make_uint2(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]));
    else
      *reinterpret_cast<uint4*>((uint16_t*)e.C + ci) =
          make_uint4(pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3]), pack_bf16x2(val[4], val[5]),
                     pack_bf16x2(val[6], val[7]));
  } else {
    *reinterpret_cast<float4*>((float*)e.C + ci) = make_float4(val[0], val[1], val[2], val[3]);
    if (!half) *reinterpret_cast<float4*>((float*)e.C + ci + 4) = make_float4(val[4], val[5], val[6], val[7]);
  }
}

// ---------------------------------------------------------------------------------------------
// Streaming main loop (DTL instantiations): operands go from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers, no ds_write), and the contraction step is a fixed
// instruction order written as volatile asm statements: the fragment reads of MFMA group g+1 are issued
// before the MFMAs of group g, and the single barrier of a step sits before its last MFMA group, so the
// loads of the step after next and the first fragment reads of the next stage are issued under that
// group's MFMAs.  The compiler allocates the registers; the order of the statements is kept as written.
//   * contraction-contiguous operands (KC16, KC8): LDS tile [row][128 B], 16-byte chunks swizzled as
//     lds_off<128>; the swizzle is applied on the global side (lane l of a load instruction lands at LDS
//     byte 16 l of its 1 KB block, so it fetches the chunk that belongs there).
//   * contraction-strided operands (KS16): the tile stays as it is in memory, [64 contraction rows][512 B],
//     chunk c of row t stored at chunk c ^ 4 (t & 3); MFMA operands come from ds_read_b64_tr_b16, which
//     hands lane i of a 16-lane group element (i % 4) of the 8-byte row addressed by lane 4 e + i / 4,
//     e = 0..3: with lane j addressing (t = j / 4, 4 columns at 4 (j % 4)) lane i receives four consecutive
//     t of column i.
//   * packed-bit B operands stay packed in LDS (32-byte chunks of a row, one 16-byte direct load per
//     wavefront and chunk, three chunk buffers) and are expanded to MFMA operands in registers, one dword
//     behind each MFMA; with B that small the A operand gets a ring of four stages instead of two.
// A wait on asm-issued reads names the registers it releases ("+v"), which orders their uses after it.
// ---------------------------------------------------------------------------------------------
typedef int pq_i32x2 __attribute__((ext_vector_type(2)));
#define PQ_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define PQ_DS_READ128(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
#define PQ_DS_READ64(dst, addr, off) asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
#define PQ_DS_READ_TR(dst, addr, off) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off) : "memory")
// The B fragment is passed as the first MFMA operand: the accumulator block is then the transpose of the usual
// one, lane l holds output row (l & 31) and register v holds column 8 (v >> 2) + 4 (l >> 5) + (v & 3), i.e. runs of
// four consecutive columns of one row, which the epilogue turns into 16-byte stores without going through LDS.
// Wave priority for the phases between two barriers of a streaming loop: 3, 2, 1, 0 from the phase after the barrier to the
// one before the next.  The two wavefronts of a SIMD then take turns: at equal priority the older one issues its group of
// MFMAs, which drops it below the other, and so on -- without it the older wavefront wins every arbitration, runs through
// its whole step and waits at the barrier while the younger one, alone on the SIMD, cannot hide its LDS latencies.
#define PQ_SETPRIO(n) asm volatile("s_setprio %0" ::"n"(n))
#define PQ_MFMA_BF16(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %1, %0" : "+v"(acc) : "v"(a), "v"(b))
#define PQ_MFMA_I8(acc, a, b) asm volatile("v_mfma_i32_32x32x32_i8 %0, %2, %1, %0" : "+v"(acc) : "v"(a), "v"(b))

// MFMA operand of +/-1 values from packed bits (bit i set = +1, clear = -1, Eq. 4): 8 bits -> 8 bf16 (bits
// above the eighth are ignored), 16 bits -> 16 int8.
__device__ __forceinline__ i32x4_t pq_bits_to_bf16(uint32_t b) {
  const uint32_t nb = ~b;
  i32x4_t o;
#pragma unroll
  for (int d = 0; d < 4; ++d)
    o[d] = (int)(0x3F803F80u | ((nb << (15 - 2 * d)) & 0x00008000u) | ((nb << (30 - 2 * d)) & 0x80000000u));
  return o;
}
__device__ __forceinline__ i32x4_t pq_bits_to_i8(uint32_t b) {
  i32x4_t o;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t m = __umul24((b >> (4 * d)) & 0xFu, 0x00204081u) & 0x01010101u;
    o[d] = (int)__builtin_amdgcn_perm(0x000001FFu, 0x000001FFu, m);
  }
  return o;
}

// One fragment set of a 128x64 wavefront tile: four A and two B operands of 16 bytes per lane.  Operands
// read with ds_read_b128 are whole (q), transposing reads deliver 8-byte halves (h) that the register
// allocator places next to each other.
template <bool ATR, bool BTR>
struct pq_frag_set {
  i32x4_t qa[ATR ? 1 : 4], qb[BTR ? 1 : 2];
  pq_i32x2 ha[ATR ? 8 : 1], hb[BTR ? 4 : 1];
  static constexpr int NREADS = (ATR ? 8 : 4) + (BTR ? 4 : 2);
  __device__ __forceinline__ i32x4_t A(int i) const {
    if constexpr (ATR) return i32x4_t{ha[2 * i][0], ha[2 * i][1], ha[2 * i + 1][0], ha[2 * i + 1][1]};
    else return qa[i];
  }
  __device__ __forceinline__ i32x4_t B(int j) const {
    if constexpr (BTR) return i32x4_t{hb[2 * j][0], hb[2 * j][1], hb[2 * j + 1][0], hb[2 * j + 1][1]};
    else return qb[j];
  }
  // waits until at most N_OUT LDS operations are outstanding; naming the registers orders their uses after it
  template <int N_OUT>
  __device__ __forceinline__ void wait() {
    if constexpr (!ATR && !BTR)
      asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(qa[0]), "+v"(qa[1]), "+v"(qa[2]), "+v"(qa[3]), "+v"(qb[0]), "+v"(qb[1]) : "n"(N_OUT));
    else if constexpr (ATR && BTR)
      asm volatile("s_waitcnt lgkmcnt(%12)"
                   : "+v"(ha[0]), "+v"(ha[1]), "+v"(ha[2]), "+v"(ha[3]), "+v"(ha[4]), "+v"(ha[5]), "+v"(ha[6]), "+v"(ha[7]),
                     "+v"(hb[0]), "+v"(hb[1]), "+v"(hb[2]), "+v"(hb[3])
                   : "n"(N_OUT));
    else if constexpr (ATR && !BTR)
      asm volatile("s_waitcnt lgkmcnt(%10)"
                   : "+v"(ha[0]), "+v"(ha[1]), "+v"(ha[2]), "+v"(ha[3]), "+v"(ha[4]), "+v"(ha[5]), "+v"(ha[6]), "+v"(ha[7]),
                     "+v"(qb[0]), "+v"(qb[1])
                   : "n"(N_OUT));
    else
      asm volatile("s_waitcnt lgkmcnt(%8)"
                   : "+v"(qa[0]), "+v"(qa[1]), "+v"(qa[2]), "+v"(qa[3]), "+v"(hb[0]), "+v"(hb[1]), "+v"(hb[2]), "+v"(hb[3])
                   : "n"(N_OUT));
  }
};

// ---------------------------------------------------------------------------------------------
// MFMA engine
// ---------------------------------------------------------------------------------------------
// One workgroup computes a BM x BN tile over the contraction range [z*kchunk, (z+1)*kchunk), z =
// blockIdx.y.  Register-staged instantiations (DTL = false): LDS holds two stages of both operand tiles;
// per 128-byte step there is a single barrier: after it, the registers prefetched during the previous
// step are written to the idle stage, the loads of the step after next are issued, and the MFMAs run on
// the ready stage.  Streaming instantiations (DTL = true) are described above.
template <int BM, int BN, int WGM, int WGN, int KB, bool FAST, bool INT8, int AK, int BKIND, int AK2 = -1, int BK2 = -1, bool DTL = false>
__global__ __launch_bounds__(WGM * WGN * 64) void mfma_gemm_kernel(int M, int N, int K, pq_operand A,
                                                                     pq_operand B, pq_epilogue epi,
                                                                     int nbn, int total_tiles, int kchunk,
                                                                     float* splitk_part, pq_gemm_group grp,
                                                                     pq_phase2 ph2) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int EPB = INT8 ? KB : KB / 2;  // contraction elements per LDS row
  constexpr int STAGE = (BM + BN) * KB;
  using acc_t = typename std::conditional<INT8, i32x16_t, f32x16_t>::type;

  // Streaming instantiations with a packed-bit B operand keep that operand as bits in LDS (three buffers of
  // 32 bytes per row), which leaves room for a ring of four stages of the A operand.
  constexpr bool BBITS = DTL && (BKIND == PQ_SRC_BITS8 || BKIND == PQ_SRC_BITS16);
  constexpr int SMEM_BYTES = BBITS ? 4 * BM * KB + 3 * BN * 32 : 2 * STAGE;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
  __shared__ double red[NT / 64];
  __shared__ float rowscale[BM];                     // per-row scale of the tile (one division per row, not per element)

  // XCD-aware tile order: consecutive workgroups go to different XCDs, so give each XCD a
  // contiguous range of tiles (its L2 then sees the same A row-panel for a run of tiles).
  // Work items are ordered (contraction split, tile row, tile column) and XCD c takes the c-th eighth of
  // that order: with a split contraction an XCD then works on one split and a band of tile rows, so the
  // operand panels it streams are shared by its workgroups instead of being fetched by every XCD.
  // paired launches exist for the 128x128 kernel with contraction-strided operands only; elsewhere the test would
  // only turn kernel arguments into run-time selections
  if constexpr (BM == 128 && !DTL && AK == PQ_SRC_KS16 && BKIND == PQ_SRC_KS16 && AK2 < 0)
  if (grp.mode == 3 && blockIdx.z == 1) {            // uniform: the second problem of a paired launch
    A = grp.second.A; B = grp.second.B;
    M = grp.second.M; N = grp.second.N; nbn = grp.second.nbn;
    splitk_part = grp.second.part;
    epi.C = grp.second.C; epi.ldc = grp.second.ldc; epi.scale = grp.second.scale;
  }
  int pid = blockIdx.x, split = blockIdx.y;
  {
    const int nb = total_tiles * (int)gridDim.y;
    if ((nb & 7) == 0) {
      const int lin = blockIdx.x + total_tiles * blockIdx.y;
      const int w = (lin & 7) * (nb >> 3) + (lin >> 3);
      split = w / total_tiles;
      pid = w - split * total_tiles;
    }
  }
  const int bm = pid / nbn, bn = pid % nbn;
  int m0 = bm * BM;
  const int n0 = bn * BN;
  int kb = split * kchunk;
  int ke = min(K, kb + kchunk);
  int Mtot = M;                 // rows of C (a split's slab has Mtot rows)
  size_t slab_group = 0;        // offset of this group's rows in a slab (grouped contraction ranges)
  if (grp.mode == 1) {          // rows of group z: [offsets[z], offsets[z+1]); row tiles are numbered group after group
    int t = bm, z = 0;
    for (; z < grp.n_groups; ++z) {
      const int nt = (grp.offsets[z + 1] - grp.offsets[z] + BM - 1) / BM;
      if (t < nt) break;
      t -= nt;
    }
    if (z == grp.n_groups) return;   // uniform for the workgroup: the launch covers the worst-case tile count
    m0 = grp.offsets[z] + t * BM;
    M = grp.offsets[z + 1];
    B.p = (const char*)B.p + (size_t)z * grp.b_stride * (BKIND == PQ_SRC_KC8 ? 1 : 2);
    if (epi.col_div) epi.col_div += (size_t)z * grp.coldiv_stride;
  } else if (grp.mode == 2) {   // contraction range of group z, own output slab
    const int z = blockIdx.z;
    kb = grp.offsets[z];
    ke = grp.offsets[z + 1];
    if (gridDim.y > 1) {
      // the group's range in gridDim.y pieces of whole 64-element steps (the last ones may be empty: they leave zeros);
      // a slab holds the outputs of all groups, one under the other
      int chunk = (ke - kb + (int)gridDim.y - 1) / (int)gridDim.y;
      chunk = (chunk + 63) & ~63;
      kb = min(ke, kb + split * chunk);
      ke = min(ke, kb + chunk);
      slab_group = (size_t)z * M * N;
      Mtot = grp.n_groups * M;
    }
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

  tile_stage<AK, BM, NT, KB, FAST> sa;
  tile_stage<BKIND, BN, NT, KB, FAST> sb;
  sa.setup(A, m0, M, tid);
  sb.setup(B, n0, N, tid);
  const int nkt = ke > kb ? (ke - kb + EPB - 1) / EPB : 0;
  constexpr int NKS = KB / 32;   // MFMA issues along the contraction per LDS stage
  // Streaming loop with a fused second contraction of one or two 64-element steps: its operand tiles (32 KB each:
  // A2 step 0, B2 step 0, A2 step 1, B2 step 1) ride in on the ring's last four refills, which the main loop no longer
  // needs, instead of being requested after it (a chain of four memory latencies in front of 64 MFMAs per wavefront).
  // Tile j goes to ring stage (pf2_s0 + j) mod 4.
  bool pf2 = false;                                  // uniform
  [[maybe_unused]] const int pf2_s0 = nkt & 3;
  if constexpr (DTL && BBITS && AK2 == PQ_SRC_KC16 && (BK2 == PQ_SRC_KC16 || BK2 == PQ_SRC_KS16)) {
#ifndef PQ_NO_PF2
    pf2 = ph2.K2 > 0 && ph2.K2 <= 128 && ph2.K2 % 64 == 0 && nkt >= 4 && ((uintptr_t)ph2.A2.p % 16) == 0 && (ph2.A2.ld * 2) % 16 == 0 &&
          ((uintptr_t)ph2.B2.p % 16) == 0 && (ph2.B2.ld * 2) % 16 == 0 && (BK2 != PQ_SRC_KS16 || N % 8 == 0);
#endif
  }

  // per-thread LDS read offsets of the MFMA operand fragments (row part and swizzle part)
  int a_rb[TM], a_fx[TM], b_rb[TN], b_fx[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int r = wm0 + i * 32 + (lane & 31);
    a_rb[i] = lds_off<KB>(r, 0) & ~(KB - 1);
    a_fx[i] = (lds_off<KB>(r, 0) & (KB - 1)) >> 4;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int r = wn0 + j * 32 + (lane & 31);
    b_rb[j] = BM * KB + (lds_off<KB>(r, 0) & ~(KB - 1));
    b_fx[j] = (lds_off<KB>(r, 0) & (KB - 1)) >> 4;
  }
  uint4 af[2][TM], bf[2][TN];
  auto read_frags = [&](const unsigned char* stage, int ks, uint4* fa, uint4* fb) {
    const int ch = 2 * ks + (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const uint4*>(stage + a_rb[i] + ((ch ^ a_fx[i]) << 4));
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const uint4*>(stage + b_rb[j] + ((ch ^ b_fx[j]) << 4));
  };

  if constexpr (DTL) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature (LDS address-space casts are device-only)
    static_assert(BM == 256 && BN == 256 && WGM == 2 && WGN == 4 && KB == 128, "streaming loop: 256x256 tile on 8 wavefronts");
    constexpr bool ATR = (AK == PQ_SRC_KS16), BTR = (BKIND == PQ_SRC_KS16);
    constexpr bool BREG = BBITS;                      // B stays packed in LDS and is expanded per fragment
    constexpr int IPW = BREG ? 4 : 8;                 // 16-byte direct-load instructions per wavefront and stage
    constexpr int NSTAGE = BREG ? 4 : 2;              // depth of the LDS ring
    constexpr int STG = BREG ? BM * KB : STAGE;       // bytes per ring stage
    constexpr int RB = INT8 ? 16 : 8;                 // bytes of packed bits per B row and step
    constexpr int CH = 32 / RB;                       // steps covered by a 32-byte chunk of a packed row
    constexpr int BITS0 = NSTAGE * BM * KB;           // LDS offset of the three chunk buffers [256 rows][32 B]
    constexpr int AES = (AK == PQ_SRC_KC8) ? 1 : 2, BES = (BKIND == PQ_SRC_KC8) ? 1 : 2;
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(size_t)smem;
#ifdef PQ_TRACE
    const int trace_kind = INT8 ? 0 : (BBITS ? 1 : 2);
    const int trace_slot = (blockIdx.y == 0 && blockIdx.z == 0 && (blockIdx.x == 0 || blockIdx.x == 100)) ? 2 * trace_kind + (blockIdx.x == 100) : -1;
#endif

    // ---- direct loads: instruction block qi of an operand is 1 KB of its LDS tile --------------------
    const bool opB = !BREG && wv >= 4;                // wave-uniform
    const int q0 = BREG ? wv * 4 : (wv & 3) * 8;
    const char* src[IPW];
    size_t adv;                                       // source bytes per contraction step
    {
      auto kc_src = [&](const pq_operand& op, int row0, int rows, int es, int qi) {
        const int r = qi * 8 + (lane >> 3), pc = lane & 7;
        const int c = pc ^ ((r ^ (r >> 3)) & 7);      // logical chunk stored at physical chunk pc of row r
        const int grow = min(row0 + r, rows - 1);      // rows past the end re-read the last row (never stored)
        return (const char*)op.p + ((size_t)grow * op.ld + kb) * es + c * 16;
      };
      auto ks_src = [&](const pq_operand& op, int col0, int cols, int qi) {
        const int t = qi * 2 + (lane >> 5), pc = lane & 31;
        const int c = pc ^ (4 * (t & 3));
        int col = col0 + c * 8;
        if (col + 8 > cols) col = col0;                // columns past the end: any valid chunk
        return (const char*)op.p + ((size_t)(kb + t) * op.ld + col) * 2;
      };
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        if (opB) {
          if constexpr (BTR) src[i] = ks_src(B, n0, N, q0 + i);
          else src[i] = kc_src(B, n0, N, BES, q0 + i);
        } else {
          if constexpr (ATR) src[i] = ks_src(A, m0, M, q0 + i);
          else src[i] = kc_src(A, m0, M, AES, q0 + i);
        }
      }
      if (opB) adv = BTR ? (size_t)64 * B.ld * 2 : (size_t)128;
      else adv = ATR ? (size_t)64 * A.ld * 2 : (size_t)128;
    }
    auto issue = [&](int kt, int stage) {
      unsigned char* base = smem + stage * STG + (opB ? BM * KB : 0) + q0 * 1024;
#pragma unroll
      for (int i = 0; i < IPW; ++i)
        __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * adv, PQ_LDS_PTR(base + i * 1024), 16, 0, 0);
    };
    // tile j of the second contraction (step j >> 1; even: A2, odd: B2) into a ring stage, in the layouts of the
    // loaders above; the addresses are formed here, in the four steps that use them, not kept across the loop
    auto issue_ph2 = [&](int j, int stage) {
      if constexpr (AK2 >= 0) {
        unsigned char* base = smem + stage * STG + q0 * 1024;
        const int k2 = (j >> 1) * 64;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
          const int qi = q0 + i;
          const char* g;
          if (!(j & 1) || BK2 != PQ_SRC_KS16) {
            const pq_operand& op = (j & 1) ? ph2.B2 : ph2.A2;
            const int row0 = (j & 1) ? n0 : m0, rows = (j & 1) ? N : M;
            const int r = qi * 8 + (lane >> 3), pc = lane & 7;
            const int c = pc ^ ((r ^ (r >> 3)) & 7);
            const int grow = min(row0 + r, rows - 1);
            g = (const char*)op.p + ((size_t)grow * op.ld + k2) * 2 + c * 16;
          } else {
            const int t = qi * 2 + (lane >> 5), pc = lane & 31;
            const int c = pc ^ (4 * (t & 3));
            int col = n0 + c * 8;
            if (col + 8 > N) col = n0;
            g = (const char*)ph2.B2.p + ((size_t)(k2 + t) * ph2.B2.ld + col) * 2;
          }
          __builtin_amdgcn_global_load_lds(g, PQ_LDS_PTR(base + i * 1024), 16, 0, 0);
        }
      }
    };
    // Packed bits of B: a row's bits are fetched 32 bytes (CH steps) at a time, two lanes per row, so a chunk
    // (256 rows, 8 KB) is one 16-byte load instruction per wavefront every CH steps.  Lanes 0..31 take the first
    // 16 bytes of the wavefront's 32 rows and lanes 32..63 the second, so in LDS a block of 32 rows is
    // [half][row][16 B]: the per-step reads (8 or 16 bytes of 32 consecutive rows) then walk consecutive
    // 16-byte slots instead of a 32-byte row stride (rows 8 apart on the same banks).
    // The last chunk of a contraction range may be half a chunk (ranges are whole multiples of 128 indices):
    // its missing half re-reads the start of the range into a place no step uses.
    const int range_bytes = (ke - kb) >> 3;
    auto issue_bits = [&](int chunk, int buf) {
      const int row = min(n0 + wv * 32 + (lane & 31), N - 1);
      int off = chunk * 32 + (lane >> 5) * 16;
      if (off + 16 > range_bytes) off = 0;
      const char* g = (const char*)B.p + (size_t)row * B.ld + (kb >> 3) + off;
      __builtin_amdgcn_global_load_lds(g, PQ_LDS_PTR(smem + BITS0 + buf * (BN * 32) + wv * 1024), 16, 0, 0);
    };

    // ---- fragment read addresses (stage 0) ------------------------------------------------------------
    const int h = lane >> 5;
    uint32_t adA[ATR ? 4 : 8], adB[BTR ? 2 : 8];
    if constexpr (ATR) {
      const int tl = 8 * h + ((lane & 15) >> 2), cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), sw = 4 * ((lane & 15) >> 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = wm0 + 32 * i + cl;
        adA[i] = lds0 + tl * 512 + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
      }
    } else {
#pragma unroll
      for (int pp = 0; pp < 2; ++pp)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) adA[pp * 4 + ks] = lds0 + a_rb[pp] + (((2 * ks + h) ^ a_fx[pp]) << 4);
    }
    if constexpr (BTR) {
      const int tl = 8 * h + ((lane & 15) >> 2), cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), sw = 4 * ((lane & 15) >> 2);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = wn0 + 32 * j + cl;
        adB[j] = lds0 + BM * KB + tl * 512 + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) adB[j * 4 + ks] = lds0 + b_rb[j] + (((2 * ks + h) ^ b_fx[j]) << 4);
    }
    if constexpr (BREG) {
      // ---- ring of four stages: A streams as above, B stays packed ------------------------------------
      // A step's bits of a B row (8 or 16 bytes) are read once per wavefront tile column; the operand of
      // contraction sub-step s+1 is expanded from them in registers while the MFMAs of sub-step s issue,
      // one 4-byte piece behind each MFMA (the two wavefronts of a SIMD run in step, so a block of
      // expansion instructions ahead of a block of MFMAs would leave the matrix pipe idle for its length).
      // Every wavefront issues IPW direct loads of A per step, whatever the step (steps and chunks past the end
      // re-load the last one into a place nobody reads), plus one load of bits, ahead of them, in the first
      // step of a chunk.  At the barrier of step t at most 2 IPW loads stay in flight, which leaves A up to
      // step t + 1 and the bits issued up to step t - 2 in LDS (when a load of bits is among the last 2 IPW,
      // the wait merely covers one more load of A).  Chunk c is issued in the first step of chunk c - 2 and
      // goes to buffer c mod 3, whose previous content (chunk c - 3) was last read one barrier earlier.
      static_assert(!ATR, "packed B goes with a contraction-contiguous A");
      using bits_t = typename std::conditional<INT8, i32x4_t, pq_i32x2>::type;
      struct aset {
        i32x4_t q[4];
        __device__ __forceinline__ void wait4() { asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3])); }
        __device__ __forceinline__ void wait0() { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3])); }
      };
      struct bfrag { int e[8]; };                      // two operands of four dwords
      aset G0, G1;
      bits_t bq0, bq1;
      const uint32_t adQ0 = lds0 + BITS0 + (wn0 / 32) * 1024 + (lane & 31) * 16, adQ1 = adQ0 + 1024;
      const uint32_t sh = INT8 ? 16u * h : 8u * h;
      // constants of the expansion kept in registers (three-operand encodings take no literals)
      uint32_t kM = INT8 ? 0x000001FFu : 0x80008000u, kC = 0x3F803F80u;
      asm volatile("" : "+v"(kM), "+v"(kC));
      auto read_a = [&](aset& G, auto ks_c, uint32_t so) {
        constexpr int ks = decltype(ks_c)::value;
        const uint32_t p0 = adA[ks] + so, p1 = adA[4 + ks] + so;
        PQ_DS_READ128(G.q[0], p0, 0);
        PQ_DS_READ128(G.q[1], p1, 0);
        PQ_DS_READ128(G.q[2], p0, 8192);
        PQ_DS_READ128(G.q[3], p1, 8192);
      };
      auto read_bits = [&](uint32_t so) {
        const uint32_t p0 = adQ0 + so, p1 = adQ1 + so;
        if constexpr (INT8) { PQ_DS_READ128(bq0, p0, 0); PQ_DS_READ128(bq1, p1, 0); }
        else { PQ_DS_READ64(bq0, p0, 0); PQ_DS_READ64(bq1, p1, 0); }
      };
      // bits of sub-step ks in the form the piecewise expansion takes: int8: the 16 bits; bf16: the 8
      // inverted bits at positions 0..7 and again at 15..22, so that one shift by 15 - 2d puts bits 2d
      // and 2d + 1 on the two sign positions of dword d
      auto prep = [&](const bits_t& q, auto ks_c) -> uint32_t {
        constexpr int ks = decltype(ks_c)::value;
        if constexpr (INT8) return (uint32_t)q[ks] >> sh;
        else {
          const uint32_t nb = ((((uint32_t)q[ks >> 1] >> (16 * (ks & 1))) >> sh) & 0xFFu) ^ 0xFFu;
          return nb | (nb << 15);
        }
      };
      // dword d of an operand: bf16: sign bits from the prepared word over the pattern (1.0, 1.0);
      // int8: nibble d -> one bit per byte (24-bit multiply) -> bytes 0x01 / 0xFF (byte permute)
#define PQ_EXPAND(dst, y, d)                                                                                     \
  do {                                                                                                           \
    if constexpr (INT8)                                                                                          \
      asm volatile("v_bfe_u32 %0, %1, %2, 4\n\tv_mul_u32_u24 %0, 0x204081, %0\n\tv_and_b32 %0, 0x1010101, %0\n\t" \
                   "v_perm_b32 %0, %3, %3, %0"                                                                    \
                   : "=&v"(dst)                                                                                  \
                   : "v"(y), "n"(4 * (d)), "v"(kM));                                                             \
    else                                                                                                         \
      asm volatile("v_lshlrev_b32 %0, %2, %1\n\tv_and_or_b32 %0, %0, %3, %4"                                      \
                   : "=&v"(dst)                                                                                  \
                   : "v"(y), "n"(15 - 2 * (d)), "v"(kM), "v"(kC));                                               \
  } while (0)
#define PQ_MFMA_AB(i, j, G, f0, f1)                                                          \
  do {                                                                                       \
    if constexpr (INT8) PQ_MFMA_I8(acc[i][j], G.q[i], (j) ? f1 : f0);                        \
    else PQ_MFMA_BF16(acc[i][j], G.q[i], (j) ? f1 : f0);                                     \
  } while (0)
      // MFMAs of one sub-step; FROM: the first MFMA that is followed by expansion pieces (0 = all eight)
      auto mfma_x = [&](const aset& G, const bfrag& cur, bfrag& nxt, uint32_t y0, uint32_t y1, auto from_c) {
        constexpr int FROM = decltype(from_c)::value;
        const i32x4_t f0 = {cur.e[0], cur.e[1], cur.e[2], cur.e[3]}, f1 = {cur.e[4], cur.e[5], cur.e[6], cur.e[7]};
        if constexpr (FROM == 0) {
          PQ_MFMA_AB(0, 0, G, f0, f1); PQ_EXPAND(nxt.e[0], y0, 0);
          PQ_MFMA_AB(0, 1, G, f0, f1); PQ_EXPAND(nxt.e[1], y0, 1);
          PQ_MFMA_AB(1, 0, G, f0, f1); PQ_EXPAND(nxt.e[2], y0, 2);
          PQ_MFMA_AB(1, 1, G, f0, f1); PQ_EXPAND(nxt.e[3], y0, 3);
          PQ_MFMA_AB(2, 0, G, f0, f1); PQ_EXPAND(nxt.e[4], y1, 0);
          PQ_MFMA_AB(2, 1, G, f0, f1); PQ_EXPAND(nxt.e[5], y1, 1);
          PQ_MFMA_AB(3, 0, G, f0, f1); PQ_EXPAND(nxt.e[6], y1, 2);
          PQ_MFMA_AB(3, 1, G, f0, f1); PQ_EXPAND(nxt.e[7], y1, 3);
        } else {
          PQ_MFMA_AB(1, 0, G, f0, f1); PQ_EXPAND(nxt.e[0], y0, 0); PQ_EXPAND(nxt.e[1], y0, 1);
          PQ_MFMA_AB(1, 1, G, f0, f1); PQ_EXPAND(nxt.e[2], y0, 2);
          PQ_MFMA_AB(2, 0, G, f0, f1); PQ_EXPAND(nxt.e[3], y0, 3); PQ_EXPAND(nxt.e[4], y1, 0);
          PQ_MFMA_AB(2, 1, G, f0, f1); PQ_EXPAND(nxt.e[5], y1, 1);
          PQ_MFMA_AB(3, 0, G, f0, f1); PQ_EXPAND(nxt.e[6], y1, 2);
          PQ_MFMA_AB(3, 1, G, f0, f1); PQ_EXPAND(nxt.e[7], y1, 3);
        }
      };
      using c0 = std::integral_constant<int, 0>;
      using c1 = std::integral_constant<int, 1>;
      using c2 = std::integral_constant<int, 2>;
      using c3 = std::integral_constant<int, 3>;
      bfrag fc, fn;
      const int nch = (nkt + CH - 1) / CH;              // the last chunk may be half used
      if (nkt > 0) {
        issue_bits(0, 0);
        issue_bits(min(1, nch - 1), 1);
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s) issue(min(s, nkt - 1), s);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 1) * IPW) : "memory");
        asm volatile("s_barrier" ::: "memory");
        read_bits(0u);
        read_a(G0, c0{}, 0u);
        asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(bq0), "+v"(bq1));
        const uint32_t y0 = prep(bq0, c0{}), y1 = prep(bq1, c0{});
        PQ_EXPAND(fc.e[0], y0, 0); PQ_EXPAND(fc.e[1], y0, 1); PQ_EXPAND(fc.e[2], y0, 2); PQ_EXPAND(fc.e[3], y0, 3);
        PQ_EXPAND(fc.e[4], y1, 0); PQ_EXPAND(fc.e[5], y1, 1); PQ_EXPAND(fc.e[6], y1, 2); PQ_EXPAND(fc.e[7], y1, 3);
      }
      uint32_t so = 0u;
      int st = 0;
      int part = 0, buf = 0, chunk = 0;                 // position of the current step in the packed operand
      for (int kt = 0; kt < nkt; ++kt) {
        const int stn = (st + 1) & (NSTAGE - 1);
        const uint32_t sn = (uint32_t)stn * STG;
        const bool wrap = (part == CH - 1);
        const int partn = wrap ? 0 : part + 1;
        const int bufn = wrap ? (buf == 2 ? 0 : buf + 1) : buf;
        PQ_SETPRIO(2);
        read_a(G1, c1{}, so);
        G0.wait4();
        mfma_x(G0, fc, fn, prep(bq0, c1{}), prep(bq1, c1{}), c0{});
        PQ_SETPRIO(1);
        read_a(G0, c2{}, so);
        G1.wait4();
        mfma_x(G1, fn, fc, prep(bq0, c2{}), prep(bq1, c2{}), c0{});
        PQ_SETPRIO(0);
        read_a(G1, c3{}, so);
        G0.wait4();
        mfma_x(G0, fc, fn, prep(bq0, c3{}), prep(bq1, c3{}), c0{});
        G1.wait0();                                     // every LDS read of this step is complete
        PQ_STAMP(trace_slot, wv, kt, 0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * IPW) : "memory");
        asm volatile("s_barrier" ::: "memory");
        PQ_STAMP(trace_slot, wv, kt, 1);
        PQ_SETPRIO(3);
        if (part == 0) issue_bits(min(chunk + 2, nch - 1), buf == 0 ? 2 : buf - 1);   // (buf + 2) mod 3
        // refill the stage just read: with the step four ahead, or, once there is none, with a tile of the second contraction
        if (pf2 && kt + NSTAGE >= nkt && kt + NSTAGE - nkt < (ph2.K2 >> 5)) issue_ph2(kt + NSTAGE - nkt, st);
        else issue(min(kt + NSTAGE, nkt - 1), st);
        read_bits((uint32_t)(bufn * (BN * 32) + ((partn * RB) >> 4) * 512 + ((partn * RB) & 15)));   // past the last step: a place nobody uses
        read_a(G0, c0{}, sn);
        {
          const i32x4_t f0 = {fn.e[0], fn.e[1], fn.e[2], fn.e[3]}, f1 = {fn.e[4], fn.e[5], fn.e[6], fn.e[7]};
          PQ_MFMA_AB(0, 0, G1, f0, f1);
          PQ_MFMA_AB(0, 1, G1, f0, f1);
        }
        asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(bq0), "+v"(bq1));   // the bits were requested ahead of G0's reads
        mfma_x(G1, fn, fc, prep(bq0, c0{}), prep(bq1, c0{}), c1{});
        st = stn;
        so = sn;
        part = partn;
        buf = bufn;
        chunk += wrap ? 1 : 0;
      }
      PQ_SETPRIO(0);
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
#undef PQ_EXPAND
#undef PQ_MFMA_AB
    } else {
    using fset = pq_frag_set<ATR, BTR>;
    fset F0, F1;
    auto read_set = [&](fset& F, auto ks_c, uint32_t so) {
      constexpr int ks = decltype(ks_c)::value;
      if constexpr (ATR) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t pa = adA[i] + so;
          PQ_DS_READ_TR(F.ha[2 * i], pa, ks * 8192);
          PQ_DS_READ_TR(F.ha[2 * i + 1], pa, ks * 8192 + 2048);
        }
      } else {
        const uint32_t p0 = adA[ks] + so, p1 = adA[4 + ks] + so;
        PQ_DS_READ128(F.qa[0], p0, 0);
        PQ_DS_READ128(F.qa[1], p1, 0);
        PQ_DS_READ128(F.qa[2], p0, 8192);
        PQ_DS_READ128(F.qa[3], p1, 8192);
      }
      if constexpr (BTR) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint32_t pb = adB[j] + so;
          PQ_DS_READ_TR(F.hb[2 * j], pb, ks * 8192);
          PQ_DS_READ_TR(F.hb[2 * j + 1], pb, ks * 8192 + 2048);
        }
      } else {
        const uint32_t pb0 = adB[ks] + so, pb1 = adB[4 + ks] + so;
        PQ_DS_READ128(F.qb[0], pb0, 0);
        PQ_DS_READ128(F.qb[1], pb1, 0);
      }
    };
    auto mfma_set = [&](const fset& F) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const i32x4_t fa = F.A(i);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const i32x4_t fb = F.B(j);
          if constexpr (INT8) PQ_MFMA_I8(acc[i][j], fa, fb);
          else PQ_MFMA_BF16(acc[i][j], fa, fb);
        }
      }
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;
    using c2 = std::integral_constant<int, 2>;
    using c3 = std::integral_constant<int, 3>;
    constexpr int NR = fset::NREADS;

    if (nkt > 0) {
      issue(0, 0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      asm volatile("s_barrier" ::: "memory");
      if (nkt > 1) issue(1, 1);
      read_set(F0, c0{}, 0u);
    }
    for (int kt = 0; kt < nkt; ++kt) {
      const uint32_t so = (kt & 1) ? (uint32_t)STAGE : 0u, sn = (kt & 1) ? 0u : (uint32_t)STAGE;
      PQ_SETPRIO(2);
      read_set(F1, c1{}, so);
      F0.template wait<NR>();
      mfma_set(F0);
      PQ_SETPRIO(1);
      read_set(F0, c2{}, so);
      F1.template wait<NR>();
      mfma_set(F1);
      PQ_SETPRIO(0);
      read_set(F1, c3{}, so);
      F0.template wait<NR>();
      mfma_set(F0);
      F1.template wait<0>();                          // every LDS access of this step is complete
      PQ_STAMP(trace_slot, wv, kt, 0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the direct loads of the next stage have landed
      asm volatile("s_barrier" ::: "memory");
      PQ_STAMP(trace_slot, wv, kt, 1);
      PQ_SETPRIO(3);
      if (kt + 2 < nkt) issue(kt + 2, kt & 1);
      if (kt + 1 < nkt) read_set(F0, c0{}, sn);
      mfma_set(F1);
    }
    PQ_SETPRIO(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    }
#endif
  } else {
  if (nkt > 0) {
      sa.load(A, kb, ke);
      sb.load(B, kb, ke);
      sa.store(smem, tid);
      sb.store(smem + BM * KB, tid);
      const int k1 = nkt > 1 ? 1 : 0;
      sa.load(A, kb + k1 * EPB, ke);
      sb.load(B, kb + k1 * EPB, ke);
    }
    __syncthreads();
    if (nkt > 0) read_frags(smem, 0, af[0], bf[0]);

    // Steady state, one barrier per stage and no branches in the body: the registers hold tile kt+1,
    // which goes to the idle LDS stage while the loads of tile kt+2 are issued and the MFMAs run on
    // the ready stage; the operand fragments of the next MFMA group are read one group ahead.  On the
    // last steps the tile index is clamped, so the same tile is (harmlessly) staged again.
    for (int kt = 0; kt < nkt; ++kt) {
      unsigned char* cur = smem + (kt & 1) * STAGE;
      unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE;
      sa.store(nxt, tid);
      sb.store(nxt + BM * KB, tid);
      const int k2 = min(kt + 2, nkt - 1);
      sa.load(A, kb + k2 * EPB, ke);
      sb.load(B, kb + k2 * EPB, ke);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        if (ks + 1 < NKS) read_frags(cur, ks + 1, af[(ks + 1) & 1], bf[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            if constexpr (INT8)
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4_t, bf[ks & 1][j]),
                                                                __builtin_bit_cast(i32x4_t, af[ks & 1][i]), acc[i][j], 0, 0, 0);
            else
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[ks & 1][j]),
                                                                  __builtin_bit_cast(bf16x8_t, af[ks & 1][i]), acc[i][j], 0, 0, 0);
          }
      }
      __syncthreads();  // stage nxt is complete and nobody still reads stage cur
      read_frags(nxt, 0, af[0], bf[0]);
    }
  }
  __syncthreads();  // all MFMA operand reads are done: LDS is reused below

  // Optional second contraction (rank-r branch): rescale the first accumulator, then run a short bf16 loop
  // over K2 into the same tile.  The first operand tiles are requested before the rescale arithmetic and the
  // tiles of step s+1 before the MFMAs of step s (two LDS stages), so the memory latencies overlap with work
  // instead of standing in a row.
  constexpr bool PH2 = (AK2 >= 0);
  constexpr bool ACC_INT = INT8 && !PH2;
  f32x16_t accf[PH2 ? TM : 1][PH2 ? TN : 1];
  if constexpr (PH2) {
    constexpr int KS2 = KB / 2;                      // contraction elements per step
    tile_stage<AK2, BM, NT, KB, FAST> sa2;
    tile_stage<BK2, BN, NT, KB, FAST> sb2;
    sa2.setup(ph2.A2, m0, M, tid);
    sb2.setup(ph2.B2, n0, N, tid);
    // the first A2 tile (activation-sized, far away) is requested before the rescale arithmetic, the first B2 tile
    // (a small factor, cache-resident) after it: holding both across the rescale overflows the register file
    if (ph2.K2 > 0 && !pf2) sa2.load(ph2.A2, 0, ph2.K2);
    const float sc1 = ph2.dev_scale1 ? __fmul_rn(ph2.scale1, *ph2.dev_scale1) : ph2.scale1;
    if (ph2.row_div1) {                              // uniform: one divisor load and one division per row of the tile
      for (int r = tid; r < BM; r += NT) rowscale[r] = sc1 / ph2.row_div1[min(m0 + r, M - 1)];
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const float sr = ph2.row_div1 ? rowscale[wm0 + i * 32 + (lane & 31)] : sc1;   // a lane holds one row of a block
#pragma unroll
      for (int v = 0; v < 16; ++v)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const auto e1 = acc[i][j][v];
          accf[i][j][v] = (float)e1 * sr;
        }
    }
    if (pf2) {
#if defined(__HIP_DEVICE_COMPILE__)
      // both operands of every step already sit in the ring (all loads were waited for after the main loop)
      typedef short v4s_t __attribute__((ext_vector_type(4)));
      const int hh = lane >> 5;
      for (int s2 = 0; s2 < (ph2.K2 >> 6); ++s2) {
        const unsigned char* ta = smem + ((pf2_s0 + 2 * s2) & 3) * (BM * KB);
        const unsigned char* tb = smem + ((pf2_s0 + 2 * s2 + 1) & 3) * (BM * KB);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const int ch = 2 * ks + hh;
          uint4 fa[TM], fb[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const uint4*>(ta + a_rb[i] + ((ch ^ a_fx[i]) << 4));
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            if constexpr (BK2 == PQ_SRC_KS16) {
              // [64 contraction rows][256 columns] as it lies in memory, 16-byte chunks of a row swizzled by the row:
              // two transposing reads (rows 16 ks + 8 h + (0..3), then + 4) make the operand of 8 contraction indices
              const int tl = 8 * hh + ((lane & 15) >> 2), cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), sw = 4 * ((lane & 15) >> 2);
              const int col = wn0 + 32 * j + cl;
              const unsigned char* pb = tb + ks * 8192 + tl * 512 + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
              const v4s_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t*)(pb));
              const v4s_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t*)(pb + 2048));
              const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
              fb[j] = make_uint4(l2.x, l2.y, h2.x, h2.y);
            } else {
              fb[j] = *reinterpret_cast<const uint4*>(tb + (b_rb[j] - BM * KB) + ((ch ^ b_fx[j]) << 4));
            }
          }
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb[j]), __builtin_bit_cast(bf16x8_t, fa[i]),
                                                                   accf[i][j], 0, 0, 0);
        }
      }
#endif
    }
    if (ph2.K2 > 0 && !pf2) sb2.load(ph2.B2, 0, ph2.K2);
    int st2 = 0;
    for (int k2 = 0; k2 < (pf2 ? 0 : ph2.K2); k2 += KS2) {
      unsigned char* stage = smem + st2 * STAGE;
      sa2.store(stage, tid);
      sb2.store(stage + BM * KB, tid);
      const int kn = (k2 + KS2 < ph2.K2) ? k2 + KS2 : k2;   // the last step re-requests itself (harmless, never stored)
      sa2.load(ph2.A2, kn, ph2.K2);
      sb2.load(ph2.B2, kn, ph2.K2);
      __syncthreads();                               // this stage is complete; the other one is free again
      read_frags(stage, 0, af[0], bf[0]);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {             // the fragments of sub-step ks + 1 are read under the MFMAs of sub-step ks
        if (ks + 1 < NKS) read_frags(stage, ks + 1, af[(ks + 1) & 1], bf[(ks + 1) & 1]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            accf[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[ks & 1][j]),
                                                                 __builtin_bit_cast(bf16x8_t, af[ks & 1][i]), accf[i][j], 0, 0, 0);
      }
      st2 ^= 1;
    }
    __syncthreads();
  }
  // Epilogue: in a 32x32 accumulator block lane l holds row (l & 31) and, per group g = v >> 2, the four columns
  // 8 g + 4 (l >> 5) + (0..3).  One half-wave exchange per register (v_permlane32_swap: the upper half of the first
  // operand against the lower half of the second) gives the lower lanes the eight columns of the even groups and
  // the upper lanes those of the odd groups, so every lane stores 8 consecutive columns of its row at a time
  // (two neighbouring lanes = 16 consecutive columns) and nothing passes through LDS.  With a split contraction
  // the raw fp32 accumulators go to this split's slab instead; splitk_reduce_kernel finishes the job.
  epi_state st;
  epi_begin(epi, st);
  float* slab = splitk_part ? splitk_part + (size_t)split * Mtot * N + slab_group : nullptr;
  const bool row_scaled = !slab && epi.row_div != nullptr;   // uniform
  if (row_scaled) {
    for (int r = tid; r < BM; r += NT) rowscale[r] = st.sc0 / epi.row_div[min(m0 + r, M - 1)];
    __syncthreads();
  }
#ifdef PQ_NO_STAGE
  constexpr bool CAN_STAGE = false;
#else
  constexpr bool CAN_STAGE = (BM == 256 && BN == 256 && SMEM_BYTES >= 8 * 16384);
#endif
  // (store limits: fp32 outputs only, where a 16-byte chunk is four columns and the column limit a multiple of four)
  const bool staged = CAN_STAGE && (slab || ((epi.out_kind == PQ_OUT_F32 || (epi.out_kind == PQ_OUT_BF16 && epi.m_limit == 0 && epi.n_limit == 0)) &&
                                             !epi.col_div && !epi.maskW && !epi.accumulate && !epi.dot_comp &&
                                             !epi.sign_bytes));   // uniform
  if (staged) {
    const bool o16 = !slab && epi.out_kind == PQ_OUT_BF16;
    int tid_e = threadIdx.x;
    asm volatile("" : "+v"(tid_e));
    const int lane_e = tid_e & 63, wave_e = tid_e >> 6;
    const int wm0_e = (wave_e / WGN) * WM, wn0_e = (wave_e % WGN) * WN;
    unsigned char* wreg = smem + wave_e * 16384;
    char* outp = slab ? (char*)slab : (char*)epi.C;
    const size_t ldo = slab ? (size_t)N * 4 : (size_t)epi.ldc * (o16 ? 2 : 4);
    const int hh = lane_e >> 5;
    const int mlim = (!slab && epi.m_limit > 0 && epi.m_limit < M) ? epi.m_limit : M;
    const int nlim = (!slab && epi.n_limit > 0 && epi.n_limit < N) ? epi.n_limit : N;
    auto run = [&](auto o16_c) {
    constexpr bool o16 = decltype(o16_c)::value;
#pragma unroll
    for (int pass = 0; pass < (o16 ? 1 : 2); ++pass) {
#pragma unroll
      for (int ii = 0; ii < (o16 ? TM : TM / 2); ++ii) {
        const int i = o16 ? ii : pass * (TM / 2) + ii;
        const int rl = ii * 32 + (lane_e & 31);
        const int m = m0 + wm0_e + i * 32 + (lane_e & 31);
        const float rs = row_scaled ? rowscale[m - m0] : __builtin_nanf("");
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            uint32_t w[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              if (slab) {
                // copy the element out first: a vector element is not a bit_cast-able lvalue
                if constexpr (PH2) { const float e = accf[i][j][4 * g + t]; w[t] = __float_as_uint(e); }
                else { const auto e = acc[i][j][4 * g + t]; w[t] = __builtin_bit_cast(uint32_t, e); }
              } else {
                const float sc = row_scaled ? rs : st.sc0;
                float a;
                if constexpr (PH2) a = accf[i][j][4 * g + t];
                else a = (float)acc[i][j][4 * g + t];
                w[t] = __float_as_uint(__fmul_rn(sc, a));
              }
            }
            if constexpr (o16) {
              const uint2 o = make_uint2(pack_bf16x2(__uint_as_float(w[0]), __uint_as_float(w[1])),
                                         pack_bf16x2(__uint_as_float(w[2]), __uint_as_float(w[3])));
              *reinterpret_cast<uint2*>(wreg + rl * 128 + (((j * 4 + g) ^ (rl & 7)) << 4) + hh * 8) = o;
            } else {
              // written as asm with two wait states behind it: the compiler puts no distance between a 16-byte LDS store and a
              // VALU write to its data registers (it does for 16-byte global stores), and a staged epilogue whose last store was
              // followed at once by such writes lost that store's data in part
              const i32x4_t o = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
              const uint32_t ad = (uint32_t)(size_t)(wreg + rl * 256 + (((j * 8 + 2 * g + hh) ^ (rl & 7)) << 4));
              asm volatile("ds_write_b128 %0, %1\n\ts_nop 1" ::"v"(ad), "v"(o) : "memory");
            }
          }
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
      if constexpr (o16) {
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int rl = it * 8 + (lane_e >> 3), c = lane_e & 7;
          const uint4 v = *reinterpret_cast<const uint4*>(wreg + rl * 128 + ((c ^ (rl & 7)) << 4));
          const int m = m0 + wm0_e + rl, n = n0 + wn0_e + c * 8;
          if (m < M && n < N) *reinterpret_cast<uint4*>(outp + (size_t)m * ldo + (size_t)n * 2) = v;
        }
      } else {
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int rl = it * 4 + (lane_e >> 4), c = lane_e & 15;
          const uint4 v = *reinterpret_cast<const uint4*>(wreg + rl * 256 + ((c ^ (rl & 7)) << 4));
          const int m = m0 + wm0_e + pass * 64 + rl, n = n0 + wn0_e + c * 4;
          if (m < mlim && n < nlim) *reinterpret_cast<uint4*>(outp + (size_t)m * ldo + (size_t)n * 4) = v;
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_wave_barrier();
    }
    };
    if (o16) run(std::true_type{});
    else run(std::false_type{});
    if (!slab) epi_end<NT>(epi, st, red, blockIdx.x);
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm0 + i * 32 + (lane & 31);
    const float rs = row_scaled ? rowscale[m - m0] : __builtin_nanf("");
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        uint32_t x[4], y[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          uint32_t lo, hi;
          // copy the elements out first: a vector element is not a bit_cast-able lvalue
          if constexpr (PH2) {
            const float e0 = accf[i][j][8 * pr + t], e1 = accf[i][j][8 * pr + 4 + t];
            lo = __builtin_bit_cast(uint32_t, e0); hi = __builtin_bit_cast(uint32_t, e1);
          } else {
            const auto e0 = acc[i][j][8 * pr + t];
            const auto e1 = acc[i][j][8 * pr + 4 + t];
            lo = __builtin_bit_cast(uint32_t, e0); hi = __builtin_bit_cast(uint32_t, e1);
          }
          const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
          x[t] = sw[0];
          y[t] = sw[1];
        }
        const int n = n0 + wn0 + j * 32 + 8 * (2 * pr + (lane >> 5));
        const uint4 r0 = make_uint4(x[0], x[1], x[2], x[3]), r1 = make_uint4(y[0], y[1], y[2], y[3]);
        if (m < M && n < N) {
          if (slab) {
            *reinterpret_cast<uint4*>(slab + (size_t)m * N + n) = r0;
            *reinterpret_cast<uint4*>(slab + (size_t)m * N + n + 4) = r1;
          } else {
            epi_vec8<ACC_INT>(epi, st, m, n, r0, r1, rs);
          }
        }
      }
    }
  }
  if (!slab) epi_end<NT>(epi, st, red, blockIdx.x);
}

// Second stage of a split contraction: sum the slabs in index order (deterministic), then apply
// the caller's epilogue.  One thread per 8 consecutive columns.
// INT: the slabs hold int32 accumulators (int8 engine); their sum is exact.
template <bool INT>
__device__ __forceinline__ void splitk_reduce_body(int M, int N, int splits, const float* __restrict__ part, const pq_epilogue& epi,
                                                   int block) {
  __shared__ double red[4];
  const size_t n8 = (size_t)N / 8, total = (size_t)M * n8;
  const size_t idx = (size_t)block * 256 + threadIdx.x;
  epi_state st;
  epi_begin(epi, st);
  if (idx < total) {
    const int m = (int)(idx / n8), n = (int)(idx % n8) * 8;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
    int4 ia = make_int4(0, 0, 0, 0), ib = ia;
    const size_t slab = (size_t)M * N;
    // four slabs are requested together (slabs past the end repeat the last one and are dropped): a load behind
    // a loop-carried wait would cost one memory latency per slab; the sums still run in slab order
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
          if constexpr (INT) {
            ia.x += __float_as_int(x[u].x); ia.y += __float_as_int(x[u].y); ia.z += __float_as_int(x[u].z); ia.w += __float_as_int(x[u].w);
            ib.x += __float_as_int(y[u].x); ib.y += __float_as_int(y[u].y); ib.z += __float_as_int(y[u].z); ib.w += __float_as_int(y[u].w);
          } else {
            a.x += x[u].x; a.y += x[u].y; a.z += x[u].z; a.w += x[u].w;
            b.x += y[u].x; b.y += y[u].y; b.z += y[u].z; b.w += y[u].w;
          }
        }
    }
    if constexpr (INT) {
      epi_vec8<true>(epi, st, m, n, make_uint4((uint32_t)ia.x, (uint32_t)ia.y, (uint32_t)ia.z, (uint32_t)ia.w),
                     make_uint4((uint32_t)ib.x, (uint32_t)ib.y, (uint32_t)ib.z, (uint32_t)ib.w));
    } else {
      const uint4 r0 = make_uint4(__float_as_uint(a.x), __float_as_uint(a.y), __float_as_uint(a.z), __float_as_uint(a.w));
      const uint4 r1 = make_uint4(__float_as_uint(b.x), __float_as_uint(b.y), __float_as_uint(b.z), __float_as_uint(b.w));
      epi_vec8<false>(epi, st, m, n, r0, r1);
    }
  }
  epi_end<256>(epi, st, red, block);
}

template <bool INT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(int M, int N, int splits, const float* __restrict__ part,
                                                            pq_epilogue epi) {
  splitk_reduce_body<INT>(M, N, splits, part, epi, blockIdx.x);
}

// The reductions of a paired launch in one launch: the first nblk0 workgroups finish problem 0, the rest problem 1.
// Up to two scalar reductions of the same call (d alpha, d beta) ride along as the last workgroups of the grid.
__global__ __launch_bounds__(256) void splitk_reduce_pair_kernel(int splits, int nblk0, int nblk1, int M0, int N0,
                                                                 const float* __restrict__ part0, pq_epilogue epi0, int M1, int N1,
                                                                 const float* __restrict__ part1, pq_epilogue epi1, pq_reduce_job j0,
                                                                 pq_reduce_job j1) {
  const int b = blockIdx.x;
  if (b < nblk0) splitk_reduce_body<false>(M0, N0, splits, part0, epi0, b);
  else if (b < nblk0 + nblk1) splitk_reduce_body<false>(M1, N1, splits, part1, epi1, b - nblk0);
  else pq_reduce_job_body(b == nblk0 + nblk1 ? j0 : j1);
}

// ---------------------------------------------------------------------------------------------
// Reference-precision engine (fp32 I/O): any source kind, products and sums in fp64 on the matrix pipe
// (v_mfma_f64_16x16x4_f64).  A workgroup owns a 128x128 tile, a wavefront 64x64 of it; sixteen contraction
// indices of both operands are converted to fp64 on the way into LDS ([k][row], row stride 129 doubles).
// ---------------------------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ double ref_elem(const pq_operand& op, int row, int k) {
  if constexpr (KIND == PQ_SRC_KC32) return ((const float*)op.p)[(size_t)row * op.ld + k];
  else if constexpr (KIND == PQ_SRC_KS32) return ((const float*)op.p)[(size_t)k * op.ld + row];
  else if constexpr (KIND == PQ_SRC_KC16) return bf16_to_f32(((const uint16_t*)op.p)[(size_t)row * op.ld + k]);
  else if constexpr (KIND == PQ_SRC_KS16) return bf16_to_f32(((const uint16_t*)op.p)[(size_t)k * op.ld + row]);
  else if constexpr (KIND == PQ_SRC_KC8) return ((const int8_t*)op.p)[(size_t)row * op.ld + k];
  else if constexpr (KIND == PQ_SRC_KS8) return ((const int8_t*)op.p)[(size_t)k * op.ld + row];
  else {                                                // packed bits: one bit per weight, set = +1
    const uint32_t byte = ((const uint8_t*)op.p)[(size_t)row * op.ld + (k >> 3)];
    return ((byte >> (k & 7)) & 1u) ? 1.0 : -1.0;
  }
}

constexpr int REF_KB = 16;
// 128x128 tiles, or 64x64 when those would leave half of the compute units without one
static int ref_tile(int M, int N) { return (long)((M + 127) / 128) * ((N + 127) / 128) < 128 ? 64 : 128; }

// Sixteen contraction indices of TILE rows, fetched into registers (rows and indices past the end become zeros) and
// later written to LDS as [k][row].  Sources whose rows are contiguous in memory are read with the row index fastest
// over the lanes, the others with the contraction index.
template <int TILE>
struct ref_stage {
  static constexpr int PER = TILE / 16, LD = TILE + 1;
  double v[PER];
  __device__ __forceinline__ static void where(bool rows_fastest, int j, int& kk, int& rl) {
    const int tid = threadIdx.x;
    kk = rows_fastest ? tid / TILE + (256 / TILE) * j : (tid & 15);
    rl = rows_fastest ? tid % TILE : (tid >> 4) + 16 * j;
  }
  // All loads of a step are issued back to back (addresses clamped into the matrix, the kind decided once), so a
  // step waits for one memory latency and not for one per element.
  template <int KIND>
  __device__ __forceinline__ void fetch_kind(const pq_operand& op, int row0, int rows, int k0, int K) {
    constexpr bool rows_fastest = KIND == PQ_SRC_KS32 || KIND == PQ_SRC_KS16 || KIND == PQ_SRC_KS8;
    double d[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      int kk, rl;
      where(rows_fastest, j, kk, rl);
      v[j] = ref_elem<KIND>(op, min(row0 + rl, rows - 1), min(k0 + kk, K - 1));
      d[j] = op.kdiv ? (double)op.kdiv[min(k0 + kk, K - 1)] : 1.0;
    }
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      int kk, rl;
      where(rows_fastest, j, kk, rl);
      if (op.kdiv) v[j] /= d[j];
      if (row0 + rl >= rows || k0 + kk >= K) v[j] = 0.0;
    }
  }
  __device__ __forceinline__ void fetch(const pq_operand& op, int row0, int rows, int k0, int K) {
    switch (op.kind) {                                  // uniform
      case PQ_SRC_KC32: fetch_kind<PQ_SRC_KC32>(op, row0, rows, k0, K); break;
      case PQ_SRC_KS32: fetch_kind<PQ_SRC_KS32>(op, row0, rows, k0, K); break;
      case PQ_SRC_KC16: fetch_kind<PQ_SRC_KC16>(op, row0, rows, k0, K); break;
      case PQ_SRC_KS16: fetch_kind<PQ_SRC_KS16>(op, row0, rows, k0, K); break;
      case PQ_SRC_KC8: fetch_kind<PQ_SRC_KC8>(op, row0, rows, k0, K); break;
      case PQ_SRC_KS8: fetch_kind<PQ_SRC_KS8>(op, row0, rows, k0, K); break;
      default: fetch_kind<PQ_SRC_BITSF>(op, row0, rows, k0, K);   // packed bits, whatever the engine they were declared for
    }
  }
  __device__ __forceinline__ void store(const pq_operand& op, double* dst) const {
    const bool rows_fastest = op.kind == PQ_SRC_KS32 || op.kind == PQ_SRC_KS16 || op.kind == PQ_SRC_KS8;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      int kk, rl;
      where(rows_fastest, j, kk, rl);
      dst[kk * LD + rl] = v[j];
    }
  }
};

template <int TILE>
__global__ __launch_bounds__(256) void ref_gemm_kernel(int M, int N, int K, pq_operand A, pq_operand B, pq_epilogue epi) {
  typedef double f64x4_t __attribute__((ext_vector_type(4)));
  constexpr int LD = TILE + 1, WT = TILE / 2, NB = WT / 16;   // a wavefront owns WT x WT: NB x NB blocks of 16x16
  __shared__ double As[REF_KB * LD], Bs[REF_KB * LD];
  __shared__ double red[4];
  const int m0 = blockIdx.y * TILE, n0 = blockIdx.x * TILE;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * WT, wn = (wave & 1) * WT;
  const int li = lane & 15, lk = lane >> 4;
  f64x4_t acc[NB][NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f64x4_t{0.0, 0.0, 0.0, 0.0};
  ref_stage<TILE> ra, rb;
  if (K > 0) {
    ra.fetch(A, m0, M, 0, K);
    rb.fetch(B, n0, N, 0, K);
  }
  for (int k0 = 0; k0 < K; k0 += REF_KB) {
    ra.store(A, As);
    rb.store(B, Bs);
    __syncthreads();
    if (k0 + REF_KB < K) {                               // the next step's elements travel while this one multiplies
      ra.fetch(A, m0, M, k0 + REF_KB, K);
      rb.fetch(B, n0, N, k0 + REF_KB, K);
    }
#pragma unroll
    for (int kk = 0; kk < REF_KB; kk += 4) {
      // operand layout of the instruction: lane (li, lk) holds element (row li, contraction index lk) of either side
      double a[NB], b[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) a[i] = As[(kk + lk) * LD + wm + 16 * i + li];
#pragma unroll
      for (int j = 0; j < NB; ++j) b[j] = Bs[(kk + lk) * LD + wn + 16 * j + li];
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  epi_state st;
  epi_begin(epi, st);
  // result layout: register v of lane (li, lk) is element (row lk + 4 v, column li) of the 16x16 block
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = m0 + wm + 16 * i + lk + 4 * v, n = n0 + wn + 16 * j + li;
        const double c = acc[i][j][v];
        if (m < M && n < N) epi_elem<double>(epi, st, m, n, c, (int)c);
      }
  epi_end<256>(epi, st, red, blockIdx.y * gridDim.x + blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// Weight-gradient GEMMs (both operands bf16 with the contraction index as rows: dW = dY^T X over the tokens):
// a 256x256 tile on FOUR wavefronts.
// ---------------------------------------------------------------------------------------------
// With real (non-constant) operand data the chip runs these kernels against its power limit: the shader clock of the
// eight-wavefront kernel above falls from 2.3 GHz on all-zero operands to 1.7 GHz on normally distributed ones, and what
// LDS reads and direct loads cost shows as clock, not as stalls.  A wavefront that owns 128x128 of the tile reads eight
// operand blocks per sixteen MFMAs where a 128x64 one reads six per eight: a third less LDS traffic for the same products.
// Its 256 accumulator registers live in AGPRs (one wavefront per SIMD has 512 registers), which leaves the arch VGPRs for
// two fragment sets.  One wavefront per SIMD keeps the matrix pipe busy on its own as long as every wait it meets has
// been satisfied long before, so the order below is fixed (volatile asm statements): a stage is 32 contraction rows
// ([32][512 B] per operand, chunk c of row t at chunk c ^ 4 (t & 3), as in the streaming loop above), the ring has four
// stages, and per stage a wavefront issues 32 MFMAs in four groups of eight: behind each MFMA of groups 0 and 2 goes one
// operand block (two transposing reads) of the fragment set after the current one, behind each MFMA of group 1 one direct
// load of the stage three ahead.  The single barrier of a stage sits between groups 0 and 1: by then the wavefront's own
// loads of the next stage have landed (vmcnt), after it everybody's have and nobody reads the stage before the current
// one, whose slot the new loads take.  Past the last stage the loads re-request the last one into a free slot, so the
// counters stay uniform.
// The epilogue passes the accumulators through the wavefront's 32 KB of the ring, 64 rows at a time, and reads whole
// 512-byte rows back: raw slabs of a split contraction and plain fp32 outputs leave as 16-byte stores of whole rows, every
// other epilogue goes through epi_vec8 with eight consecutive columns per lane.
#define PQ_MFMA_BF16_ACC(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %2, %1, %0" : "+a"(acc) : "v"(a), "v"(b))
struct pq_frag_set_w4 {
  pq_i32x2 h[16];   // h[2q], h[2q+1]: the halves of operand block q; q = 0..3 rows of A (tile rows), 4..7 rows of B (tile columns)
  __device__ __forceinline__ i32x4_t op(int q) const { return i32x4_t{h[2 * q][0], h[2 * q][1], h[2 * q + 1][0], h[2 * q + 1][1]}; }
  __device__ __forceinline__ void wait_all() {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7]), "+v"(h[8]), "+v"(h[9]),
                   "+v"(h[10]), "+v"(h[11]), "+v"(h[12]), "+v"(h[13]), "+v"(h[14]), "+v"(h[15]));
  }
};

__global__ __launch_bounds__(256) void gemm_tn_w4_kernel(int M, int N, int K, pq_operand A, pq_operand B, pq_epilogue epi, int nbn,
                                                          int total_tiles, int kchunk, float* splitk_part) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int STG = 32768;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * STG];
  __shared__ double red[4];
  int pid = blockIdx.x, split = blockIdx.y;
  {   // XCD-aware order, as in mfma_gemm_kernel
    const int nb = total_tiles * (int)gridDim.y;
    if ((nb & 7) == 0) {
      const int lin = blockIdx.x + total_tiles * blockIdx.y;
      const int w = (lin & 7) * (nb >> 3) + (lin >> 3);
      split = w / total_tiles;
      pid = w - split * total_tiles;
    }
  }
  const int bm = pid / nbn, bn = pid % nbn;
  const int m0 = bm * 256, n0 = bn * 256;
  const int kb = split * kchunk, ke = min(K, kb + kchunk);
  const int nkt = ke > kb ? (ke - kb) >> 5 : 0;      // whole stages (the launcher checks)
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm0 = (wv >> 1) * 128, wn0 = (wv & 1) * 128;
  const uint32_t lds0 = (uint32_t)(size_t)smem;

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // direct loads: instruction block qi of an operand is 1 KB of its stage (two contraction rows); a wavefront owns four
  // blocks of each operand.  Columns past the end fetch the tile's first chunk (any valid address: never stored).
  const char* src[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int qi = wv * 4 + (i & 3);
    const int t = qi * 2 + (lane >> 5), pc = lane & 31;
    const int c = pc ^ (4 * (t & 3));
    const pq_operand& op = i < 4 ? A : B;
    const int col0 = i < 4 ? m0 : n0, cols = i < 4 ? M : N;
    int col = col0 + c * 8;
    if (col + 8 > cols) col = col0;
    src[i] = (const char*)op.p + ((size_t)(kb + t) * op.ld + col) * 2;
  }
  const size_t advA = (size_t)32 * A.ld * 2, advB = (size_t)32 * B.ld * 2;
  auto issue1 = [&](int kt, int slot, int i) {
    unsigned char* base = smem + slot * STG + wv * 4096;
    if (i < 4) __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * advA, PQ_LDS_PTR(base + i * 1024), 16, 0, 0);
    else __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * advB, PQ_LDS_PTR(base + 16384 + (i - 4) * 1024), 16, 0, 0);
  };

  // fragment read addresses (slot 0, contraction rows 0..15): see the transposing reads of the streaming loop
  uint32_t ad[8];
  {
    const int h = lane >> 5;
    const int tl = 8 * h + ((lane & 15) >> 2), cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), sw = 4 * ((lane & 15) >> 2);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int col = (q < 4 ? wm0 + 32 * q : wn0 + 32 * (q - 4)) + cl;
      ad[q] = lds0 + (q < 4 ? 0 : 16384) + tl * 512 + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
    }
  }
  pq_frag_set_w4 F0, F1;
  auto rd = [&](pq_frag_set_w4& F, int q, uint32_t so, auto ks_c) {
    constexpr int ks = decltype(ks_c)::value;
    const uint32_t pa = ad[q] + so;
    PQ_DS_READ_TR(F.h[2 * q], pa, ks * 8192);
    PQ_DS_READ_TR(F.h[2 * q + 1], pa, ks * 8192 + 2048);
  };
  auto mf = [&](const pq_frag_set_w4& X, int n) {
    const int i = n >> 2, j = (n & 3) ^ ((i & 1) ? 3 : 0);   // a block of B stays for two MFMAs in a row
    PQ_MFMA_BF16_ACC(acc[i][j], X.op(i), X.op(4 + j));
  };
  using c0 = std::integral_constant<int, 0>;
  using c1 = std::integral_constant<int, 1>;

  if (nkt > 0) {
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) issue1(min(u, nkt - 1), u, i);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int q = 0; q < 8; ++q) rd(F0, q, 0u, c0{});
  }
  for (int kt = 0; kt < nkt; ++kt) {
    const uint32_t so = (uint32_t)(kt & 3) * STG, sn = (uint32_t)((kt + 1) & 3) * STG;
    const int ktl = min(kt + 3, nkt - 1), sl = (kt + 3) & 3;
    F0.wait_all();
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      mf(F0, n);
      rd(F1, n, so, c1{});
    }
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // the wavefront's own loads of stage kt+1 have landed
    asm volatile("s_barrier" ::: "memory");            // everybody's have; nobody reads stage kt-1 any more
#pragma unroll
    for (int n = 8; n < 16; ++n) {
      mf(F0, n);
      issue1(ktl, sl, n - 8);
    }
    F1.wait_all();
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      mf(F1, n);
      if (n < 8) rd(F0, n, sn, c0{});                  // past the last stage: a slot nobody uses
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  asm volatile("s_barrier" ::: "memory");

  // ---- epilogue ----------------------------------------------------------------------------------
  epi_state st;
  epi_begin(epi, st);
  float* slab = splitk_part ? splitk_part + (size_t)split * M * N : nullptr;
  const bool plain = !slab && epi.out_kind == PQ_OUT_F32 && !epi.col_div && !epi.maskW && !epi.accumulate && !epi.dot_comp &&
                     !epi.sign_bytes;                 // uniform
  unsigned tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int lane_e = tid_e & 63, wave_e = tid_e >> 6;
  const int wm_e = (wave_e >> 1) * 128, wn_e = (wave_e & 1) * 128;
  unsigned char* wreg = smem + wave_e * STG;
  const int mlim = (!slab && epi.m_limit > 0 && epi.m_limit < M) ? epi.m_limit : M;
  const int nlim = (!slab && epi.n_limit > 0 && epi.n_limit < N) ? epi.n_limit : N;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int i = 2 * pass + ii;
          // (copy the elements out first: a vector element is not a bit_cast-able lvalue)
          const float w0 = acc[i][j][4 * g], w1 = acc[i][j][4 * g + 1], w2 = acc[i][j][4 * g + 2], w3 = acc[i][j][4 * g + 3];
          const i32x4_t o = {(int)__float_as_uint(w0), (int)__float_as_uint(w1), (int)__float_as_uint(w2), (int)__float_as_uint(w3)};
          const int rl = ii * 32 + (lane_e & 31);
          const uint32_t adw = (uint32_t)(size_t)(wreg + rl * 512 + (((j * 8 + 2 * g + (lane_e >> 5)) ^ (rl & 31)) << 4));
          // (asm with two wait states behind it: see the staged epilogue of mfma_gemm_kernel)
          asm volatile("ds_write_b128 %0, %1\n\ts_nop 1" ::"v"(adw), "v"(o) : "memory");
        }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    if (slab || plain) {
      char* outp = slab ? (char*)slab : (char*)epi.C;
      const size_t ldo = (slab ? (size_t)N : (size_t)epi.ldc) * 4;
#pragma unroll 4
      for (int it = 0; it < 32; ++it) {
        const int rl = it * 2 + (lane_e >> 5), c = lane_e & 31;
        uint4 v = *reinterpret_cast<const uint4*>(wreg + rl * 512 + ((c ^ (rl & 31)) << 4));
        if (!slab) {
          v.x = __float_as_uint(__fmul_rn(st.sc0, __uint_as_float(v.x)));
          v.y = __float_as_uint(__fmul_rn(st.sc0, __uint_as_float(v.y)));
          v.z = __float_as_uint(__fmul_rn(st.sc0, __uint_as_float(v.z)));
          v.w = __float_as_uint(__fmul_rn(st.sc0, __uint_as_float(v.w)));
        }
        const int m = m0 + wm_e + pass * 64 + rl, n = n0 + wn_e + c * 4;
        if (m < mlim && n < nlim) *reinterpret_cast<uint4*>(outp + (size_t)m * ldo + (size_t)n * 4) = v;
      }
    } else {
#pragma unroll 2
      for (int it = 0; it < 16; ++it) {
        const int rl = it * 4 + (lane_e >> 4), c = (lane_e & 15) * 2;
        const uint4 r0 = *reinterpret_cast<const uint4*>(wreg + rl * 512 + ((c ^ (rl & 31)) << 4));
        const uint4 r1 = *reinterpret_cast<const uint4*>(wreg + rl * 512 + (((c + 1) ^ (rl & 31)) << 4));
        const int m = m0 + wm_e + pass * 64 + rl, n = n0 + wn_e + c * 4;
        if (m < M && n < N) epi_vec8<false>(epi, st, m, n, r0, r1);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
  }
  if (!slab) epi_end<256>(epi, st, red, blockIdx.x);
#endif
}

template <int BM, int BN, int WGM, int WGN, int KB, bool FAST, bool INT8, int AK, int BKIND, int AK2 = -1, int BK2 = -1, bool DTL = false>
int launch_mfma(const pq_gemm_plan& pl, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                const pq_epilogue& epi, hipStream_t s, float* part, const pq_gemm_group& grp, const pq_phase2& ph2) {
  // grouped rows: every group may end in a partial tile, so at most ceil(rows / BM) + n_groups row tiles exist
  const int nbm = grp.mode == 1 ? (grp.max_rows + BM - 1) / BM + grp.n_groups : (M + BM - 1) / BM;
  const int nbn = (N + BN - 1) / BN;
  const int tiles = nbm * nbn;
  dim3 grid(tiles, pl.splits, grp.mode == 2 ? grp.n_groups : grp.mode == 3 ? 2 : 1), block(WGM * WGN * 64);
  mfma_gemm_kernel<BM, BN, WGM, WGN, KB, FAST, INT8, AK, BKIND, AK2, BK2, DTL><<<grid, block, 0, s>>>(
      M, N, K, A, B, epi, nbn, tiles, pl.kchunk, pl.splits > 1 ? part : nullptr, grp, ph2);
  PQ_CHECK_LAUNCH("mfma_gemm_kernel");
  return PQ_OK;
}

template <bool INT8, int AK, int BKIND, int AK2 = -1, int BK2 = -1>
int launch_mfma_cfg(const pq_gemm_plan& pl, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                    const pq_epilogue& epi, hipStream_t s, float* part, const pq_gemm_group& grp, const pq_phase2& ph2) {
  constexpr int EPB = INT8 ? 128 : 64;
  if (pl.bm == 256) {
    // whole tiles everywhere: the instantiation without validity masks
    const bool whole = grp.mode == 0 && M % 256 == 0 && N % 256 == 0 && K % EPB == 0 && pl.kchunk % EPB == 0 &&
                       ph2.K2 % 64 == 0;
    // Streaming main loop: plain tiles or row groups (expert segments as row ranges), whole contraction steps in every
    // split, rows of both operands 16-byte aligned.  Ragged M or N are fine there (edge rows are clamped, never stored).
    constexpr bool kinds_ok = (AK == PQ_SRC_KC16 || AK == PQ_SRC_KS16 || AK == PQ_SRC_KC8) &&
                              (BKIND == PQ_SRC_KC16 || BKIND == PQ_SRC_KS16 || BKIND == PQ_SRC_BITS8 || BKIND == PQ_SRC_BITS16);
    if constexpr (kinds_ok) {
      const long aes = AK == PQ_SRC_KC8 ? 1 : 2;
      const bool a_ok = (A.ld * aes) % 16 == 0 && ((uintptr_t)A.p % 16) == 0 && (AK != PQ_SRC_KS16 || M % 8 == 0);
      // packed rows are fetched in 16-byte halves of 32-byte chunks: ranges of whole multiples of 128 contraction
      // indices, a split's range starting on a chunk
      constexpr bool b_bits = (BKIND == PQ_SRC_BITS8 || BKIND == PQ_SRC_BITS16);
      const bool b_ok = b_bits ? (K % 128 == 0 && (pl.splits == 1 || pl.kchunk % 256 == 0) && B.ld % 16 == 0 && ((uintptr_t)B.p % 16) == 0) :
                        ((B.ld * 2) % 16 == 0 && ((uintptr_t)B.p % 16) == 0 && (BKIND != PQ_SRC_KS16 || N % 8 == 0));
      const bool stream = (grp.mode == 0 || grp.mode == 1) && K % EPB == 0 && pl.kchunk % EPB == 0 && a_ok && b_ok && M >= 1 && N >= 1;
#ifndef PQ_NO_W4
      // weight gradients: the four-wavefront kernel (whole 32-row stages in every split; no per-row divisor, no int32 output)
      if constexpr (AK == PQ_SRC_KS16 && BKIND == PQ_SRC_KS16 && AK2 < 0) {
        if (grp.mode == 0 && ph2.K2 == 0 && K % 32 == 0 && pl.kchunk % 32 == 0 && a_ok && b_ok && !A.kdiv && !B.kdiv && !epi.row_div &&
            epi.out_kind != PQ_OUT_I32) {
          const int nbm = (M + 255) / 256, nbn = (N + 255) / 256;
          dim3 grid(nbm * nbn, pl.splits), block(256);
          gemm_tn_w4_kernel<<<grid, block, 0, s>>>(M, N, K, A, B, epi, nbn, nbm * nbn, pl.kchunk, pl.splits > 1 ? part : nullptr);
          PQ_CHECK_LAUNCH("gemm_tn_w4_kernel");
          return PQ_OK;
        }
      }
#endif
      if (stream) {
        if (whole) return launch_mfma<256, 256, 2, 4, 128, true, INT8, AK, BKIND, AK2, BK2, true>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
        return launch_mfma<256, 256, 2, 4, 128, false, INT8, AK, BKIND, AK2, BK2, true>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
      }
    }
    if (whole) return launch_mfma<256, 256, 2, 4, 128, true, INT8, AK, BKIND, AK2, BK2>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    return launch_mfma<256, 256, 2, 4, 128, false, INT8, AK, BKIND, AK2, BK2>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
  }
  return launch_mfma<128, 128, 2, 2, 128, false, INT8, AK, BKIND, AK2, BK2>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Rank-r products with a long row dimension: C[M][128] = scale * A[M][K] B^T, bf16, A with the contraction index
// contiguous.  B is [128][K] (H = X A^T of the high-precision branch, Sec. 3.2) or, contraction-strided, [K][128]
// (dH = alpha dY B of its backward), then with sum(comp * (A B^T)) as a side result (d alpha).
// ---------------------------------------------------------------------------------------------
// With 128 output columns the tile engine has one workgroup per CU and two loads in flight per thread, so it runs as
// a chain of memory latencies, and it needs a split contraction with slabs to occupy the chip at all.  Here a
// workgroup of four wavefronts owns 64 (or 32) rows and the whole contraction: the operand tiles of a 64-element step
// ([64][128 B] of A, chunks swizzled by row as in the tile engine, then 16 KB of B: [128][128 B] the same way, or
// [64][256 B] as it lies in memory for the transposing LDS reads) go straight into a ring of six LDS stages, five
// steps ahead of the MFMAs, so about 120 KB per CU are in flight and nothing is reduced afterwards; one barrier per step.
constexpr int SK_BN = 128;

// BM = 64: wavefront w computes rows 32 (w >> 1) and columns 64 (w & 1), six stages of 24 KB.  BM = 32: one row block,
// wavefront w computes columns 32 w, seven stages of 20 KB (twice the workgroups for the same rows: B is streamed by
// twice as many CUs, A by each of them half as long).
// I8: int8 operands (128 contraction elements per 128-byte step, exact int32 accumulation) and the de-quantising
// epilogue of the INT8 high-precision branch: value = ((scale / row_div[m]) * acc) / col_div[n], each step rounded to fp32.
template <bool BTR, int BM, bool I8>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const void* __restrict__ A, long lda,
                                                         const void* __restrict__ B, long ldb, int M, int K,
                                                         uint16_t* __restrict__ C, long ldc, float scale,
                                                         const uint16_t* __restrict__ comp, long ld_comp,
                                                         double* __restrict__ partials, const float* __restrict__ row_div,
                                                         const float* __restrict__ col_div) {
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(BM == 64 || BM == 32, "one or two 32-row blocks");
  static_assert(!(I8 && BTR), "int8 operands are contraction-contiguous");
  constexpr int ES = I8 ? 1 : 2;                      // bytes per operand element
  constexpr int NA = BM / 8;                          // 1 KB load blocks of A per stage; B has 16
  constexpr int LPW = (NA + 16) / 4;                  // load blocks per wavefront and stage
  constexpr int NST = BM == 64 ? 6 : 7;               // ring stages
  constexpr int STAGE = (NA + 16) * 1024;
  constexpr int NJ = BM == 64 ? 2 : 1;                // 32-column blocks per wavefront
  static_assert((NA + 16) % 4 == 0 && NST * STAGE <= 150 * 1024, "even split of the loads; the ring fits LDS");
  __shared__ __attribute__((aligned(16))) unsigned char smem[NST * STAGE];
  __shared__ double red[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = blockIdx.x * BM;
  const int wr0 = BM == 64 ? (wv >> 1) * 32 : 0;      // the wavefront's rows and columns inside the tile
  const int wc0 = BM == 64 ? (wv & 1) * 64 : wv * 32;
  const int nkt = (K * ES) >> 7;
  const uint32_t lds0 = (uint32_t)(size_t)smem;

  // direct loads: lane l of a load lands at byte 16 l of its 1 KB block.  A, and a contraction-contiguous B: a block is
  // 8 rows x 128 B and lane l fetches physical chunk l & 7 of row 8 b + (l >> 3).  Contraction-strided B: a block is
  // 4 contraction rows x 256 B and lane l fetches physical chunk l & 15 of row 4 b + (l >> 4).
  const char* src[LPW];
  size_t adv[LPW];                                    // source bytes per contraction step
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int b = wv * LPW + i;                       // 0..NA-1: A, then 16 blocks of B
    if (BTR && b >= NA) {
      const int t = (b - NA) * 4 + (lane >> 4), pc = lane & 15;
      const int c = pc ^ (4 * (t & 3));
      src[i] = (const char*)B + ((size_t)t * ldb + c * 8) * 2;
      adv[i] = (size_t)64 * ldb * 2;
    } else {
      const int r = (b < NA ? b : b - NA) * 8 + (lane >> 3), pc = lane & 7;
      const int c = pc ^ ((r ^ (r >> 3)) & 7);
      src[i] = b < NA ? (const char*)A + ((size_t)min(m0 + r, M - 1) * lda) * ES + c * 16   // rows past the end: the last row
                      : (const char*)B + ((size_t)r * ldb) * ES + c * 16;
      adv[i] = 128;
    }
  }
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * adv[i], PQ_LDS_PTR(smem + stage * STAGE + (wv * LPW + i) * 1024), 16, 0, 0);
  };

  // fragment addresses in stage 0.  A (and a contraction-contiguous B): row l & 31 of the wavefront's block, logical
  // chunk 2 ks + (l >> 5).  Contraction-strided B: the transposing read takes, per lane, the address of four
  // consecutive columns in contraction row 8 (l >> 5) + ((l & 15) >> 2) (+ 4 for the second half of the operand).
  const int h = lane >> 5;
  uint32_t adA[4], adB[NJ][BTR ? 1 : 4];
  {
    const int ra = wr0 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) adA[ks] = lds0 + ra * 128 + ((((2 * ks + h) ^ ra ^ (ra >> 3)) & 7) << 4);
    if constexpr (BTR) {
      const int tl = 8 * h + ((lane & 15) >> 2), cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3), sw = 4 * ((lane & 15) >> 2);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int col = wc0 + 32 * j + cl;
        adB[j][0] = lds0 + NA * 1024 + tl * 256 + (((col >> 3) ^ sw) << 4) + (col & 7) * 2;
      }
    } else {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int rb = wc0 + j * 32 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) adB[j][ks] = lds0 + NA * 1024 + rb * 128 + ((((2 * ks + h) ^ rb ^ (rb >> 3)) & 7) << 4);
      }
    }
  }
  using acc_t = typename std::conditional<I8, i32x16_t, f32x16_t>::type;
  acc_t acc[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0;

#pragma unroll
  for (int st = 0; st < NST - 1; ++st) issue(min(st, nkt - 1), st);   // steps past the end: the last one again, never read
  int st = 0;
  for (int kt = 0; kt < nkt; ++kt) {
    // all but the NST - 2 latest steps have landed: this step's tiles are there (for this wavefront; the barrier makes
    // it everybody's), and every wavefront is past its reads of the stage that is refilled next
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * LPW) : "memory");
    asm volatile("s_barrier" ::: "memory");
    issue(min(kt + NST - 1, nkt - 1), st == 0 ? NST - 1 : st - 1);
    const uint32_t so = (uint32_t)(st * STAGE);
    i32x4_t fa[4];
    if constexpr (BTR) {
      constexpr int RPS = 1 + 2 * NJ;                 // LDS reads per sub-step
      pq_i32x2 hb[2][2 * NJ];                         // two sub-steps of B in flight: [parity][2 j + half]
      uint32_t pb[NJ];
#pragma unroll
      for (int j = 0; j < NJ; ++j) pb[j] = adB[j][0] + so;
#define PQ_SK_READ(ks)                                                                      \
  do {                                                                                      \
    PQ_DS_READ128(fa[ks], adA[ks] + so, 0);                                                 \
    PQ_DS_READ_TR(hb[(ks) & 1][0], pb[0], (ks) * 4096);                                      \
    PQ_DS_READ_TR(hb[(ks) & 1][1], pb[0], (ks) * 4096 + 1024);                               \
    if constexpr (NJ == 2) {                                                                \
      PQ_DS_READ_TR(hb[(ks) & 1][2 * (NJ - 1)], pb[NJ - 1], (ks) * 4096);                    \
      PQ_DS_READ_TR(hb[(ks) & 1][2 * (NJ - 1) + 1], pb[NJ - 1], (ks) * 4096 + 1024);         \
    }                                                                                       \
  } while (0)
#define PQ_SK_MFMA(ks, NOUT)                                                                                      \
  do {                                                                                                            \
    if constexpr (NJ == 2)                                                                                        \
      asm volatile("s_waitcnt lgkmcnt(%5)"                                                                        \
                   : "+v"(fa[ks]), "+v"(hb[(ks) & 1][0]), "+v"(hb[(ks) & 1][1]), "+v"(hb[(ks) & 1][2 * (NJ - 1)]),  \
                     "+v"(hb[(ks) & 1][2 * (NJ - 1) + 1])                                                         \
                   : "n"(NOUT));                                                                                  \
    else                                                                                                          \
      asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(fa[ks]), "+v"(hb[(ks) & 1][0]), "+v"(hb[(ks) & 1][1]) : "n"(NOUT)); \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                                              \
      const i32x4_t b = {hb[(ks) & 1][2 * j][0], hb[(ks) & 1][2 * j][1], hb[(ks) & 1][2 * j + 1][0], hb[(ks) & 1][2 * j + 1][1]}; \
      PQ_MFMA_BF16(acc[j], fa[ks], b);                                                                            \
    }                                                                                                             \
  } while (0)
      PQ_SK_READ(0);
      PQ_SK_READ(1);
      PQ_SK_MFMA(0, RPS);
      PQ_SK_READ(2);
      PQ_SK_MFMA(1, RPS);
      PQ_SK_READ(3);
      PQ_SK_MFMA(2, RPS);
      PQ_SK_MFMA(3, 0);
#undef PQ_SK_READ
#undef PQ_SK_MFMA
    } else {
      constexpr int RPS = 1 + NJ;
      i32x4_t fb[NJ][4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        PQ_DS_READ128(fa[ks], adA[ks] + so, 0);
#pragma unroll
        for (int j = 0; j < NJ; ++j) PQ_DS_READ128(fb[j][ks], adB[j][ks] + so, 0);
      }
#define PQ_SK_MFMA(ks)                                                                                             \
  do {                                                                                                             \
    if constexpr (NJ == 2)                                                                                         \
      asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(fa[ks]), "+v"(fb[0][ks]), "+v"(fb[NJ - 1][ks]) : "n"((3 - (ks)) * RPS)); \
    else                                                                                                           \
      asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(fa[ks]), "+v"(fb[0][ks]) : "n"((3 - (ks)) * RPS));              \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                                                               \
      if constexpr (I8) PQ_MFMA_I8(acc[j], fa[ks], fb[j][ks]);                                                     \
      else PQ_MFMA_BF16(acc[j], fa[ks], fb[j][ks]);                                                                \
    }                                                                                                              \
  } while (0)
      PQ_SK_MFMA(0);
      PQ_SK_MFMA(1);
      PQ_SK_MFMA(2);
      PQ_SK_MFMA(3);
#undef PQ_SK_MFMA
    }
    st = st == NST - 1 ? 0 : st + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the redundant loads of the last steps are done before the workgroup ends

  // the B fragment was the first MFMA operand: lane l holds row l & 31, register v column 8 (v >> 2) + 4 (l >> 5) + (v & 3)
  const int m = m0 + wr0 + (lane & 31);
  double psum = 0.0;
  if (m < M) {
    const float sc = row_div ? scale / row_div[m] : scale;
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = wc0 + j * 32 + 8 * g + 4 * h;
        if constexpr (I8) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = __fmul_rn(sc, (float)acc[j][4 * g + e]);
          if (col_div) {                             // uniform
            const float4 cd = *reinterpret_cast<const float4*>(col_div + n);
            v[0] = v[0] / cd.x; v[1] = v[1] / cd.y; v[2] = v[2] / cd.z; v[3] = v[3] / cd.w;
          }
          *reinterpret_cast<uint2*>(C + (size_t)m * ldc + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          continue;
        }
        if (comp) {                                  // uniform
          const uint2 u = *reinterpret_cast<const uint2*>(comp + (size_t)m * ld_comp + n);
          psum += (double)__uint_as_float(u.x << 16) * (double)acc[j][4 * g];
          psum += (double)__uint_as_float(u.x & 0xFFFF0000u) * (double)acc[j][4 * g + 1];
          psum += (double)__uint_as_float(u.y << 16) * (double)acc[j][4 * g + 2];
          psum += (double)__uint_as_float(u.y & 0xFFFF0000u) * (double)acc[j][4 * g + 3];
        }
        const float v0 = __fmul_rn(sc, (float)acc[j][4 * g]), v1 = __fmul_rn(sc, (float)acc[j][4 * g + 1]);
        const float v2 = __fmul_rn(sc, (float)acc[j][4 * g + 2]), v3 = __fmul_rn(sc, (float)acc[j][4 * g + 3]);
        *reinterpret_cast<uint2*>(C + (size_t)m * ldc + n) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
      }
  }
  if (partials) {                                    // uniform: one partial sum per workgroup, added in a fixed order
    const double t = block_sum_d<256>(psum, red);
    if (tid == 0) partials[blockIdx.x] = t;
  }
#endif
}

// The two weight gradients of the rank-128 branch, dB = alpha dY^T H and dA = dH^T X (Sec. 3.2, STE backward): the
// contraction runs over the tokens and both operands are stored token-major.  Same ring as above with both tiles as
// they lie in memory ([64 tokens][128 B] of the wide operand's 64 columns, [64 tokens][256 B] of the rank-128 one)
// and transposing LDS reads for both.  A workgroup owns 64 columns of the wide operand and one of 4 to 16 token
// ranges (blockIdx.y), and writes a 64 x 128 fp32 tile of that range's slab; blockIdx.z selects the problem.  For dA the wide
// operand is X, so the tile is the transpose of the output's and is stored transposed (dA is [128][d_in]).
struct skt_problem {
  const uint16_t* W;   // wide operand [T][ldw], M columns used
  long ldw;
  const uint16_t* R;   // rank-128 operand [T][ldr]
  long ldr;
  int M;               // multiple of 64
  int trans;           // 0: slab[split][M][128], 1: slab[split][128][M]
  float* slab;
};

__global__ __launch_bounds__(256) void skinny_tn_pair_kernel(skt_problem p0, skt_problem p1, int tokens_per_split) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NST = 6, LPW = 6, STAGE = 24 * 1024;
  __shared__ __attribute__((aligned(16))) unsigned char smem[NST * STAGE];
  const skt_problem& p = blockIdx.z ? p1 : p0;        // uniform
  const int m0 = blockIdx.x * 64;
  if (m0 >= p.M) return;                              // uniform, ahead of every barrier
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int split = blockIdx.y;
  const size_t kb = (size_t)split * tokens_per_split;
  const int nkt = tokens_per_split >> 6;
  const uint32_t lds0 = (uint32_t)(size_t)smem;
  const int wr0 = (wv >> 1) * 32, wc0 = (wv & 1) * 64;

  // direct loads, lane l at byte 16 l of a 1 KB block.  Wide operand: a block is 8 tokens x 128 B, lane l fetches
  // physical chunk l & 7 of token 8 b + (l >> 3); rank-128 operand: 4 tokens x 256 B, chunk l & 15 of token 4 b + (l >> 4).
  // Chunks are XOR-swizzled by the token's two low bits so that the transposing reads spread over the banks.
  const char* src[LPW];
  size_t adv[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int b = wv * LPW + i;                       // 0..7: wide operand, 8..23: rank-128 operand
    if (b < 8) {
      const int t = b * 8 + (lane >> 3), pc = lane & 7;
      const int c = pc ^ (2 * (t & 3));
      src[i] = (const char*)p.W + ((kb + t) * p.ldw + m0 + c * 8) * 2;
      adv[i] = (size_t)64 * p.ldw * 2;
    } else {
      const int t = (b - 8) * 4 + (lane >> 4), pc = lane & 15;
      const int c = pc ^ (4 * (t & 3));
      src[i] = (const char*)p.R + ((kb + t) * p.ldr + c * 8) * 2;
      adv[i] = (size_t)64 * p.ldr * 2;
    }
  }
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < LPW; ++i)
      __builtin_amdgcn_global_load_lds(src[i] + (size_t)kt * adv[i], PQ_LDS_PTR(smem + stage * STAGE + (wv * LPW + i) * 1024), 16, 0, 0);
  };

  // transposing reads: per lane the address of four consecutive columns in token 8 (l >> 5) + ((l & 15) >> 2) of a
  // 16-token sub-step (+ 4 tokens for the second half of the operand)
  const int h = lane >> 5, q = (lane & 15) >> 2;
  const int tl = 8 * h + q, cl = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  uint32_t adW, adR[2];
  {
    const int col = wr0 + cl;
    adW = lds0 + tl * 128 + ((((col >> 3) ^ (2 * q)) & 7) << 4) + (col & 7) * 2;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int cr = wc0 + 32 * j + cl;
      adR[j] = lds0 + 8 * 1024 + tl * 256 + (((cr >> 3) ^ (4 * q)) << 4) + (cr & 7) * 2;
    }
  }
  f32x16_t acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

#pragma unroll
  for (int st = 0; st < NST - 1; ++st) issue(min(st, nkt - 1), st);
  int st = 0;
  for (int kt = 0; kt < nkt; ++kt) {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * LPW) : "memory");
    asm volatile("s_barrier" ::: "memory");
    issue(min(kt + NST - 1, nkt - 1), st == 0 ? NST - 1 : st - 1);
    const uint32_t so = (uint32_t)(st * STAGE);
    const uint32_t pw = adW + so, pr0 = adR[0] + so, pr1 = adR[1] + so;
    pq_i32x2 hw[2][2], hr[2][4];                      // two sub-steps in flight: [parity][...]
#define PQ_SKT_READ(ks)                                                     \
  do {                                                                      \
    PQ_DS_READ_TR(hw[(ks) & 1][0], pw, (ks) * 2048);                         \
    PQ_DS_READ_TR(hw[(ks) & 1][1], pw, (ks) * 2048 + 512);                   \
    PQ_DS_READ_TR(hr[(ks) & 1][0], pr0, (ks) * 4096);                        \
    PQ_DS_READ_TR(hr[(ks) & 1][1], pr0, (ks) * 4096 + 1024);                 \
    PQ_DS_READ_TR(hr[(ks) & 1][2], pr1, (ks) * 4096);                        \
    PQ_DS_READ_TR(hr[(ks) & 1][3], pr1, (ks) * 4096 + 1024);                 \
  } while (0)
#define PQ_SKT_MFMA(ks, NOUT)                                                                                    \
  do {                                                                                                           \
    asm volatile("s_waitcnt lgkmcnt(%6)"                                                                         \
                 : "+v"(hw[(ks) & 1][0]), "+v"(hw[(ks) & 1][1]), "+v"(hr[(ks) & 1][0]), "+v"(hr[(ks) & 1][1]),   \
                   "+v"(hr[(ks) & 1][2]), "+v"(hr[(ks) & 1][3])                                                  \
                 : "n"(NOUT));                                                                                   \
    const i32x4_t fw = {hw[(ks) & 1][0][0], hw[(ks) & 1][0][1], hw[(ks) & 1][1][0], hw[(ks) & 1][1][1]};         \
    const i32x4_t f0 = {hr[(ks) & 1][0][0], hr[(ks) & 1][0][1], hr[(ks) & 1][1][0], hr[(ks) & 1][1][1]};         \
    const i32x4_t f1 = {hr[(ks) & 1][2][0], hr[(ks) & 1][2][1], hr[(ks) & 1][3][0], hr[(ks) & 1][3][1]};         \
    PQ_MFMA_BF16(acc[0], fw, f0);                                                                                \
    PQ_MFMA_BF16(acc[1], fw, f1);                                                                                \
  } while (0)
    PQ_SKT_READ(0);
    PQ_SKT_READ(1);
    PQ_SKT_MFMA(0, 6);
    PQ_SKT_READ(2);
    PQ_SKT_MFMA(1, 6);
    PQ_SKT_READ(3);
    PQ_SKT_MFMA(2, 6);
    PQ_SKT_MFMA(3, 0);
#undef PQ_SKT_READ
#undef PQ_SKT_MFMA
    st = st == NST - 1 ? 0 : st + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // lane l holds row l & 31 (a column of the wide operand), register v column 8 (v >> 2) + 4 (l >> 5) + (v & 3)
  const int m = m0 + wr0 + (lane & 31);
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = wc0 + j * 32 + 8 * g + 4 * h;
      if (p.trans) {                                  // uniform
#pragma unroll
        for (int e = 0; e < 4; ++e) p.slab[((size_t)split * SK_BN + n + e) * p.M + m] = acc[j][4 * g + e];
      } else {
        *reinterpret_cast<float4*>(p.slab + ((size_t)split * p.M + m) * SK_BN + n) =
            make_float4(acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]);
      }
    }
#endif
}

// Shapes, alignments and epilogues the kernel above takes: 128 columns, whole 64-element steps, a plain bf16 store,
// optionally with the dot product against a bf16 matrix of the output's shape.
bool pq_skinny_applies(int M, int N, int K, const pq_operand& A, const pq_operand& B, const pq_epilogue& e) {
  const bool btr = B.kind == PQ_SRC_KS16;
  const bool i8 = A.kind == PQ_SRC_KC8 && B.kind == PQ_SRC_KC8;
  const bool b16 = A.kind == PQ_SRC_KC16 && (B.kind == PQ_SRC_KC16 || btr);
  const long es = i8 ? 1 : 2;
  if (!(i8 || b16)) return false;
  if (!(M >= 1024 && N == SK_BN && K * es >= 128 && (K * es) % 128 == 0 && !A.kdiv && !B.kdiv && A.ld >= K && B.ld >= (btr ? N : K) &&
        (A.ld * es) % 16 == 0 && (B.ld * es) % 16 == 0 && ((uintptr_t)A.p % 16) == 0 && ((uintptr_t)B.p % 16) == 0))
    return false;
  if (!(e.out_kind == PQ_OUT_BF16 && e.ldc >= N && (e.ldc * 2) % 8 == 0 && ((uintptr_t)e.C % 8) == 0 && !e.sign_bytes && !e.maskW &&
        !e.accumulate && !e.dev_scale))
    return false;
  if (i8) return !e.dot_comp && !e.partials && (!e.col_div || ((uintptr_t)e.col_div % 16) == 0);   // de-quantising epilogue
  return !e.row_div && !e.col_div &&
         (!e.dot_comp || (e.comp_kind == PQ_OUT_BF16 && e.partials && e.ld_comp >= N && (e.ld_comp * 2) % 8 == 0 &&
                          ((uintptr_t)e.dot_comp % 8) == 0)) &&
         (e.dot_comp || !e.partials);
}

#ifndef PQ_SK_ROWS
#define PQ_SK_ROWS 32
#endif
int pq_skinny_blocks(int M) { return (M + PQ_SK_ROWS - 1) / PQ_SK_ROWS; }

int pq_launch_skinny(int M, int K, const pq_operand& A, const pq_operand& B, const pq_epilogue& e, hipStream_t s, int prof_label) {
  pq_prof_scope prof(prof_label, s);
  const dim3 grid(pq_skinny_blocks(M)), block(256);
  if (A.kind == PQ_SRC_KC8)
    skinny_gemm_kernel<false, PQ_SK_ROWS, true><<<grid, block, 0, s>>>(A.p, A.ld, B.p, B.ld, M, K, (uint16_t*)e.C, e.ldc, e.scale, nullptr, 0,
                                                                       nullptr, e.row_div, e.col_div);
  else if (B.kind == PQ_SRC_KS16)
    skinny_gemm_kernel<true, PQ_SK_ROWS, false><<<grid, block, 0, s>>>(A.p, A.ld, B.p, B.ld, M, K, (uint16_t*)e.C, e.ldc, e.scale,
                                                                       (const uint16_t*)e.dot_comp, e.ld_comp, e.partials, nullptr, nullptr);
  else
    skinny_gemm_kernel<false, PQ_SK_ROWS, false><<<grid, block, 0, s>>>(A.p, A.ld, B.p, B.ld, M, K, (uint16_t*)e.C, e.ldc, e.scale,
                                                                        (const uint16_t*)e.dot_comp, e.ld_comp, e.partials, nullptr, nullptr);
  PQ_CHECK_LAUNCH("skinny_gemm_kernel");
  return PQ_OK;
}

// Tile shape and contraction split for one GEMM.  A 256x256 tile (8 wavefronts, 128x64 each) when
// the output is large enough, else 128x128 (4 wavefronts); when the tiles alone cannot occupy the
// 256 compute units the contraction is split and reduced in a second, fixed-order pass.
pq_gemm_plan pq_plan_gemm(int engine, int M, int N, int K, bool int8, bool split_int8) {
  pq_gemm_plan pl;
  memset(&pl, 0, sizeof(pl));
  pl.splits = 1;
  if (engine == 1) {
    pl.bm = pl.bn = ref_tile(M, N);
    pl.kchunk = K;
    pl.red_blocks = ((M + pl.bm - 1) / pl.bm) * ((N + pl.bn - 1) / pl.bn);
    return pl;
  }
  const bool big = (M >= 256 && N >= 256);
  pl.bm = pl.bn = big ? 256 : 128;
  const long tiles = (long)((M + pl.bm - 1) / pl.bm) * ((N + pl.bn - 1) / pl.bn);
  pl.kchunk = K > 0 ? K : 1;
  if ((!int8 || split_int8) && tiles > 0 && tiles <= 128 && K >= 512) {
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


int pq_launch_gemm_pair_ks16(int K, int M0, int N0, const pq_operand& A0, const pq_operand& B0, float* C0, int ldc0, float scale0,
                             int M1, int N1, const pq_operand& A1, const pq_operand& B1, float* C1, int ldc1, float scale1,
                             hipStream_t s, int prof_label0, int prof_label1, void* splitk_ws0, void* splitk_ws1,
                             const pq_reduce_job* jobs, bool* jobs_done) {
  if (jobs_done) *jobs_done = false;
  pq_epilogue e0;
  memset(&e0, 0, sizeof(e0));
  e0.C = C0; e0.ldc = ldc0; e0.out_kind = PQ_OUT_F32; e0.scale = scale0;
  pq_epilogue e1 = e0;
  e1.C = C1; e1.ldc = ldc1; e1.scale = scale1;
  const pq_gemm_plan p0 = pq_plan_gemm(0, M0, N0, K), p1 = pq_plan_gemm(0, M1, N1, K);
  {
    // rank 128 over many tokens: the streaming pair kernel (problem 1 runs transposed).  Four token ranges when that
    // already gives a workgroup per CU (fewer slabs to write and add), up to sixteen for small matrices, never
    // shorter than 256 tokens
    auto al = [](const pq_operand& o) { return o.kind == PQ_SRC_KS16 && !o.kdiv && (o.ld * 2) % 16 == 0 && ((uintptr_t)o.p % 16) == 0; };
    int splits = 4;
    while (splits < 16 && (M0 / 64 + N1 / 64) * splits < 256 && K % (splits * 2 * 64) == 0 && K / (splits * 2) >= 256) splits *= 2;
    const size_t need0 = (size_t)splits * M0 * N0 * sizeof(float), need1 = (size_t)splits * M1 * N1 * sizeof(float);
    const bool tn = N0 == SK_BN && M1 == SK_BN && M0 >= 64 && N1 >= 64 && M0 % 64 == 0 && N1 % 64 == 0 && K >= 2048 &&
                    K % (splits * 64) == 0 && al(A0) && al(B0) && al(A1) && al(B1) && A0.ld >= M0 && B0.ld >= N0 && A1.ld >= M1 &&
                    B1.ld >= N1 && splitk_ws0 && splitk_ws1 && p0.ws_bytes >= need0 && p1.ws_bytes >= need1 &&
                    ((uintptr_t)splitk_ws0 % 16) == 0 && ((uintptr_t)splitk_ws1 % 16) == 0;
    if (tn) {
      skt_problem q0{(const uint16_t*)A0.p, A0.ld, (const uint16_t*)B0.p, B0.ld, M0, 0, (float*)splitk_ws0};
      skt_problem q1{(const uint16_t*)B1.p, B1.ld, (const uint16_t*)A1.p, A1.ld, N1, 1, (float*)splitk_ws1};
      {
        pq_prof_scope prof(prof_label0, s);
        const dim3 grid((M0 > N1 ? M0 : N1) / 64, splits, 2);
        skinny_tn_pair_kernel<<<grid, 256, 0, s>>>(q0, q1, K / splits);
        PQ_CHECK_LAUNCH("skinny_tn_pair_kernel");
      }
      pq_prof_scope prof(PQP_SPLITK_REDUCE, s);
      pq_reduce_job none;
      memset(&none, 0, sizeof(none));
      const int rb0 = (int)(((size_t)M0 * (N0 / 8) + 255) / 256), rb1 = (int)(((size_t)M1 * (N1 / 8) + 255) / 256);
      splitk_reduce_pair_kernel<<<rb0 + rb1 + (jobs ? 2 : 0), 256, 0, s>>>(splits, rb0, rb1, M0, N0, (const float*)splitk_ws0, e0, M1, N1,
                                                                          (const float*)splitk_ws1, e1, jobs ? jobs[0] : none,
                                                                          jobs ? jobs[1] : none);
      PQ_CHECK_LAUNCH("splitk_reduce_pair_kernel");
      if (jobs && jobs_done) *jobs_done = true;
      return PQ_OK;
    }
  }
  const int nbm0 = (M0 + 127) / 128, nbn0 = (N0 + 127) / 128, nbm1 = (M1 + 127) / 128, nbn1 = (N1 + 127) / 128;
  const bool same = M0 > 0 && N0 > 0 && M1 > 0 && N1 > 0 && K > 0 && p0.bm == 128 && p1.bm == 128 && p0.splits == p1.splits &&
                    p0.kchunk == p1.kchunk && nbm0 * nbn0 == nbm1 * nbn1 && A0.kind == PQ_SRC_KS16 && B0.kind == PQ_SRC_KS16 &&
                    A1.kind == PQ_SRC_KS16 && B1.kind == PQ_SRC_KS16 && (p0.splits == 1 || (splitk_ws0 && splitk_ws1));
  if (!same) {
    if (int rc = pq_launch_gemm(0, M0, N0, K, A0, B0, e0, s, prof_label0, splitk_ws0)) return rc;
    return pq_launch_gemm(0, M1, N1, K, A1, B1, e1, s, prof_label1, splitk_ws1);
  }
  pq_gemm_group grp;
  memset(&grp, 0, sizeof(grp));
  grp.mode = 3;
  grp.second.A = A1; grp.second.B = B1; grp.second.C = C1; grp.second.ldc = ldc1; grp.second.scale = scale1;
  grp.second.part = p0.splits > 1 ? (float*)splitk_ws1 : nullptr; grp.second.M = M1; grp.second.N = N1; grp.second.nbn = nbn1;
  pq_phase2 ph2;
  memset(&ph2, 0, sizeof(ph2));
  {
    pq_prof_scope prof(prof_label0, s);
    if (int rc = launch_mfma<128, 128, 2, 2, 128, false, false, PQ_SRC_KS16, PQ_SRC_KS16>(p0, M0, N0, K, A0, B0, e0, s, (float*)splitk_ws0, grp, ph2))
      return rc;
  }
  if (p0.splits > 1) {
    pq_prof_scope prof(PQP_SPLITK_REDUCE, s);
    pq_reduce_job none;
    memset(&none, 0, sizeof(none));
    const int extra = jobs ? 2 : 0;
    splitk_reduce_pair_kernel<<<p0.red_blocks + p1.red_blocks + extra, 256, 0, s>>>(
        p0.splits, p0.red_blocks, p1.red_blocks, M0, N0, (const float*)splitk_ws0, e0, M1, N1, (const float*)splitk_ws1, e1,
        jobs ? jobs[0] : none, jobs ? jobs[1] : none);
    PQ_CHECK_LAUNCH("splitk_reduce_pair_kernel");
    if (jobs && jobs_done) *jobs_done = true;
  }
  return PQ_OK;
}

// Grouped contraction ranges (per-expert weight gradients): with few output tiles per group and few groups the launch is
// far from a workgroup per CU, so every group's range is cut into up to 8 pieces whose slabs a second launch adds.
int pq_mode2_splits(int M, int N, int n_groups, int total_k) {
  if (M <= 0 || N <= 0 || n_groups <= 0) return 1;
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128) * n_groups;
  long want = 512 / tiles;
  const long by_len = (long)total_k / n_groups / 256;   // pieces of about 256 contraction indices or more
  if (want > by_len) want = by_len;
  if (want > 8) want = 8;
  return want > 1 ? (int)want : 1;
}
size_t pq_mode2_ws_bytes(int M, int N, int n_groups, int total_k) {
  const int sp = pq_mode2_splits(M, N, n_groups, total_k);
  return sp > 1 ? (size_t)sp * n_groups * M * N * sizeof(float) : 0;
}

int pq_launch_gemm(int engine, int M, int N, int K, const pq_operand& A, const pq_operand& B,
                   const pq_epilogue& epi, hipStream_t s, int prof_label, void* splitk_ws,
                   const pq_gemm_group* group, const pq_phase2* phase2) {
  if (M <= 0 || N <= 0) return PQ_OK;
  pq_gemm_group grp;
  memset(&grp, 0, sizeof(grp));
  if (group) grp = *group;
  pq_phase2 ph2;
  memset(&ph2, 0, sizeof(ph2));
  if (phase2) ph2 = *phase2;
  if (ph2.K2 > 0 && (engine == 1 || grp.mode)) return pq_set_error(PQ_ERR_BAD_ARG, "a fused second contraction needs the plain MFMA engine");
  if ((epi.n_limit > 0 || epi.m_limit > 0) && (epi.accumulate || epi.maskW || epi.dot_comp || epi.n_limit % 4 != 0))
    return pq_set_error(PQ_ERR_BAD_ARG, "store limits go with plain stores and a column limit that is a multiple of 4");
  if (grp.mode && engine == 1) return pq_set_error(PQ_ERR_DTYPE, "grouped GEMMs run on the MFMA engine only (bf16 I/O)");
  // plain rank-128 products over many rows: the streaming kernel (callers that want per-block partial sums or the
  // slabs of a split contraction choose it themselves, since it changes how many of those there are)
  if (engine == 0 && !grp.mode && ph2.K2 == 0 && !epi.partials && !epi.defer_reduce && pq_skinny_applies(M, N, K, A, B, epi))
    return pq_launch_skinny(M, K, A, B, epi, s, prof_label);
  if (engine == 1) {
    pq_prof_scope prof(prof_label, s);
    const int tile = ref_tile(M, N);
    dim3 grid((N + tile - 1) / tile, (M + tile - 1) / tile), block(256);
    if (tile == 64) ref_gemm_kernel<64><<<grid, block, 0, s>>>(M, N, K, A, B, epi);
    else ref_gemm_kernel<128><<<grid, block, 0, s>>>(M, N, K, A, B, epi);
    PQ_CHECK_LAUNCH("ref_gemm_kernel");
    return PQ_OK;
  }
  const int ak = A.kind, bk = B.kind;
  const bool int8 = (ak == PQ_SRC_KC8);
  pq_gemm_plan pl = pq_plan_gemm(0, M, N, K, int8, epi.split_int8 != 0);
  if (grp.mode) {
    pl.splits = 1;
    pl.kchunk = K > 0 ? K : 1;
    pl.bm = pl.bn = 128;
    // wide row groups (experts of several hundred hidden units, Table 1: r = 384): the 256x256 streaming instantiation,
    // whose loaders clamp a group's last rows like any ragged edge
    if (grp.mode == 1 && N >= 256 && grp.max_rows >= 256 && K % 64 == 0) pl.bm = pl.bn = 256;
    // contraction ranges with a plain fp32 output whose groups lie one behind the other: cut the ranges (see above)
    if (grp.mode == 2 && splitk_ws && epi.out_kind == PQ_OUT_F32 && epi.ldc == N && grp.c_stride == (long)M * N && N % 8 == 0 &&
        !epi.partials && !epi.dot_comp && !epi.sign_bytes && !epi.maskW && !epi.accumulate && !epi.row_div && !epi.col_div &&
        epi.m_limit == 0 && epi.n_limit == 0) {
      const int sp = pq_mode2_splits(M, N, grp.n_groups, K);
      if (sp > 1) {
        pl.splits = sp;
        pl.red_blocks = (int)(((size_t)grp.n_groups * M * (N / 8) + 255) / 256);
        pl.ws_bytes = pq_mode2_ws_bytes(M, N, grp.n_groups, K);
      }
    }
    // row groups with a narrow output and a long contraction (expert up/gate projections, their input
    // gradients): too few tiles to fill the chip, so the contraction is split as for plain GEMMs
    // (a per-group column divisor is applied in the GEMM's own epilogue only: such products are not split)
    // (likewise experts of several hundred hidden units on the 256x256 tiles: Table 1's r = 384 gives 99 tiles at 8192 slots)
    const bool wide_few = pl.bm == 256 && (long)((grp.max_rows + 255) / 256 + grp.n_groups) * ((N + 255) / 256) <= 128 && K % 512 == 0 &&
                          epi.out_kind == PQ_OUT_BF16 && !epi.accumulate && !epi.row_div;
    if (grp.mode == 1 && (N <= 128 || wide_few) && K >= 1024 && splitk_ws && !(epi.col_div && grp.coldiv_stride)) {
      const long tiles = wide_few ? (long)((grp.max_rows + 255) / 256 + grp.n_groups) * ((N + 255) / 256)
                                  : (long)((grp.max_rows + 127) / 128 + grp.n_groups) * ((N + 127) / 128);
      long want = tiles > 0 ? 256 / tiles : 1;
      if (want > 8) want = 8;
      if (want > 1) {
        long chunk = (K + want - 1) / want;
        chunk = (chunk + 255) / 256 * 256;
        pl.kchunk = (int)chunk;
        pl.splits = (int)((K + chunk - 1) / chunk);
        pl.red_blocks = (int)(((size_t)M * (N / 8) + 255) / 256);
        pl.ws_bytes = (size_t)pl.splits * M * N * sizeof(float);
      }
    }
  }
  if (pl.splits > 1 && !splitk_ws) return pq_set_error(PQ_ERR_WORKSPACE, "split contraction needs scratch");
  float* part = (float*)splitk_ws;
  int rc;
  {
    pq_prof_scope prof(prof_label, s);   // the MFMA kernel alone; a split's reduction is timed under its own label
    if (ph2.K2 > 0) {
      if (pl.splits > 1) return pq_set_error(PQ_ERR_BAD_ARG, "a fused second contraction cannot be combined with a split contraction");
      if (ak == PQ_SRC_KC8 && bk == PQ_SRC_BITS8 && ph2.A2.kind == PQ_SRC_KC16 && ph2.B2.kind == PQ_SRC_KC16)
        return launch_mfma_cfg<true, PQ_SRC_KC8, PQ_SRC_BITS8, PQ_SRC_KC16, PQ_SRC_KC16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
      if (ak == PQ_SRC_KC16 && bk == PQ_SRC_BITS16 && ph2.A2.kind == PQ_SRC_KC16 && ph2.B2.kind == PQ_SRC_KS16)
        return launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_BITS16, PQ_SRC_KC16, PQ_SRC_KS16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
      return pq_set_error(PQ_ERR_BAD_ARG, "no fused MFMA kernel for these operand kinds");
    }
    if (ak == PQ_SRC_KC8 && bk == PQ_SRC_BITS8) rc = launch_mfma_cfg<true, PQ_SRC_KC8, PQ_SRC_BITS8>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else if (ak == PQ_SRC_KC8 && bk == PQ_SRC_KC8) rc = launch_mfma_cfg<true, PQ_SRC_KC8, PQ_SRC_KC8>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_KC16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_KC16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_KS16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_KS16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else if (ak == PQ_SRC_KC16 && bk == PQ_SRC_BITS16) rc = launch_mfma_cfg<false, PQ_SRC_KC16, PQ_SRC_BITS16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else if (ak == PQ_SRC_KS16 && bk == PQ_SRC_KS16) rc = launch_mfma_cfg<false, PQ_SRC_KS16, PQ_SRC_KS16>(pl, M, N, K, A, B, epi, s, part, grp, ph2);
    else return pq_set_error(PQ_ERR_BAD_ARG, "no MFMA kernel for operand kinds (%d, %d)", ak, bk);
  }
  if (rc != PQ_OK) return rc;
  if (pl.splits > 1 && !epi.defer_reduce) {
    pq_prof_scope prof(PQP_SPLITK_REDUCE, s);
    const int Mred = grp.mode == 2 ? grp.n_groups * M : M;   // grouped ranges: the groups' outputs as one matrix
    if (int8) splitk_reduce_kernel<true><<<pl.red_blocks, 256, 0, s>>>(Mred, N, pl.splits, part, epi);
    else splitk_reduce_kernel<false><<<pl.red_blocks, 256, 0, s>>>(Mred, N, pl.splits, part, epi);
    PQ_CHECK_LAUNCH("splitk_reduce_kernel");
  }
  return PQ_OK;
}
