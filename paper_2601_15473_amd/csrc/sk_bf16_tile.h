// Building blocks of the bf16 MFMA kernels: operand tiles in LDS, fragment
// reads in the v_mfma_f32_32x32x16_bf16 lane layout, and the tile epilogue.
//
// Lane layout of v_mfma_f32_32x32x16_bf16 (D = P . Q, P 32x16, Q 16x32), lane l:
//   P fragment: row  l % 32, k = 8 * (l / 32) + 0..7      (8 bf16 = 16 bytes)
//   Q fragment: col  l % 32, k = 8 * (l / 32) + 0..7
//   D: col l % 32, rows 8 * (r / 4) + 4 * (l / 32) + r % 4 for r = 0..15
// Both operand fragments have the same shape, so the kernels pass the B-side
// fragment as P and the A-side fragment as Q: each lane then owns one output
// row (m = l % 32) and, per r / 4, four consecutive output columns -- which
// packs into 8-byte (bf16) or 16-byte (fp32) pieces for the epilogue.
#pragma once
#include "sk_common.h"

namespace sk {

constexpr int BK = 64;           // k extent of one LDS chunk
constexpr int KC_LD = BK + 8;    // LDS row stride (elements) of a k-contiguous tile:
                                 // 144 bytes, so 16 consecutive rows start 4 banks apart
                                 // modulo 64 and a 16-byte-per-lane read is conflict free

// One operand tile of EXT rows (m or n extent) by BK in LDS.
//   KC  = true : source is [EXT, K] with k contiguous; stored [EXT][KC_LD].
//   KC  = false: source is [K, EXT] with m/n contiguous; stored [BK][EXT + 32] and
//                read through the LDS transpose read (ds_read_b64_tr_b16).  The row
//                stride is 16 dwords modulo 32, so the four k rows a 16-lane group
//                reads sit in disjoint banks.
template <int EXT, bool KC>
struct OpTile {
  static constexpr int LD = KC ? KC_LD : EXT + 32;
  static constexpr int ELEMS = KC ? EXT * KC_LD : BK * (EXT + 32);
  static constexpr int PIECES = EXT / 32;  // 16-byte pieces per thread per chunk (256 threads)

  // Global -> registers.  `ext0` is the tile's first row/col, `ext_total` the
  // array's extent in that dimension; k in [k0, k0 + BK) is clipped at k_end.
  // Everything outside is read as zero.  Extents along a contiguous dimension
  // are multiples of 8, so a 16-byte piece is wholly inside or wholly outside.
  static __device__ __forceinline__ void load(uint4 (&r)[PIECES], const bf16* __restrict__ g,
                                              int64_t ld, int ext0, int ext_total, int k0,
                                              int k_end, int tid) {
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (KC) {
        const int e = ext0 + p * 32 + (tid >> 3);
        const int kk = k0 + (tid & 7) * 8;
        if (e < ext_total && kk < k_end) v = *reinterpret_cast<const uint4*>(g + (int64_t)e * ld + kk);
      } else {
        constexpr int PPR = EXT / 8;
        const int piece = p * 256 + tid;
        const int kk = k0 + piece / PPR;
        const int e = ext0 + (piece % PPR) * 8;
        if (e < ext_total && kk < k_end) v = *reinterpret_cast<const uint4*>(g + (int64_t)kk * ld + e);
      }
      r[p] = v;
    }
  }

  // Registers -> LDS tile.
  static __device__ __forceinline__ void store(bf16* tile, const uint4 (&r)[PIECES], int tid) {
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
      if (KC) {
        *reinterpret_cast<uint4*>(tile + (p * 32 + (tid >> 3)) * LD + (tid & 7) * 8) = r[p];
      } else {
        constexpr int PPR = EXT / 8;
        const int piece = p * 256 + tid;
        *reinterpret_cast<uint4*>(tile + (piece / PPR) * LD + (piece % PPR) * 8) = r[p];
      }
    }
  }
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// MFMA operand fragment for the 32 rows/cols starting at `e0`, k step `ks`
// (16 k values) of an LDS tile with row stride LD.
template <bool KC, int LD>
__device__ __forceinline__ bf16x8 read_frag(const bf16* tile, int e0, int ks, int lane) {
  if (KC) {
    return *reinterpret_cast<const bf16x8*>(tile + (e0 + (lane & 31)) * LD + ks * 16 + (lane >> 5) * 8);
  } else {
    // ds_read_b64_tr_b16, per group of 16 lanes: lane i receives, as element e,
    // element (i % 4) of what lane 4 e + i / 4 of the group addressed.  With lane j
    // addressing k row j / 4 and columns 4 (j % 4) .. +3, lane i ends up with column i
    // of k rows 0..3: four k-consecutive values of one column, as the MFMA wants.
    const int krow = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int col = e0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
    const bf16* p = tile + krow * LD + col;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LD));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  // round to nearest even; inputs are finite sums
  const bf16 a = (bf16)lo, b = (bf16)hi;
  return (uint32_t)__builtin_bit_cast(unsigned short, a) |
         ((uint32_t)__builtin_bit_cast(unsigned short, b) << 16);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}

}  // namespace sk
