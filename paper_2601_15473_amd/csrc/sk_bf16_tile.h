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

// A window onto a dense row-major global array, as a raw buffer resource: loads
// through it take a 32-bit byte offset from the window's origin and return zero
// for any offset at or past the end of the array, so ragged edges need no branch
// (a lane that must read zero for another reason is pointed past the end).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned OOB_OFFSET = 0x80000000u;

struct GWindow {
  __amdgpu_buffer_rsrc_t rsrc;
};

// Window starting `origin` elements into an array of `total` elements of `esize` bytes.
__device__ __forceinline__ GWindow make_window(const void* base, int64_t origin, int64_t total,
                                               int esize) {
  int64_t bytes = (total - origin) * esize;
  if (bytes < 0) bytes = 0;
  if (bytes > 0x7fffffff) bytes = 0x7fffffff;
  GWindow w;
  w.rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(static_cast<const char*>(base)) + origin * esize, 0, (int)bytes, 0x00020000);
  return w;
}

__device__ __forceinline__ uint4 window_load16(const GWindow& w, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(w.rsrc, (int)byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte store through a window: dropped when the offset is at or past the window's end.
__device__ __forceinline__ void window_store16(const GWindow& w, unsigned byte_off, const uint4& v) {
  const u32x4 d = {v.x, v.y, v.z, v.w};
  __builtin_amdgcn_raw_buffer_store_b128(d, w.rsrc, (int)byte_off, 0, 0);
}

// One operand tile of EXT rows (m or n extent) by KX (k extent, default BK) in LDS,
// moved by a work-group of NTH threads.
//   KC  = true : source is [EXT, K] with k contiguous; stored [EXT][KX] without padding,
//                the 16-byte pieces of each row XOR-swizzled by the row number
//                (kc_piece): a store instruction then fills whole 256-byte bank rows
//                and the 16 rows a fragment read touches per pass land in 16 different
//                bank groups -- both conflict free.
//   KC  = false: source is [K, EXT] with m/n contiguous; stored [KX][EXT + 32] and
//                read through the LDS transpose read (ds_read_b64_tr_b16).  The row
//                stride is 16 dwords modulo 32, so the four k rows a 16-lane group
//                reads sit in disjoint banks.
// Physical position of logical 16-byte piece `pc` of row `row` in a k-contiguous tile
// whose rows hold KX elements (KX / 8 pieces, a power of two up to 32).  Rows that
// share a 256-byte bank row get different XOR keys, as do the 16 consecutive rows of
// one fragment-read pass.
template <int KX>
__device__ __forceinline__ int kc_piece(int row, int pc) {
  constexpr int PPR = KX / 8;
  constexpr int ROWS_PER_BANKROW = PPR >= 16 ? 1 : 16 / PPR;
  return pc ^ ((row / ROWS_PER_BANKROW) & (PPR - 1));
}

// Compile-time loop: f(IntC<I>{}) for I = BEGIN .. END - 1.
template <int V>
struct IntC {
  static constexpr int value = V;
};
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(IntC<BEGIN>{});
    static_for<BEGIN + 1, END>(f);
  }
}

// One scheduling phase: NM MFMAs with ND LDS reads, NV global loads and NW LDS stores
// spread evenly between them, then a fence for the scheduler.
template <int NM, int ND, int NV, int NW, int I = 0>
__device__ __forceinline__ void sched_phase() {
  if constexpr (I < NM) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    constexpr int d = (I + 1) * ND / NM - I * ND / NM;
    constexpr int v = (I + 1) * NV / NM - I * NV / NM;
    constexpr int w = (I + 1) * NW / NM - I * NW / NM;
    if constexpr (d > 0) __builtin_amdgcn_sched_group_barrier(0x100, d, 0);
    if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
    if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
    sched_phase<NM, ND, NV, NW, I + 1>();
  } else {
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int EXT, bool KC, int KX = BK, int NTH = 256>
struct OpTile {
  static constexpr int LD = KC ? KX : EXT + 32;
  static constexpr int ELEMS = KC ? EXT * KX : KX * (EXT + 32);
  static constexpr int PIECES = EXT * KX / (8 * NTH);  // 16-byte pieces per thread (NTH threads)
  static_assert(EXT * KX % (8 * NTH) == 0, "tile must split evenly over the work-group");

  // Global -> registers, branch free.  `g` is the whole array ([ext_total, k_total]
  // for KC, [k_total, ext_total] otherwise, row stride ld).  The tile starts at
  // row/col ext0 and k0; k is clipped at k_end and ext at ext_total; everything
  // outside reads as zero.  Extents along a contiguous dimension are multiples of
  // 8, so a 16-byte piece is wholly inside or wholly outside.
  // (P0, P1 select a run of the thread's pieces, for callers that spread a tile's loads
  // over several scheduling phases.)
  template <int P0 = 0, int P1 = PIECES>
  static __device__ __forceinline__ void load(uint4 (&r)[PIECES], const bf16* __restrict__ g,
                                              int64_t ld, int ext0, int ext_total, int k0,
                                              int k_end, int k_total, int tid) {
    const int64_t rows = KC ? ext_total : k_total;
    const int64_t origin = KC ? (int64_t)ext0 * ld + k0 : (int64_t)k0 * ld + ext0;
    const GWindow w = make_window(g, origin, rows * ld, 2);
    const unsigned ldb = (unsigned)ld * 2u;
#pragma unroll
    for (int p = P0; p < P1; ++p) {
      const int piece = p * NTH + tid;
      constexpr int PPR = KC ? KX / 8 : EXT / 8;
      const int row = piece / PPR, col = (piece % PPR) * 8;
      // rows past the end of the array fall outside the window by themselves
      const bool ok = KC ? (k0 + col < k_end) : (ext0 + col < ext_total && k0 + row < k_end);
      const unsigned off = (unsigned)row * ldb + (unsigned)col * 2u;
      r[p] = window_load16(w, ok ? off : OOB_OFFSET);
    }
  }

  // Registers -> LDS tile (pieces P0 .. P1 - 1 of the thread).
  template <int P0 = 0, int P1 = PIECES>
  static __device__ __forceinline__ void store(bf16* tile, const uint4 (&r)[PIECES], int tid) {
#pragma unroll
    for (int p = P0; p < P1; ++p) {
      const int piece = p * NTH + tid;
      constexpr int PPR = KC ? KX / 8 : EXT / 8;
      const int row = piece / PPR;
      const int pc = KC ? kc_piece<KX>(row, piece % PPR) : piece % PPR;
      *reinterpret_cast<uint4*>(tile + row * LD + pc * 8) = r[p];
    }
  }
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// MFMA operand fragment for the 32 rows/cols starting at `e0`, k step `ks`
// (16 k values) of an LDS tile with row stride LD.
template <bool KC, int LD>
__device__ __forceinline__ bf16x8 read_frag(const bf16* tile, int e0, int ks, int lane) {
  if (KC) {
    const int row = e0 + (lane & 31);
    return *reinterpret_cast<const bf16x8*>(tile + row * LD + kc_piece<LD>(row, ks * 2 + (lane >> 5)) * 8);
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

// Fragment of a plain row-major [rows][LD] bf16 tile (k contiguous, rows padded by the
// caller so that LD / 2 is 4 modulo 8 dwords): 16 bytes per lane, no swizzle.
template <int LD>
__device__ __forceinline__ bf16x8 read_frag_rowmajor(const bf16* tile, int e0, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + (e0 + (lane & 31)) * LD + ks * 16 + (lane >> 5) * 8);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  // round to nearest even, both halves in one v_cvt_pk_bf16_f32
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}

}  // namespace sk
