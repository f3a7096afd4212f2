// Shared declarations of libsk's HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sk {

constexpr int NUM_CUS = 256;  // compute units of an MI355X

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// How a GEMM result tile leaves the kernel.
enum Epilogue : int {
  EPI_STORE = 0,    // C = scale * acc (+ bias[n]), rounded to the storage type
  EPI_PARTIAL = 1,  // split-K: raw fp32 partial sums, one [M, N] slab per split
};

// C[M, N] = A . B over k in [0, K), optionally split over blockIdx-derived k ranges.
//   a_kc: A is stored [M, K] (k contiguous); otherwise [K, M] (m contiguous)
//   b_kc: B is stored [N, K] (k contiguous); otherwise [K, N] (n contiguous)
// lda/ldb/ldc are row strides in elements of the stored arrays.
struct GemmArgs {
  const void* A;
  const void* B;
  void* C;             // storage type (EPI_STORE) or fp32 partial slabs (EPI_PARTIAL)
  const void* bias;    // [N] storage type, or null (EPI_STORE only)
  float* colsum;       // [splits, N] fp32 sums of B over k, or null (EPI_PARTIAL only)
  int64_t lda, ldb, ldc;
  int M, N, K;
  int n_store;         // columns written per row: N, or up to ldc to zero-fill row padding
                       // (columns >= N of the product are exact zeros); 0 means N
  int k_per_split;     // multiple of the kernel's k chunk; K when not split
  int splits;
  int tiles_m, tiles_n;
  float scale;
};

// Column sums of a dense row-major bf16 matrix [rows, cols]: out[run][c] = sum of the rows
// of run `run` (rows_per_split rows each), for col_groups groups of 512 columns.
struct ColsumArgs {
  const void* in;
  float* out;
  int rows, cols, rows_per_split, col_groups;
};

// Sum of split-K slabs in split order (deterministic), two outputs in one launch:
//   out[i]  = scale  * sum_s part[s][i]   for i < n      (slabs n elements apart)
//   out2[j] = scale2 * sum_s part2[s][j]  for j < n2     (splits2 slabs n2 elements apart; n2 may be 0)
struct ReduceArgs {
  const float* part;
  float* out;
  int64_t n;
  const float* part2;
  float* out2;
  int64_t n2;
  int splits, splits2;
  float scale, scale2;
};

// One segment of a split reduction, the part that falls to work-group `block` of `nblocks`
// (256 threads each): 16-byte pieces are dealt round-robin, U per thread and pass so that
// their loads overlap; every piece sums its slabs in index order.  Every load is
// unconditional -- a piece past the end re-reads the thread's first piece and is not
// written -- so a pass issues all of its loads before it waits for any (under a per-piece
// bounds branch the compiler waited for each load by itself).
template <int U>
__device__ __forceinline__ void reduce_segment_pass(const float* __restrict__ part, float* __restrict__ out,
                                                    int64_t n, int splits, float scale, int block,
                                                    int nblocks, int tid) {
  const int64_t pieces = n / 4, stride = (int64_t)nblocks * 256;
  for (int64_t q0 = (int64_t)block * 256 + tid; q0 < pieces; q0 += stride * U) {
    const float* src[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      src[u] = part + (q < pieces ? q : q0) * 4;
    }
    float4 s[U];
#pragma unroll
    for (int u = 0; u < U; ++u) s[u] = *reinterpret_cast<const float4*>(src[u]);
#pragma unroll 8
    for (int k = 1; k < splits; ++k) {
      float4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const float4*>(src[u] + (int64_t)k * n);
#pragma unroll
      for (int u = 0; u < U; ++u) { s[u].x += v[u].x; s[u].y += v[u].y; s[u].z += v[u].z; s[u].w += v[u].w; }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      if (q < pieces)
        *reinterpret_cast<float4*>(out + q * 4) =
            make_float4(s[u].x * scale, s[u].y * scale, s[u].z * scale, s[u].w * scale);
    }
  }
}

__device__ __forceinline__ void reduce_segment_part(const float* __restrict__ part, float* __restrict__ out,
                                                    int64_t n, int splits, float scale, int block,
                                                    int nblocks, int tid) {
  // one piece per thread at most: no point in asking for four
  if (n / 4 <= (int64_t)nblocks * 256) reduce_segment_pass<1>(part, out, n, splits, scale, block, nblocks, tid);
  else reduce_segment_pass<4>(part, out, n, splits, scale, block, nblocks, tid);
}

// Both segments of a split reduction (see ReduceArgs), this work-group's part.
__device__ __forceinline__ void reduce_splits_part(const ReduceArgs& p, int block, int nblocks, int tid) {
  if (p.n > 0) reduce_segment_part(p.part, p.out, p.n, p.splits, p.scale, block, nblocks, tid);
  if (p.n2 > 0) reduce_segment_part(p.part2, p.out2, p.n2, p.splits2, p.scale2, block, nblocks, tid);
}

// XCD-aware work-group order.  Work-groups are handed to the 8 XCDs round-robin,
// so consecutive hardware ids land on different L2s.  Remap so that each XCD
// gets one contiguous run of logical tile ids (neighbouring tiles share operand
// panels in that XCD's L2).
__device__ __forceinline__ int xcd_remap(int hw_id, int total) {
  const int per = total >> 3;
  if (hw_id >= (per << 3)) return hw_id;
  return (hw_id & 7) * per + (hw_id >> 3);
}

// Logical tile id -> (tile_m, tile_n): bands of 8 tile rows, walked row-first
// inside a band, so a run of ids covers a compact block of the output.
__device__ __forceinline__ void tile_coords(int id, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int GM = 8;
  const int band_sz = GM * tiles_n;
  const int band = id / band_sz;
  const int first_m = band * GM;
  const int rows = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_band = id - band * band_sz;
  tm = first_m + in_band % rows;
  tn = in_band / rows;
}

}  // namespace sk
