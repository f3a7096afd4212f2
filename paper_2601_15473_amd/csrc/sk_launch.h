// Host-side launchers of libsk's kernels (internal; the public ABI is include/sk.h).
#pragma once
#include "sk_common.h"

namespace sk {

enum GemmKind : int {
  GEMM_NN = 0,      // A [M,K], B [K,N]            -> storage type
  GEMM_NT = 1,      // A [M,K], B [N,K]            -> storage type
  GEMM_TN_F32 = 2,  // A [K,M], B [K,N], split-K   -> fp32 (+ column sums of B)
  GEMM_NN_F32 = 3,  // as GEMM_NN, split-K          -> fp32 slabs
  GEMM_NT_F32 = 4,  // as GEMM_NT, split-K          -> fp32 slabs
  GEMM_TT = 5,      // A [K,M], B [N,K]            -> storage type
  GEMM_NN_F32_COLSUM = 6,  // as GEMM_NN_F32, plus the column sums of B
  GEMM_TN_F32_PLAIN = 7,   // as GEMM_TN_F32 without the column sums (any tile)
  GEMM_TT_F32 = 8,         // as GEMM_TT, split-K          -> fp32 slabs
};

enum TileCfg : int {
  TILE_256x256 = 0,
  TILE_128x128 = 1,
  TILE_128x64 = 2,
  TILE_64x128 = 3,
  TILE_64x64 = 4,
  TILE_256x128 = 5,
  TILE_128x256 = 6,
  TILE_256x256_W8 = 7,   // 256 x 256 with eight waves (2 x 4), two per SIMD
  TILE_COUNT = 8,
};

inline void tile_dims(int tile, int& bm, int& bn) {
  static const int dims[TILE_COUNT][2] = {{256, 256}, {128, 128}, {128, 64}, {64, 128},
                                          {64, 64},   {256, 128}, {128, 256}, {256, 256}};
  bm = dims[tile][0];
  bn = dims[tile][1];
}

// bf16 operands, fp32 accumulation (MFMA).  `tiles_m/tiles_n` of `a` are filled in here.
hipError_t launch_gemm_bf16(GemmKind kind, int tile, const GemmArgs& a, hipStream_t s);
// fp32 operands and accumulation (MFMA), one tile shape.
hipError_t launch_gemm_f32(GemmKind kind, const GemmArgs& a, hipStream_t s);
constexpr int F32_BM = 64, F32_BN = 64, F32_BK = 16;

hipError_t launch_reduce_splits(const ReduceArgs& a, hipStream_t s);
// out[i] = bf16(sum over s of part[s][i]), i < n (n a multiple of 4; slabs n elements apart,
// summed in index order)
hipError_t launch_reduce_to_bf16(const float* part, void* out, int64_t n, int splits, hipStream_t s);
// out[r * ld_out + c] = scale * sum over s of part[s][r * cols + c] (r < rows, c < cols, cols a multiple of 4;
// slabs rows * cols elements apart, summed in index order): a column range of a wider matrix
hipError_t launch_reduce_splits_2d(const float* part, float* out, int rows, int cols, int64_t ld_out,
                                   int splits, float scale, hipStream_t s);
// Two GEMMs that do not depend on each other in one launch (see dual_gemm_kernel); built
// for a few (kind, tile) pairs only -- ask dual_gemm_supported first.  `a` should be the
// longer-running one.
bool dual_gemm_supported(GemmKind kind_a, int tile_a, GemmKind kind_b, int tile_b);
hipError_t launch_dual_gemm_bf16(GemmKind kind_a, int tile_a, GemmArgs a, GemmKind kind_b, int tile_b,
                                 GemmArgs b, hipStream_t s);
// fp32 column sums of the dense row-major bf16 matrix in [rows, cols], one output row of
// `cols` sums per run of rows_per_split rows (splits runs)
hipError_t launch_colsum_bf16(const void* in, float* out, int rows, int cols, int splits,
                              int rows_per_split, hipStream_t s);
// The split-K GEMM_NN_F32 `a` on the eight-wave 256 x 256 tile with the column sums above
// computed in the same launch, on the CUs the GEMM's work-groups leave free.
hipError_t launch_gemm_f32slabs_with_colsum(int tile, GemmArgs a, const void* in, float* out, int rows,
                                            int cols, int splits, int rows_per_split, hipStream_t s);

// Second contraction of the layer with the R-wide intermediate of a 64-token tile
// resident on chip (bf16, R <= 512), optionally with the first contraction fused in:
//   C[M, N] = scale * Zt . B2 (+ bias)
//   fused    : Zt = bf16(A[M, K1] . B1)                       (R <= 256)
//   not fused: Zt read from Z: bf16 [M, R] when z_splits == 0, else the sum of
//              z_splits fp32 slabs [M, R] that are z_slab elements apart
//   b_kc = false: B1 [K1, R], B2 [R, N]   (forward:      x, S_cat, U_cat)
//   b_kc = true : B1 [R, K1], B2 [N, R]   (input grad:   dY, U_cat, S_cat)
struct ChainArgs {
  const void* A;       // [M, K1]      (fused)
  const void* B1;      //              (fused)
  const void* Z;       //              (not fused)
  const void* B2;
  const void* bias;    // [N] or null
  void* C;             // [M, N]
  int64_t lda, ldb1, ldb2, ldc, z_slab;
  int M, K1, R, N;
  int z_splits;
  int n_slices;        // the N range is cut into this many runs of tiles, one per work-group
  int bm;              // rows of a token tile: 64 (0 means 64), or 128 for R <= 128
  int tiles_m;         // filled in by the launcher
  float scale;
  // An unrelated split reduction that this launch carries along (narrow-sketch kernels
  // only; tail.n + tail.n2 == 0 for none): its pieces are dealt over the work-groups,
  // which saves the reduction a launch of its own.
  ReduceArgs tail;
};
bool chain_supported(int R);
constexpr int CHAIN_FUSED_MAX_R = 256;
int chain_bn(int R);   // width of the N tiles the chain kernels walk
hipError_t launch_chain_bf16(bool b_kc, bool fused, ChainArgs a, hipStream_t s);

}  // namespace sk
