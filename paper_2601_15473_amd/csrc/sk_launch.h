// Host-side launchers of libsk's kernels (internal; the public ABI is include/sk.h).
#pragma once
#include <string>
#include <type_traits>

#include "sk_common.h"

namespace sk {

// ---------------------------------------------------------------------------
// Launch plumbing: every kernel of the library goes out through launch_kernel, which
// reports the launch's own status (not a stale error some earlier HIP call of the process
// left behind) and serves the two testing aids of include/sk_debug.h -- the host-only
// launch trace and the per-kernel event timing.
// ---------------------------------------------------------------------------
struct LaunchHooks {
  virtual ~LaunchHooks() {}
  // trace mode: returns true when launches are to be recorded instead of made
  virtual bool tracing() const = 0;
  virtual void access(const void* p, uint64_t bytes, bool write) = 0;   // of the launch that follows
  virtual void launch_recorded() = 0;
  // profile mode: events around the launch
  virtual void before(const char* name, unsigned groups, double flops, double bytes, hipStream_t s) = 0;
  virtual void after(hipStream_t s) = 0;
};
LaunchHooks* launch_hooks();   // the calling thread's, or null (the normal case)

inline bool tracing() {
  LaunchHooks* h = launch_hooks();
  return h != nullptr && h->tracing();
}
// Byte range a kernel about to be launched reads or writes: a dense or strided matrix of
// `rows` rows of `cols` elements, rows `ld` elements apart (from the first byte of the
// first row to the last byte of the last row).  Recorded in trace mode only.
inline void note_matrix(const void* p, int64_t rows, int64_t cols, int64_t ld, int esize, bool write) {
  LaunchHooks* h = launch_hooks();
  if (h == nullptr || !h->tracing() || p == nullptr || rows <= 0 || cols <= 0) return;
  h->access(p, (uint64_t)(((rows - 1) * ld + cols) * esize), write);
}

// What a launch is worth to the method, for the per-kernel timing: the flops of the products
// it forms and the bytes it must move (each operand read once, each result written once --
// re-reads across tiles and cache traffic are not counted).
struct Work {
  double flops, bytes;
};

template <typename... KArgs>
inline hipError_t launch_kernel(const char* name, Work work, void (*kernel)(KArgs...), dim3 grid, dim3 block,
                                hipStream_t s, typename std::common_type<KArgs>::type... args) {
  LaunchHooks* h = launch_hooks();
  if (h != nullptr && h->tracing()) {
    h->launch_recorded();
    return hipSuccess;
  }
  if (h != nullptr) h->before(name, grid.x * grid.y * grid.z, work.flops, work.bytes, s);
  void* ptrs[] = {const_cast<void*>(static_cast<const void*>(&args))...};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, s);
  if (h != nullptr) h->after(s);
  return e;
}

// "kernel<256, 256, 2, 4, true, false, bf16, false, 1>": a template instance's name as a
// profiler prints it.
inline std::string kernel_label(const char* base, std::initializer_list<std::string> params) {
  std::string n = base;
  n += "<";
  bool first = true;
  for (const std::string& q : params) {
    if (!first) n += ", ";
    n += q;
    first = false;
  }
  return n + ">";
}
inline std::string lbl(int v) { return std::to_string(v); }
inline std::string lbl(bool v) { return v ? "true" : "false"; }

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

inline void gemm_kind_traits(GemmKind kind, bool& a_kc, bool& b_kc, bool& out_f32) {
  a_kc = !(kind == GEMM_TN_F32 || kind == GEMM_TN_F32_PLAIN || kind == GEMM_TT || kind == GEMM_TT_F32);
  b_kc = kind == GEMM_NT || kind == GEMM_NT_F32 || kind == GEMM_TT || kind == GEMM_TT_F32;
  out_f32 = !(kind == GEMM_NN || kind == GEMM_NT || kind == GEMM_TT);
}

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

// What a GEMM launch touches (trace mode): operands of `esize` bytes per element, result of
// `osize` bytes; `slabs`: the result is `splits` slabs of [M, ldc], one per k range.
inline void note_gemm(const GemmArgs& a, bool a_kc, bool b_kc, int esize, int osize, bool slabs) {
  if (!tracing()) return;
  note_matrix(a.A, a_kc ? a.M : a.K, a_kc ? a.K : a.M, a.lda, esize, false);
  note_matrix(a.B, b_kc ? a.N : a.K, b_kc ? a.K : a.N, a.ldb, esize, false);
  const int n_store = a.n_store > 0 ? a.n_store : a.N;
  const int64_t rows = slabs ? (int64_t)(a.splits - 1) * a.M + a.M : a.M;
  note_matrix(a.C, rows, n_store, a.ldc, osize, true);
  if (a.bias != nullptr) note_matrix(a.bias, 1, a.N, a.N, esize, false);
  if (a.colsum != nullptr) note_matrix(a.colsum, a.splits, a.N, a.N, 4, true);
}
inline Work gemm_work(const GemmArgs& a, int esize, int osize, bool slabs) {
  const double n_store = a.n_store > 0 ? a.n_store : a.N;
  Work w;
  w.flops = 2.0 * a.M * a.N * a.K;
  w.bytes = ((double)a.M * a.K + (double)a.K * a.N) * esize + (double)a.M * n_store * osize * (slabs ? a.splits : 1) +
            (a.bias != nullptr ? (double)a.N * esize : 0.0) + (a.colsum != nullptr ? (double)a.splits * a.N * 4 : 0.0);
  return w;
}
inline Work reduce_work(const ReduceArgs& r) {
  Work w;
  w.flops = 0.0;
  w.bytes = 4.0 * ((double)r.n * (r.n > 0 ? r.splits + 1 : 0) + (double)r.n2 * (r.n2 > 0 ? r.splits2 + 1 : 0));
  return w;
}
inline void note_reduce(const ReduceArgs& r) {
  if (!tracing()) return;
  if (r.n > 0) {
    note_matrix(r.part, r.splits, r.n, r.n, 4, false);
    note_matrix(r.out, 1, r.n, r.n, 4, true);
  }
  if (r.n2 > 0) {
    note_matrix(r.part2, r.splits2, r.n2, r.n2, 4, false);
    note_matrix(r.out2, 1, r.n2, r.n2, 4, true);
  }
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

// Backward pass of a narrow sketch (bf16, R <= 32) in one pass over x and dY: per token
// tile (32 or 64 tokens) the kernel recomputes Z = x . S_cat, forms G = dY . U_cat^T and from it the tile of
// dX, and leaves the tile's term of dU_cat (and of dbias) as an fp32 slab; a second kernel
// (launch_reduce_tiles) sums the slabs in tile order.
struct NarrowBwdArgs {
  const void* x;     // [M, K1]
  const void* S;     // [K1, R]
  const void* dY;    // [M, N]
  const void* U;     // [R, N]
  void* dX;          // [M, K1]
  float* du_slabs;   // [tiles_m][R][N]:  Z_tile^T . dY_tile
  float* db_slabs;   // [tiles_m][N]:     column sums of dY_tile, or null
  int M, K1, R, N;
  int tm;            // tokens per work-group: 32 or 64
  int tiles_m;       // filled in by the launcher
  float scale;       // of dX
};
int narrow_bwd_max_in(int R);   // largest K1 whose S_cat fits the kernel's LDS (0: R not served)
hipError_t launch_reduce_tiles(const ReduceArgs& a, hipStream_t s);
hipError_t launch_bwd_narrow_bf16(NarrowBwdArgs a, hipStream_t s);

}  // namespace sk
