// libsk's C ABI (include/sk.h): argument validation, per-shape plan, launches.
// Validation runs before any HIP call, so error paths work without a GPU.
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <string>

#include <vector>

#include "../../include/sk.h"
#include "../../include/sk_debug.h"
#include "sk_launch.h"

// Scratch of sk_linear_bwd_weight_noalloc (SK_NOALLOC_SCRATCH_BYTES, include/sk.h): device
// memory that belongs to the loaded code object (one copy per GPU, held until the process
// ends), so that entry point needs no workspace from its caller and no allocation of its
// own.  In host code this name is only a handle for hipGetSymbolAddress; kernels are given
// the address that call returns.
static __device__ __align__(256) unsigned char scratch[SK_NOALLOC_SCRATCH_BYTES];

namespace {

using namespace sk;

constexpr size_t WS_ALIGN = 256;

thread_local std::string g_hip_error;
std::atomic<int> g_plan{0};

// Forced plan parameters (sk_set_tuning; negative = the planner chooses).
std::atomic<int> g_tune[SK_TUNE_COUNT] = {{-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}, {-1}};
int tune(sk_tune_knob knob) { return g_tune[knob].load(std::memory_order_relaxed); }

// The calling thread's launch trace or kernel timer (include/sk_debug.h); null otherwise.
struct Hooks : LaunchHooks {
  bool trace = false;
  std::vector<sk_trace_access> accesses;
  int launches = 0;
  // profile mode
  std::vector<hipEvent_t> events;       // 2 per kernel: before, after
  std::vector<std::string> names;
  std::vector<unsigned> groups;
  std::vector<Work> work;
  int max_kernels = 0;
  bool recording = false;               // the current launch got its `before` event

  bool tracing() const override { return trace; }
  void access(const void* p, uint64_t bytes, bool write) override {
    sk_trace_access a;
    a.address = (uint64_t)reinterpret_cast<uintptr_t>(p);
    a.bytes = bytes;
    a.write = write ? 1 : 0;
    a.launch = launches;
    accesses.push_back(a);
  }
  void launch_recorded() override { ++launches; }
  void before(const char* name, unsigned g, double flops, double bytes, hipStream_t s) override {
    recording = (int)names.size() < max_kernels;
    if (!recording) return;
    if (hipEventRecord(events[2 * names.size()], s) != hipSuccess) { recording = false; return; }
    names.push_back(name);
    groups.push_back(g);
    work.push_back(Work{flops, bytes});
  }
  void after(hipStream_t s) override {
    if (recording) (void)hipEventRecord(events[2 * names.size() - 1], s);
    recording = false;
  }
};
thread_local Hooks* g_hooks = nullptr;

size_t align_up(size_t v) { return (v + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }

sk_status hip_fail(hipError_t e, const char* what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  return SK_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Shape {
  int64_t T, in, out;
  int l, k, R;
  sk_dtype dtype;
  size_t esize;
};

// Checks everything that does not involve pointers.
sk_status check_shape(int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                      sk_dtype dtype, Shape& s) {
  if (tokens < 1 || in < 1 || out < 1 || l < 1 || k < 1) return SK_ERR_INVALID_ARG;
  if (dtype != SK_F32 && dtype != SK_BF16) return SK_ERR_UNSUPPORTED;
  const int64_t R = (int64_t)l * k;
  if ((in & 15) || (out & 15) || (R & 15)) return SK_ERR_UNSUPPORTED;
  // index arithmetic inside the kernels is 32-bit per dimension
  if (tokens > (1 << 24) || in > (1 << 20) || out > (1 << 20) || R > (1 << 16))
    return SK_ERR_UNSUPPORTED;
  s.T = tokens; s.in = in; s.out = out; s.l = l; s.k = k; s.R = (int)R; s.dtype = dtype;
  s.esize = dtype == SK_BF16 ? 2 : 4;
  return SK_OK;
}

}  // namespace

namespace sk {
LaunchHooks* launch_hooks() { return g_hooks; }
}  // namespace sk

namespace {

// Tile choice for the general GEMM (measured on MI355X).  The 256 x 256 tile with eight
// waves has the best steady state (fewest LDS instructions per MFMA) but a long prologue,
// so it pays from a contraction of 512 on when its tiles fill the chip; 128 x 128 runs two work-groups per CU, which overlaps one
// tile's stores with the other's MFMAs.  Otherwise: the largest tile that still gives
// every CU a work-group without being mostly padding, the smallest when the problem
// cannot fill the chip.
int choose_tile(int64_t M, int64_t N, int64_t K, int splits) {
  if (const int t = tune(SK_TUNE_TILE); t >= 0 && t < TILE_COUNT) return t;  // forced (tests, sweeps)
  const int64_t m_cap = (M + 63) / 64 * 64, n_cap = (N + 63) / 64 * 64;
  static const int order[] = {TILE_256x256_W8, TILE_128x128, TILE_128x64, TILE_64x128, TILE_64x64};
  for (int i = 0; i < (int)(sizeof(order) / sizeof(order[0])); ++i) {
    const int t = order[i];
    int bm, bn;
    tile_dims(t, bm, bn);
    if (bm > m_cap || bn > n_cap) continue;
    if (t == TILE_256x256_W8 && K / splits < 512) continue;
    const int64_t wgs = ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * splits;
    if (wgs >= NUM_CUS) return t;
  }
  return TILE_64x64;
}

// fp32 first contraction (one tile shape, 64 x 64): split over a long contraction when its
// tiles leave most of the chip idle -- ranges at least 256 long, at most 8.
int f32_first_splits(int64_t M, int64_t N, int64_t K) {
  const int64_t tiles = ((M + F32_BM - 1) / F32_BM) * ((N + F32_BN - 1) / F32_BN);
  int64_t sp = NUM_CUS / tiles;
  if (sp > K / 256) sp = K / 256;
  if (sp > 8) sp = 8;
  if (sp < 2 || K < 1024) return 1;
  const int64_t kps = ((K + sp - 1) / sp + F32_BK - 1) / F32_BK * F32_BK;
  return (int)((K + kps - 1) / kps);
}

// A first contraction of the layer run as a general GEMM: bf16 [M, N] result (the narrow
// intermediate, or its transpose), contraction length K.  Over a long K a small output
// leaves the choice between small tiles that fill the chip unsplit and large tiles split
// over K into fp32 slabs, which one more small kernel sums into the bf16 result.  The same
// rates as the token-split model rank the two (per work-group flop/s by tile; slabs written
// and re-read at 4 TB/s; 5 us for the extra launch), and the split form has to win by a
// tenth to be taken (measured on the 8192-wide layers: modelled ratios of 0.85 paid, 0.95
// did not).  8192-wide layer, R = 256, 4096 tokens: 54 us unsplit on 64 x 64 tiles.
struct FirstPlan {
  int tile, splits, k_per_split;
  size_t slab_bytes;   // fp32 slabs (0 when not split)
};
FirstPlan plan_first(int64_t M, int64_t N, int64_t K) {
  FirstPlan f{};
  f.tile = choose_tile(M, N, K, 1);
  f.splits = 1;
  f.k_per_split = (int)((K + 63) / 64 * 64);
  f.slab_bytes = 0;
  auto rate = [](int bm, int bn) {
    return bm * bn >= 256 * 256 ? 5.0e12 : bm * bn >= 128 * 128 ? 3.5e12 : bm * bn >= 128 * 64 ? 2.2e12 : 1.5e12;
  };
  auto time_of = [&](int tile, int64_t splits, int64_t kps) {
    int bm, bn;
    tile_dims(tile, bm, bn);
    const int64_t wgs = ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * splits;
    const int64_t rounds = (wgs + NUM_CUS - 1) / NUM_CUS;
    double t = rounds * (double)kps * 2.0 * bm * bn / rate(bm, bn);
    if (splits > 1) t += splits * (double)M * N * 8.0 / 4.0e12 + 5.0e-6;
    return t;
  };
  if (tune(SK_TUNE_TILE) >= 0) return f;  // a forced tile is taken as it is
  const double t_plain = time_of(f.tile, 1, K);
  double best = t_plain * 0.9;
  static const int cand[] = {TILE_128x128, TILE_128x64, TILE_64x128};
  for (int c = 0; c < 3; ++c) {
    int bm, bn;
    tile_dims(cand[c], bm, bn);
    if (bm > (M + 63) / 64 * 64 || bn > (N + 63) / 64 * 64) continue;
    for (int64_t sp = 2; sp <= 8; ++sp) {
      int64_t kps = (K + sp - 1) / sp;
      kps = (kps + 63) / 64 * 64;
      if (kps < 512) break;
      const int64_t sp_eff = (K + kps - 1) / kps;
      if (sp_eff < 2) continue;
      const double t = time_of(cand[c], sp_eff, kps);
      if (t < best) { best = t; f.tile = cand[c]; f.splits = (int)sp_eff; f.k_per_split = (int)kps; }
    }
  }
  if (f.splits > 1) f.slab_bytes = align_up((size_t)f.splits * M * N * 4);
  return f;
}

struct WeightPlan {
  int tile;
  int splits;
  int k_per_split;
  int64_t ldz;         // bf16: row stride of Z^T [R, ldz]
  bool own_colsum;     // db from its own kernel (the big tile has no registers for it)
  int colsum_splits;   // rows of column-sum partials: `splits`, or the own kernel's row runs
  int colsum_rows;     // tokens per row run of the own kernel
  // Uneven split (big tile only): the first head_cols output columns are one full round
  // of tiles over all tokens, straight into dU; only the rest is split over the tokens.
  int head_cols;       // 0: the whole output is split evenly (`splits`)
  int z_tile;          // bf16: tile of the GEMM that recomputes Z^T
  int z_splits;        // split of that GEMM over `in` (fp32 slabs, summed into bf16 Z^T)
  int z_k_per_split;
  size_t z_bytes, part_bytes, csum_bytes, zpart_bytes;
  size_t total() const { return z_bytes + part_bytes + csum_bytes + zpart_bytes; }
};

// A contraction over the token axis with a small fp32 output [M, N] (a weight gradient):
// tile and split of the tokens.  Every split writes and re-reads a slab of the output,
// so: as few splits as fill the chip, at least 256 tokens each, summed in a fixed
// order (deterministic).
struct TokenPlan {
  int tile;            // bf16 tile configuration; -1 for fp32 (one tile shape)
  bool big_tile;       // 256 x 256: no registers left for column sums in the kernel
  int splits, k_per_split;
};

// Split count with the least modelled time for one tile shape: rounds of work-groups over
// the chip x tokens per split x the tile's time per token, plus writing and re-reading one
// fp32 slab per split.  Rates are measured ones (flop/s one work-group sustains; HBM
// bytes/s); the model only has to rank the candidates.
struct SplitChoice {
  double time;
  int64_t splits, kps;
};
static SplitChoice best_split(int64_t M, int64_t N, int64_t T, int bm, int bn, bool bf16) {
  const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  const double wg_rate = !bf16 ? 0.3e12 : bm * bn >= 256 * 256 ? 5.0e12
                         : bm * bn >= 128 * 128 ? 3.5e12 : bm * bn >= 128 * 64 ? 2.2e12 : 1.5e12;
  const double t_token = 2.0 * bm * bn / wg_rate;
  const double t_slab = (double)M * N * 8.0 / 4.0e12;
  int64_t max_splits = (T + 255) / 256;   // at least 256 tokens each
  if (max_splits > 32) max_splits = 32;
  SplitChoice c{-1.0, 1, (T + 63) / 64 * 64};
  for (int64_t sp = 1; sp <= max_splits; ++sp) {
    int64_t k = (T + sp - 1) / sp;
    k = (k + 63) / 64 * 64;
    const int64_t sp_eff = (T + k - 1) / k;
    const int64_t rounds = (tiles * sp_eff + NUM_CUS - 1) / NUM_CUS;
    const double t = rounds * k * t_token + (sp_eff > 1 ? sp_eff * t_slab + 2.0e-6 : 0.0);
    if (c.time < 0.0 || t < c.time) { c.time = t; c.splits = sp_eff; c.kps = k; }
  }
  return c;
}

TokenPlan plan_tokens(int64_t M, int64_t N, int64_t T, sk_dtype dtype, bool tunable) {
  TokenPlan w{};
  int bm, bn;
  if (dtype == SK_BF16) {
    w.tile = M > 64 ? TILE_128x64 : TILE_64x64;
    if (((M + 255) / 256) * ((N + 255) / 256) >= NUM_CUS) {
      w.tile = TILE_256x256_W8;
    } else if (M > 64) {
      // 128 x 64 or 128 x 128, whichever the model has finishing first: the narrower
      // tile fills the chip with fewer token splits (few tokens: c1, c2), the square one
      // moves fewer bytes per flop (from half a chip of tiles on, or many tokens:
      // [65536 x 768 -> 3072], R = 128 measured 152 -> 132 us)
      if (best_split(M, N, T, 128, 128, true).time < best_split(M, N, T, 128, 64, true).time)
        w.tile = TILE_128x128;
    }
    if (const int t = tunable ? tune(SK_TUNE_WTILE) : -1; t >= 0 && t < TILE_COUNT) w.tile = t;  // forced
    w.big_tile = w.tile == TILE_256x256_W8 || w.tile == TILE_256x256;
    tile_dims(w.tile, bm, bn);
  } else {
    w.tile = -1;
    bm = F32_BM; bn = F32_BN;
  }
  const SplitChoice c = best_split(M, N, T, bm, bn, dtype == SK_BF16);
  int64_t splits = c.splits, kps = c.kps;
  int64_t max_splits = (T + 255) / 256;
  if (max_splits > 32) max_splits = 32;
  if (const int f = tunable ? tune(SK_TUNE_WSPLITS) : -1; f >= 0) {  // forced (clamped to 1..max)
    splits = f < 1 ? 1 : (f > max_splits ? max_splits : f);
    kps = ((T + splits - 1) / splits + 63) / 64 * 64;
    splits = (T + kps - 1) / kps;
  }
  w.splits = (int)splits;
  w.k_per_split = (int)kps;
  return w;
}

// dU = Z^T . dY with Z recomputed: where its pieces live in the workspace.
WeightPlan plan_weight(const Shape& s) {
  WeightPlan w{};
  const TokenPlan t = plan_tokens(s.R, s.out, s.T, s.dtype, true);
  w.tile = t.tile;
  w.own_colsum = t.big_tile;
  w.z_splits = 1;
  w.z_k_per_split = (int)s.in;
  if (s.dtype == SK_BF16) {
    w.ldz = (s.T + 63) / 64 * 64;
    w.z_bytes = align_up((size_t)s.R * w.ldz * 2);
    // Z^T [R, T] recomputed as a general GEMM over `in` (plan_first: split over a long
    // `in` when its tiles are few -- the paper's 8192-wide layers at R = 16: 64 tiles of
    // 64 x 64 walking 128 chunks each took 51 us, four ranges and the sum take 17)
    const FirstPlan f = plan_first(s.R, s.T, s.in);
    w.z_tile = f.tile;
    w.z_splits = f.splits;
    w.z_k_per_split = f.k_per_split;
    w.zpart_bytes = w.z_splits > 1 ? align_up((size_t)w.z_splits * s.R * w.ldz * 4) : 0;
  } else {
    w.ldz = s.R;
    w.z_bytes = align_up((size_t)s.T * s.R * 4);
    w.z_tile = -1;
    w.z_splits = f32_first_splits(s.T, s.R, s.in);   // Z = x . S_cat, split like any first GEMM
    w.zpart_bytes = w.z_splits > 1 ? align_up((size_t)w.z_splits * s.T * s.R * 4) : 0;
  }
  const int64_t splits = t.splits, kps = t.k_per_split;
  w.splits = (int)splits;
  w.k_per_split = (int)kps;
  w.colsum_splits = w.splits;
  w.colsum_rows = w.k_per_split;
  if (w.own_colsum) {
    // the column-sum kernel splits the tokens by itself, enough to fill the chip
    const int64_t col_groups = (s.out + 511) / 512;
    int64_t cs = (4 * NUM_CUS + col_groups - 1) / col_groups;
    const int64_t max_cs = (s.T + 127) / 128;
    if (cs > max_cs) cs = max_cs;
    if (cs > 48) cs = 48;
    if (cs < 1) cs = 1;
    int64_t rows = (s.T + cs - 1) / cs;
    rows = (rows + 31) / 32 * 32;
    w.colsum_rows = (int)rows;
    w.colsum_splits = (int)((s.T + rows - 1) / rows);
  }
  w.head_cols = 0;
  if (w.own_colsum && splits > 1 && s.R <= 65535 && tune(SK_TUNE_WSPLITS) < 0) {
    // More tiles than CUs but fewer than two rounds (c4: 344 tiles of 256 x 256): a round of
    // whole-token tiles covering as many tile columns as fit, then the remaining columns
    // split over the tokens so that they fill one more, shorter round.  Against the even
    // split that is the same MFMA time with a fraction of the slabs (c4: 2 x 90 MB -> 2 x 23 MB).
    const int64_t tm = (s.R + 255) / 256, tn = (s.out + 255) / 256;
    const int64_t head_tn = NUM_CUS / tm;
    if (tm * tn > NUM_CUS && tm * tn < 2 * NUM_CUS && head_tn >= 1 && head_tn < tn &&
        head_tn * tm * 4 >= NUM_CUS * 3) {
      const int64_t tail_tiles = (tn - head_tn) * tm;
      int64_t sp = NUM_CUS / tail_tiles;
      if (sp > (s.T + 1023) / 1024) sp = (s.T + 1023) / 1024;
      if (sp > 8) sp = 8;
      if (sp >= 2) {
        int64_t k2 = ((s.T + sp - 1) / sp + 63) / 64 * 64;
        w.head_cols = (int)(head_tn * 256);
        w.splits = (int)((s.T + k2 - 1) / k2);
        w.k_per_split = (int)k2;
      }
    }
  }
  const int64_t split_cols = s.out - w.head_cols;
  w.part_bytes = w.splits > 1 ? align_up((size_t)w.splits * s.R * split_cols * 4) : 0;
  w.csum_bytes = w.colsum_splits > 1 ? align_up((size_t)w.colsum_splits * s.out * 4) : 0;
  return w;
}

// Kernel plans of the forward and the input gradient.
enum Plan : int {
  PLAN_AUTO = 0,
  PLAN_FUSED = 1,         // one kernel, intermediate tile never leaves the chip (bf16, R <= 256)
  PLAN_TWO_GEMM = 2,      // two general GEMMs, bf16/fp32 intermediate through the workspace
  PLAN_SPLIT_EXPAND = 3,  // split-K sketch GEMM into fp32 slabs, then the expand kernel that
                          // sums them on the way into LDS (bf16, R <= 512)
};

// Shape of the expand/fused launch: rows of a token tile and the number of N slices (one
// work-group per CU).
struct ChainShape {
  int bm, slices;
};
ChainShape chain_shape(int64_t T, int64_t N, int R, bool share_cu) {
  ChainShape c;
  // 128-row token tiles halve the B2 traffic and the LDS reads per MFMA of stage 2; they
  // pay once their tiles alone fill the chip (measured on [T x 768 -> 3072], R = 128:
  // forward -14..16 % from 65536 tokens on, +17 % at 4096 tokens, where they double the
  // number of work-groups that repeat stage 1)
  c.bm = (R <= 128 && T >= 128 * (int64_t)NUM_CUS) ? 128 : 64;
  if (const int v = tune(SK_TUNE_BM); v == 64 || (v == 128 && R <= 128)) c.bm = v;  // forced
  const int64_t tiles_m = (T + c.bm - 1) / c.bm;
  const int64_t n_tiles = (N + chain_bn(R) - 1) / chain_bn(R);
  int64_t sl = NUM_CUS / tiles_m;
  // share_cu: the expansion alone (no first contraction to repeat per slice, no carried
  // reduction to deal out) of a sketch up to 64 wide is small enough in LDS for two
  // work-groups per CU (8192-wide layer, R = 16: input gradient 39.8 -> 33.5 us)
  if (share_cu && R <= 64) sl = 2 * NUM_CUS / tiles_m;
  // No work-group walks more than 24 output tiles: with many tokens and a wide output every
  // CU otherwise streams its own 64 rows end to end, 16384 rows are being written at once
  // and the stores crawl ([65536 x 8192 -> 8192], R = 128: forward 1030 us with one run of
  // 64 tiles per token tile, 550 us with four runs of 16)
  if (sl < (n_tiles + 23) / 24) sl = (n_tiles + 23) / 24;
  if (const int v = tune(SK_TUNE_SLICES); v >= 0) sl = v;  // forced (clamped below)
  if (sl > n_tiles) sl = n_tiles;
  if (sl < 1) sl = 1;
  c.slices = (int)sl;
  return c;
}

Plan pick_plan(const Shape& s, sk_op op) {
  const int forced = g_plan.load(std::memory_order_relaxed);
  const bool chain_ok = s.dtype == SK_BF16 && chain_supported(s.R);
  const bool fused_ok = chain_ok && s.R <= CHAIN_FUSED_MAX_R;
  switch (forced) {
    case PLAN_FUSED: return fused_ok ? PLAN_FUSED : (chain_ok ? PLAN_SPLIT_EXPAND : PLAN_TWO_GEMM);
    case PLAN_TWO_GEMM: return PLAN_TWO_GEMM;
    case PLAN_SPLIT_EXPAND: return chain_ok ? PLAN_SPLIT_EXPAND : PLAN_TWO_GEMM;
    default: break;
  }
  // automatic (measured on MI355X): the on-chip plans win while the sketch is narrow
  // (R <= 128: the layer is bound by bytes and by launch count); wider sketches run
  // faster as two general GEMMs with large tiles.  One fused kernel recomputes the first
  // contraction once per N slice, which is cheap while length x slices stays small: up to
  // about 6000 (the forward of an up-projection at 4096 tokens: 768 x 4; its input
  // gradient, 3072 long, from two slices down, i.e. from 6144 tokens on, where it
  // measured level at two slices and 16-20 % ahead at one).  Beyond that the first
  // contraction is split over its length instead and the expansion sums the slabs.
  if (chain_ok && s.R <= 128) {
    const int64_t k1 = op == SK_OP_FWD ? s.in : s.out;
    const int64_t n2 = op == SK_OP_FWD ? s.out : s.in;
    return k1 * chain_shape(s.T, n2, s.R, false).slices <= 6144 ? PLAN_FUSED : PLAN_SPLIT_EXPAND;
  }
  return PLAN_TWO_GEMM;
}

// Split of the first contraction (M = tokens, N = R, contraction length K) so that a
// skinny output still fills the chip: fp32 slabs, one per k range, summed in order by
// the consumer.  splits == 1 means the bf16 result is written directly.
struct SketchPlan {
  int tile, splits, k_per_split;
  size_t bytes;
};

SketchPlan plan_sketch(const Shape& s, int64_t K) {
  SketchPlan q{};
  q.tile = s.R <= 64 ? TILE_64x64 : (s.R <= 256 ? TILE_64x128 : TILE_128x128);
  if (const int t = tune(SK_TUNE_STILE);  // forced
      t == TILE_64x64 || t == TILE_64x128 || t == TILE_128x128 || t == TILE_128x64)
    q.tile = t;
  int bm, bn;
  tile_dims(q.tile, bm, bn);
  const int64_t tiles = ((s.T + bm - 1) / bm) * ((s.R + bn - 1) / bn);
  // one work-group per CU; two for the 64 x 64 tile (R <= 64), whose work-groups are small
  // enough to share a CU and, streaming a long x from HBM, need the loads in flight of
  // two (8192-wide layer, R = 16: forward 36.8 -> 33.5 us)
  const int64_t want = s.R <= 64 ? 2 * NUM_CUS : NUM_CUS;
  int64_t splits = (want + tiles - 1) / tiles;
  if (const int v = tune(SK_TUNE_SSPLITS); v >= 0) splits = v;  // forced (clamped below)
  const int64_t max_splits = K / 128 > 0 ? K / 128 : 1;   // at least two k chunks each
  if (splits > max_splits) splits = max_splits;
  if (splits > 8) splits = 8;
  if (splits < 1) splits = 1;
  int64_t kps = (K + splits - 1) / splits;
  kps = (kps + 63) / 64 * 64;
  splits = (K + kps - 1) / kps;
  q.splits = (int)splits;
  q.k_per_split = (int)kps;
  q.bytes = splits > 1 ? align_up((size_t)splits * s.T * s.R * 4) : align_up((size_t)s.T * s.R * 2);
  return q;
}

// Workspace of the first-stage gradient for nc columns: G = dY . U_sub^T [T, nc] in the
// storage type, then the token-split slabs of dA [in, nc].
size_t first_stage_bytes(const Shape& s, int64_t nc) {
  const TokenPlan t = plan_tokens(s.in, nc, s.T, s.dtype, false);
  const size_t da_slabs = t.splits > 1 ? align_up((size_t)t.splits * s.in * nc * 4) : 0;
  // slabs of G when its GEMM is split over `out`: dead once summed, so they share the
  // region of the dA slabs
  size_t g_slabs;
  if (s.dtype == SK_BF16) {
    g_slabs = plan_first(s.T, nc, s.out).slab_bytes;
  } else {
    const int sp = f32_first_splits(s.T, nc, s.out);
    g_slabs = sp > 1 ? align_up((size_t)sp * s.T * nc * 4) : 0;
  }
  return align_up((size_t)s.T * nc * s.esize) + (da_slabs > g_slabs ? da_slabs : g_slabs);
}

// Both gradients of a narrow sketch in one pass over x and dY (sk_bwd_narrow.hip): a
// work-group per tile of 32 or 64 tokens produces its rows of dX outright and leaves one
// fp32 slab of dU_cat (and of dbias) behind, which a second kernel sums; G never leaves the
// chip and three launches become two.  A work-group is four waves on a CU of its own, so
// nothing hides its latencies but its own prefetching, and it takes 13-18 us for its tile
// whatever the token count; a second round of work-groups doubles that.  Measured on MI355X
// (in = out = 768, R = 32, backward call; 32-token tiles / 64-token tiles / the three-launch
// schedule, us): 512 tokens 16.2 / - / 20.7, 2048 18.4 / 22.1 / 22.6, 4096 21.1 / 24.4 /
// 23.2, 8192 25.9 / 27.5 / 30.5, 12288 41.4 / 30.7 / 35.4, 16384 46.3 / 34.8 / 38.8, 20480
// - / 52.9 / 44.5; R = 64 (a variant of the kernel since removed) lost at every size.
// A sweep over in = 64..768 and out = 64..3072 at 256..16384 tokens (same call, one pass
// over three launches): out <= 256 0.63-0.84, out = 768 0.80-1.04, out = 1024 0.83-1.14
// (R = 16: 0.82-1.03), out = 2048 1.06-1.31, out = 3072 1.20-1.59 -- a work-group walks all
// of `out`, and the walk is what it cannot hide.
// So: R <= 32, out <= 896 (1024 for R = 16), one round of work-groups, slabs of at most 32 MiB.
struct NarrowPlan {
  bool ok;
  int tm, tiles_m;   // tokens per work-group (32 or 64), work-groups
  size_t du_bytes, db_bytes;
  size_t total() const { return du_bytes + db_bytes; }
};

NarrowPlan plan_narrow(const Shape& s) {
  NarrowPlan n{};
  const int forced = tune(SK_TUNE_NARROW_BWD);
  if (s.dtype != SK_BF16 || g_plan.load(std::memory_order_relaxed) != PLAN_AUTO || forced == 0) return n;
  if (s.in > narrow_bwd_max_in(s.R)) return n;   // (0 for a sketch the kernel does not serve)
  // 32-token tiles while they make one round of work-groups with slabs under the cap, 64-token
  // tiles beyond; only while a work-group's walk over `out` stays short
  for (int tm = 32; tm <= 64; tm *= 2) {
    if ((forced == 32 || forced == 64) && tm != forced) continue;
    const int64_t tiles_m = (s.T + tm - 1) / tm;
    const size_t du = (size_t)tiles_m * s.R * s.out * 4;
    const bool fits = du <= ((size_t)32 << 20) && tiles_m <= NUM_CUS && s.out <= (s.R <= 16 ? 1024 : 896);
    if (forced < 0 && !fits) continue;
    if (forced > 0 && forced != 32 && forced != 64 && !fits && tm == 32) continue;   // forced without a tile height: 64 unless 32 fits
    n.ok = true;
    n.tm = tm;
    n.tiles_m = (int)tiles_m;
    n.du_bytes = align_up(du);
    n.db_bytes = align_up((size_t)tiles_m * s.out * 4);
    return n;
  }
  return n;
}

size_t workspace_for(sk_op op, const Shape& s) {
  const size_t mid = align_up((size_t)s.T * s.R * s.esize);  // Z or G
  switch (op) {
    case SK_OP_FWD:
    case SK_OP_BWD_INPUT: {
      // the maximum over the plans, so one buffer serves whichever is selected
      size_t need = mid;
      if (s.dtype == SK_BF16)   // two GEMMs with the first one split: slabs behind the intermediate
        need += plan_first(s.T, s.R, op == SK_OP_FWD ? s.in : s.out).slab_bytes;
      else {
        const int sp = f32_first_splits(s.T, s.R, op == SK_OP_FWD ? s.in : s.out);
        if (sp > 1) need += align_up((size_t)sp * s.T * s.R * 4);
      }
      if (s.dtype == SK_BF16 && chain_supported(s.R)) {
        const size_t b = plan_sketch(s, op == SK_OP_FWD ? s.in : s.out).bytes;
        if (b > need) need = b;
      }
      return need;
    }
    case SK_OP_BWD_WEIGHT:
      return plan_weight(s).total();
    case SK_OP_BWD: {
      const size_t two = workspace_for(SK_OP_BWD_INPUT, s) + workspace_for(SK_OP_BWD_WEIGHT, s);
      const NarrowPlan n = plan_narrow(s);
      return n.ok && n.total() > two ? n.total() : two;
    }
    case SK_OP_BWD_WEIGHT_FIRST: {
      // the maximum over every admissible column count (narrow ranges split the tokens
      // further), so one buffer serves any range
      size_t need = 0;
      for (int64_t nc = 16; nc <= s.R; nc += 16) {
        const size_t b = first_stage_bytes(s, nc);
        if (b > need) need = b;
      }
      return need;
    }
  }
  return 0;
}

hipError_t gemm(const Shape& s, GemmKind kind, GemmArgs a, hipStream_t st) {
  if (s.dtype == SK_BF16) return launch_gemm_bf16(kind, choose_tile(a.M, a.N, a.K, 1), a, st);
  return launch_gemm_f32(kind, a, st);
}

// The first of the two GEMMs of a call: as it is, or (bf16, plan_first) split over its
// contraction into fp32 slabs at `slabs` that are then summed into the bf16 result a.C.
hipError_t first_gemm(const Shape& s, GemmKind kind, GemmKind kind_slabs, GemmArgs a, void* slabs,
                      hipStream_t st) {
  if (s.dtype != SK_BF16) {
    const int splits = f32_first_splits(a.M, a.N, a.K);
    if (splits == 1) return launch_gemm_f32(kind, a, st);
    // fp32: the same kernel writes the slabs (one per range of the contraction); summed in order
    float* out = static_cast<float*>(a.C);
    a.C = slabs; a.splits = splits;
    a.k_per_split = (int)(((a.K + splits - 1) / splits + F32_BK - 1) / F32_BK * F32_BK);
    a.splits = (a.K + a.k_per_split - 1) / a.k_per_split;
    const hipError_t e = launch_gemm_f32(kind, a, st);
    if (e != hipSuccess) return e;
    ReduceArgs r{};
    r.part = static_cast<const float*>(slabs); r.out = out; r.n = (int64_t)a.M * a.N; r.scale = 1.0f;
    r.splits = a.splits; r.splits2 = 1; r.scale2 = 1.0f;
    return launch_reduce_splits(r, st);
  }
  const FirstPlan f = plan_first(a.M, a.N, a.K);
  if (f.splits == 1) return launch_gemm_bf16(kind, f.tile, a, st);
  void* out = a.C;
  a.C = slabs; a.splits = f.splits; a.k_per_split = f.k_per_split;
  const hipError_t e = launch_gemm_bf16(kind_slabs, f.tile, a, st);
  if (e != hipSuccess) return e;
  return launch_reduce_to_bf16(static_cast<const float*>(slabs), out, (int64_t)a.M * a.N, f.splits, st);
}

// C[M,N] = scale * (A[M,K] . B) + bias through the workspace-free single GEMM.
GemmArgs dense_args(const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                    int64_t M, int64_t N, int64_t K, float scale, const void* bias) {
  GemmArgs a{};
  a.A = A; a.B = B; a.C = C; a.bias = bias; a.colsum = nullptr;
  a.lda = lda; a.ldb = ldb; a.ldc = ldc;
  a.M = (int)M; a.N = (int)N; a.K = (int)K;
  a.k_per_split = (int)((K + 63) / 64 * 64);
  a.splits = 1;
  a.scale = scale;
  return a;
}

}  // namespace

extern "C" {

const char* sk_status_string(sk_status status) {
  switch (status) {
    case SK_OK: return "SK_OK";
    case SK_ERR_INVALID_ARG: return "SK_ERR_INVALID_ARG: null or misaligned pointer, or non-positive size";
    case SK_ERR_UNSUPPORTED: return "SK_ERR_UNSUPPORTED: unknown dtype/op, or in/out/l*k not a multiple of 16";
    case SK_ERR_WORKSPACE: return "SK_ERR_WORKSPACE: workspace missing or too small";
    case SK_ERR_HIP: return "SK_ERR_HIP: a HIP call failed (see sk_last_hip_error)";
  }
  return "unknown sk_status";
}

const char* sk_last_hip_error(void) { return g_hip_error.c_str(); }

int sk_set_plan(int plan) {
  if (plan < 0 || plan > 3) return -1;
  return g_plan.exchange(plan);
}

int32_t sk_set_tuning(sk_tune_knob knob, int32_t value) {
  if ((int)knob < 0 || (int)knob >= SK_TUNE_COUNT) return INT32_MIN;
  return g_tune[knob].exchange(value < 0 ? -1 : value);
}

void sk_trace_begin(void) {
  delete g_hooks;
  g_hooks = new Hooks();
  g_hooks->trace = true;
}

int64_t sk_trace_end(sk_trace_access* out, int64_t max, int32_t* launches) {
  if (g_hooks == nullptr || !g_hooks->trace) return 0;
  const int64_t n = (int64_t)g_hooks->accesses.size();
  for (int64_t i = 0; i < n && i < max && out != nullptr; ++i) out[i] = g_hooks->accesses[i];
  if (launches != nullptr) *launches = g_hooks->launches;
  delete g_hooks;
  g_hooks = nullptr;
  return n;
}

int32_t sk_profile_begin(int32_t max_kernels) {
  delete g_hooks;
  g_hooks = nullptr;
  if (max_kernels < 1) return -1;
  Hooks* h = new Hooks();
  h->max_kernels = max_kernels;
  h->events.resize(2 * (size_t)max_kernels);
  for (size_t i = 0; i < h->events.size(); ++i) {
    if (hipEventCreate(&h->events[i]) != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(h->events[j]);
      delete h;
      return -2;
    }
  }
  g_hooks = h;
  return 0;
}

int32_t sk_profile_end(sk_kernel_time* out, int32_t max) {
  Hooks* h = g_hooks;
  if (h == nullptr || h->trace) return -1;
  g_hooks = nullptr;
  const int32_t n = (int32_t)h->names.size();
  int32_t rc = n;
  if (n > 0 && hipEventSynchronize(h->events[2 * (size_t)n - 1]) != hipSuccess) rc = -3;
  for (int32_t i = 0; rc >= 0 && i < n && i < max && out != nullptr; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, h->events[2 * (size_t)i], h->events[2 * (size_t)i + 1]) != hipSuccess) {
      rc = -4;
      break;
    }
    strncpy(out[i].name, h->names[i].c_str(), sizeof(out[i].name) - 1);
    out[i].name[sizeof(out[i].name) - 1] = 0;
    out[i].ms = ms;
    out[i].groups = (int32_t)h->groups[i];
    out[i].flops = h->work[i].flops;
    out[i].bytes = h->work[i].bytes;
  }
  for (hipEvent_t e : h->events) (void)hipEventDestroy(e);
  delete h;
  return rc;
}

size_t sk_linear_workspace_bytes(sk_op op, int64_t tokens, int64_t in, int64_t out, int32_t l,
                                 int32_t k, sk_dtype dtype) {
  Shape s;
  if (op != SK_OP_FWD && op != SK_OP_BWD_INPUT && op != SK_OP_BWD_WEIGHT &&
      op != SK_OP_BWD_WEIGHT_FIRST && op != SK_OP_BWD)
    return (size_t)-1;
  if (check_shape(tokens, in, out, l, k, dtype, s) != SK_OK) return (size_t)-1;
  return workspace_for(op, s);
}

sk_status sk_linear_fwd(const void* x, const void* S_cat, const void* U_cat, const void* bias,
                        void* y, int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                        sk_dtype dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !S_cat || !U_cat || !y) return SK_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(S_cat) || !aligned16(U_cat) || !aligned16(y) ||
      !aligned16(bias) || !aligned16(workspace))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float scale = 1.0f / (float)l;
  g_hip_error.clear();

  const Plan plan = pick_plan(s, SK_OP_FWD);
  if (plan != PLAN_FUSED && (!workspace || workspace_bytes < workspace_for(SK_OP_FWD, s)))
    return SK_ERR_WORKSPACE;
  if (plan == PLAN_FUSED || plan == PLAN_SPLIT_EXPAND) {
    ChainArgs c{};
    c.A = x; c.B1 = S_cat; c.B2 = U_cat; c.bias = bias; c.C = y;
    c.lda = in; c.ldb1 = s.R; c.ldb2 = out; c.ldc = out;
    c.M = (int)tokens; c.K1 = (int)in; c.R = s.R; c.N = (int)out; c.scale = scale;
    { const ChainShape cs = chain_shape(tokens, out, s.R, plan != PLAN_FUSED); c.n_slices = cs.slices; c.bm = cs.bm; }
    if (plan == PLAN_SPLIT_EXPAND) {
      const SketchPlan q = plan_sketch(s, in);
      GemmArgs a = dense_args(x, in, S_cat, s.R, workspace, s.R, tokens, s.R, in, 1.0f, nullptr);
      a.splits = q.splits; a.k_per_split = q.k_per_split;
      const hipError_t e1 = launch_gemm_bf16(q.splits > 1 ? GEMM_NN_F32 : GEMM_NN, q.tile, a, hs);
      if (e1 != hipSuccess) return hip_fail(e1, "sk_linear_fwd (x.S, split)");
      c.Z = workspace; c.z_splits = q.splits > 1 ? q.splits : 0; c.z_slab = (int64_t)tokens * s.R;
    }
    const hipError_t e = launch_chain_bf16(false, plan == PLAN_FUSED, c, hs);
    return e == hipSuccess ? SK_OK : hip_fail(e, "sk_linear_fwd (expand)");
  }
  // Z = x . S_cat, then y = scale * Z . U_cat + bias
  hipError_t e;
  e = first_gemm(s, GEMM_NN, GEMM_NN_F32,
                 dense_args(x, in, S_cat, s.R, workspace, s.R, tokens, s.R, in, 1.0f, nullptr),
                 static_cast<unsigned char*>(workspace) + align_up((size_t)tokens * s.R * s.esize), hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_fwd (x.S)");
  e = gemm(s, GEMM_NN, dense_args(workspace, s.R, U_cat, out, y, out, tokens, out, s.R, scale, bias), hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_fwd (Z.U)");
  return SK_OK;
}

sk_status sk_linear_bwd_input(const void* dY, const void* S_cat, const void* U_cat, void* dX,
                              int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                              sk_dtype dtype, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!dY || !S_cat || !U_cat || !dX) return SK_ERR_INVALID_ARG;
  if (!aligned16(dY) || !aligned16(S_cat) || !aligned16(U_cat) || !aligned16(dX) ||
      !aligned16(workspace))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float scale = 1.0f / (float)l;
  g_hip_error.clear();

  const Plan plan = pick_plan(s, SK_OP_BWD_INPUT);
  if (plan != PLAN_FUSED && (!workspace || workspace_bytes < workspace_for(SK_OP_BWD_INPUT, s)))
    return SK_ERR_WORKSPACE;
  if (plan == PLAN_FUSED || plan == PLAN_SPLIT_EXPAND) {
    ChainArgs c{};
    c.A = dY; c.B1 = U_cat; c.B2 = S_cat; c.bias = nullptr; c.C = dX;
    c.lda = out; c.ldb1 = out; c.ldb2 = s.R; c.ldc = in;
    c.M = (int)tokens; c.K1 = (int)out; c.R = s.R; c.N = (int)in; c.scale = scale;
    { const ChainShape cs = chain_shape(tokens, in, s.R, plan != PLAN_FUSED); c.n_slices = cs.slices; c.bm = cs.bm; }
    if (plan == PLAN_SPLIT_EXPAND) {
      const SketchPlan q = plan_sketch(s, out);
      GemmArgs a = dense_args(dY, out, U_cat, out, workspace, s.R, tokens, s.R, out, 1.0f, nullptr);
      a.splits = q.splits; a.k_per_split = q.k_per_split;
      const hipError_t e1 = launch_gemm_bf16(q.splits > 1 ? GEMM_NT_F32 : GEMM_NT, q.tile, a, hs);
      if (e1 != hipSuccess) return hip_fail(e1, "sk_linear_bwd_input (dY.U^T, split)");
      c.Z = workspace; c.z_splits = q.splits > 1 ? q.splits : 0; c.z_slab = (int64_t)tokens * s.R;
    }
    const hipError_t e = launch_chain_bf16(true, plan == PLAN_FUSED, c, hs);
    return e == hipSuccess ? SK_OK : hip_fail(e, "sk_linear_bwd_input (expand)");
  }
  // G = dY . U_cat^T (U_cat read as [N = R, K = out]), then dX = scale * G . S_cat^T
  hipError_t e = first_gemm(s, GEMM_NT, GEMM_NT_F32,
                            dense_args(dY, out, U_cat, out, workspace, s.R, tokens, s.R, out, 1.0f, nullptr),
                            static_cast<unsigned char*>(workspace) + align_up((size_t)tokens * s.R * s.esize), hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_input (dY.U^T)");
  e = gemm(s, GEMM_NT, dense_args(workspace, s.R, S_cat, s.R, dX, in, tokens, in, s.R, scale, nullptr), hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_input (G.S^T)");
  return SK_OK;
}

sk_status sk_linear_bwd_weight(const void* x, const void* S_cat, const void* dY, float* dU_cat,
                               float* dbias, int64_t tokens, int64_t in, int64_t out, int32_t l,
                               int32_t k, sk_dtype dtype, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (!x || !S_cat || !dY || !dU_cat) return SK_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(S_cat) || !aligned16(dY) || !aligned16(dU_cat) ||
      !aligned16(dbias) || !aligned16(workspace))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  const WeightPlan w = plan_weight(s);
  if (!workspace || workspace_bytes < workspace_for(SK_OP_BWD_WEIGHT, s)) return SK_ERR_WORKSPACE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float scale = 1.0f / (float)l;
  g_hip_error.clear();

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  void* Z = ws;
  float* part = reinterpret_cast<float*>(ws + w.z_bytes);
  float* cpart = reinterpret_cast<float*>(ws + w.z_bytes + w.part_bytes);

  // Z = x . S_cat is recomputed here rather than kept from the forward pass.  In bf16
  // it is produced transposed (Z^T = S_cat^T . x^T, [R, ldz] with zero-filled row
  // padding) so that the token contraction below reads it k-contiguous.
  GemmArgs a{};
  hipError_t e;
  if (s.dtype == SK_BF16) {
    GemmArgs z = dense_args(S_cat, s.R, x, in, Z, w.ldz, s.R, tokens, in, 1.0f, nullptr);
    z.n_store = (int)w.ldz;
    if (w.z_splits > 1) {
      float* zpart = reinterpret_cast<float*>(ws + w.z_bytes + w.part_bytes + w.csum_bytes);
      z.C = zpart; z.splits = w.z_splits; z.k_per_split = w.z_k_per_split;
      e = launch_gemm_bf16(GEMM_TT_F32, w.z_tile, z, hs);
      if (e == hipSuccess) e = launch_reduce_to_bf16(zpart, Z, (int64_t)s.R * w.ldz, w.z_splits, hs);
    } else {
      e = launch_gemm_bf16(GEMM_TT, w.z_tile, z, hs);
    }
    a.A = Z; a.lda = w.ldz;
  } else {
    e = first_gemm(s, GEMM_NN, GEMM_NN_F32, dense_args(x, in, S_cat, s.R, Z, s.R, tokens, s.R, in, 1.0f, nullptr),
                   ws + w.z_bytes + w.part_bytes + w.csum_bytes, hs);
    a.A = Z; a.lda = s.R;
  }
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (x.S)");

  // dU = scale * Z^T . dY and db = column sums of dY, the token axis split in order
  a.B = dY; a.ldb = out; a.ldc = out;
  a.M = s.R; a.N = (int)out; a.K = (int)tokens;
  a.splits = w.splits; a.k_per_split = w.k_per_split;
  a.bias = nullptr;
  if (w.splits == 1) {
    a.C = dU_cat; a.colsum = dbias; a.scale = scale;
  } else {
    a.C = part; a.colsum = dbias ? cpart : nullptr; a.scale = 1.0f;
  }
  if (s.dtype == SK_BF16 && w.own_colsum) {
    // the bias gradient from its own kernel -- or, with the uneven split, inside the launch of
    // the second, shorter round, whose GEMM leaves CUs free
    const bool ride = dbias && w.head_cols > 0 && w.tile == TILE_256x256_W8;
    if (dbias && !ride) {
      e = launch_colsum_bf16(dY, w.colsum_splits == 1 ? dbias : cpart, (int)tokens, (int)out,
                             w.colsum_splits, w.colsum_rows, hs);
      if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (column sums)");
    }
    if (w.head_cols > 0) {
      // first round: whole-token tiles of the first head_cols columns, straight into dU
      GemmArgs hd = a;
      hd.N = w.head_cols; hd.C = dU_cat; hd.colsum = nullptr; hd.scale = scale;
      hd.splits = 1; hd.k_per_split = (int)((tokens + 63) / 64 * 64);
      e = launch_gemm_bf16(GEMM_NN_F32, w.tile, hd, hs);
      if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (Z^T.dY, first columns)");
      // second, shorter round: the remaining columns, split over the tokens into slabs
      a.B = static_cast<const unsigned char*>(dY) + (size_t)w.head_cols * s.esize;
      a.N = (int)out - w.head_cols; a.ldc = a.N; a.C = part; a.colsum = nullptr; a.scale = 1.0f;
    }
    a.colsum = nullptr;   // (the big tiles have no column-sum epilogue: that is what the kernel above is for)
    if (ride)
      e = launch_gemm_f32slabs_with_colsum(w.tile, a, dY, w.colsum_splits == 1 ? dbias : cpart, (int)tokens,
                                           (int)out, w.colsum_splits, w.colsum_rows, hs);
    else
      e = launch_gemm_bf16(GEMM_NN_F32, w.tile, a, hs);
  } else {
    e = s.dtype == SK_BF16 ? launch_gemm_bf16(GEMM_NN_F32_COLSUM, w.tile, a, hs)
                           : launch_gemm_f32(GEMM_TN_F32, a, hs);
  }
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (Z^T.dY)");
  if (w.head_cols > 0) {
    e = launch_reduce_splits_2d(part, dU_cat + w.head_cols, s.R, (int)out - w.head_cols, out, w.splits,
                                scale, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (sum of the split columns)");
  }
  const bool sum_dU = w.splits > 1 && w.head_cols == 0;
  const bool sum_db = dbias && w.colsum_splits > 1;
  if (sum_dU || sum_db) {
    ReduceArgs r{};
    r.part = part; r.out = dU_cat; r.n = sum_dU ? (int64_t)s.R * out : 0; r.scale = scale;
    r.part2 = cpart; r.out2 = dbias; r.n2 = sum_db ? out : 0; r.scale2 = 1.0f;
    r.splits = w.splits; r.splits2 = w.colsum_splits;
    e = launch_reduce_splits(r, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight (sum of splits)");
  }
  return SK_OK;
}

sk_status sk_linear_bwd_weight_noalloc(const void* x, const void* S_cat, const void* dY,
                                       float* dU_cat, float* dbias, int64_t tokens, int64_t in,
                                       int64_t out, int32_t l, int32_t k, sk_dtype dtype,
                                       void* stream) {
  // everything sk_linear_bwd_weight would reject is rejected here first, before any HIP call
  if (!x || !S_cat || !dY || !dU_cat) return SK_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(S_cat) || !aligned16(dY) || !aligned16(dU_cat) || !aligned16(dbias))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  if (workspace_for(SK_OP_BWD_WEIGHT, s) > SK_NOALLOC_SCRATCH_BYTES) return SK_ERR_WORKSPACE;
  // the address of this GPU's copy of the array, looked up once per device
  constexpr int MAX_DEVICES = 64;
  static std::atomic<void*> device_scratch[MAX_DEVICES];
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight_noalloc (hipGetDevice)");
  if (dev < 0 || dev >= MAX_DEVICES) return SK_ERR_UNSUPPORTED;
  void* ptr = device_scratch[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return hip_fail(e != hipSuccess ? e : hipErrorInvalidSymbol,
                      "sk_linear_bwd_weight_noalloc (hipGetSymbolAddress)");
    device_scratch[dev].store(ptr, std::memory_order_release);
  }
  // Every region of the workspace is written by the call before it is read (Z^T with its
  // zero-filled row padding, the split slabs, the column-sum partials), so what an earlier
  // call left in the array needs no clearing.
  return sk_linear_bwd_weight(x, S_cat, dY, dU_cat, dbias, tokens, in, out, l, k, dtype, ptr,
                              SK_NOALLOC_SCRATCH_BYTES, stream);
}

sk_status sk_linear_bwd(const void* x, const void* dY, const void* S_cat, const void* U_cat,
                        void* dX, float* dU_cat, float* dbias, int64_t tokens, int64_t in,
                        int64_t out, int32_t l, int32_t k, sk_dtype dtype, void* workspace,
                        size_t workspace_bytes, void* stream) {
  if (!x || !dY || !S_cat || !U_cat || !dX || !dU_cat) return SK_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(dY) || !aligned16(S_cat) || !aligned16(U_cat) || !aligned16(dX) ||
      !aligned16(dU_cat) || !aligned16(dbias) || !aligned16(workspace))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  const size_t in_bytes = workspace_for(SK_OP_BWD_INPUT, s);
  const size_t w_bytes = workspace_for(SK_OP_BWD_WEIGHT, s);
  if (!workspace || workspace_bytes < workspace_for(SK_OP_BWD, s)) return SK_ERR_WORKSPACE;
  unsigned char* ws_in = static_cast<unsigned char*>(workspace);
  unsigned char* ws_w = ws_in + in_bytes;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float scale = 1.0f / (float)l;

  // --- narrow sketch, short input: one pass over x and dY | sum of the token tiles' slabs ---
  if (const NarrowPlan n = plan_narrow(s); n.ok) {
    g_hip_error.clear();
    NarrowBwdArgs b{};
    b.x = x; b.S = S_cat; b.dY = dY; b.U = U_cat; b.dX = dX;
    b.du_slabs = reinterpret_cast<float*>(ws_in);
    b.db_slabs = dbias ? reinterpret_cast<float*>(ws_in + n.du_bytes) : nullptr;
    b.M = (int)tokens; b.K1 = (int)in; b.R = s.R; b.N = (int)out; b.scale = scale; b.tm = n.tm;
    hipError_t e = launch_bwd_narrow_bf16(b, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (one pass over x and dY)");
    ReduceArgs t{};
    t.part = b.du_slabs; t.out = dU_cat; t.n = (int64_t)s.R * out; t.splits = n.tiles_m; t.scale = scale;
    t.part2 = b.db_slabs; t.out2 = dbias; t.n2 = dbias ? out : 0; t.splits2 = n.tiles_m; t.scale2 = 1.0f;
    e = launch_reduce_tiles(t, hs);
    return e == hipSuccess ? SK_OK : hip_fail(e, "sk_linear_bwd (sum of the token tiles)");
  }

  // Shared-launch schedules exist for the shapes the automatic plans produce on the
  // benchmark configurations (bf16; the dual kernel is built for a few tile pairs only);
  // everything else runs the two gradients one after the other.
  const WeightPlan w = plan_weight(s);
  // (not when Z^T is recomputed in split form: that is four launches of its own)
  const bool bf16_auto = s.dtype == SK_BF16 && g_plan.load(std::memory_order_relaxed) == PLAN_AUTO &&
                         !w.own_colsum && w.z_splits == 1;
  const Plan in_plan = pick_plan(s, SK_OP_BWD_INPUT);
  const int z_tile = bf16_auto ? choose_tile(s.R, tokens, in, 1) : -1;
  const GemmKind du_kind = GEMM_NN_F32_COLSUM;

  void* Z = ws_w;
  float* part = reinterpret_cast<float*>(ws_w + w.z_bytes);
  float* cpart = reinterpret_cast<float*>(ws_w + w.z_bytes + w.part_bytes);
  // Z^T = S_cat^T . x^T (zero-filled row padding)
  GemmArgs z = dense_args(S_cat, s.R, x, in, Z, w.ldz, s.R, tokens, in, 1.0f, nullptr);
  z.n_store = (int)w.ldz;
  // dU (or its slabs) = Z^T . dY with the column sums of dY, the token axis split in order
  GemmArgs du{};
  du.A = Z; du.lda = w.ldz;
  du.B = dY; du.ldb = out; du.ldc = out;
  du.M = s.R; du.N = (int)out; du.K = (int)tokens;
  du.splits = w.splits; du.k_per_split = w.k_per_split;
  if (w.splits == 1) { du.C = dU_cat; du.colsum = dbias; du.scale = scale; }
  else { du.C = part; du.colsum = dbias ? cpart : nullptr; du.scale = 1.0f; }
  ReduceArgs red{};
  red.part = part; red.out = dU_cat; red.n = w.splits > 1 ? (int64_t)s.R * out : 0; red.scale = scale;
  red.part2 = cpart; red.out2 = dbias; red.n2 = (dbias && w.colsum_splits > 1) ? out : 0; red.scale2 = 1.0f;
  red.splits = w.splits; red.splits2 = w.colsum_splits;

  // --- narrow sketch: split-K slabs of G beside Z^T | Z^T.dY | expand dX, carrying the sums ---
  const SketchPlan q = plan_sketch(s, out);
  if (bf16_auto && chain_supported(s.R) && s.R <= 128 && q.splits > 1 && w.splits > 1 &&
      dual_gemm_supported(GEMM_NT_F32, q.tile, GEMM_TT, z_tile)) {
    g_hip_error.clear();
    GemmArgs g = dense_args(dY, out, U_cat, out, ws_in, s.R, tokens, s.R, out, 1.0f, nullptr);
    g.splits = q.splits; g.k_per_split = q.k_per_split;
    hipError_t e = launch_dual_gemm_bf16(GEMM_NT_F32, q.tile, g, GEMM_TT, z_tile, z, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (dY.U^T beside x.S)");
    ChainArgs c{};
    c.A = dY; c.B1 = U_cat; c.B2 = S_cat; c.bias = nullptr; c.C = dX;
    c.lda = out; c.ldb1 = out; c.ldb2 = s.R; c.ldc = in;
    c.M = (int)tokens; c.K1 = (int)out; c.R = s.R; c.N = (int)in; c.scale = scale;
    { const ChainShape cs = chain_shape(tokens, in, s.R, false); c.n_slices = cs.slices; c.bm = cs.bm; }
    c.Z = ws_in; c.z_splits = q.splits; c.z_slab = (int64_t)tokens * s.R;
    // Z^T.dY, then the expansion of dX carrying the sum of the token splits
    e = launch_gemm_bf16(du_kind, w.tile, du, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (Z^T.dY)");
    c.tail = red;
    e = launch_chain_bf16(true, false, c, hs);
    return e == hipSuccess ? SK_OK : hip_fail(e, "sk_linear_bwd (expand + sum of splits)");
  }

  // --- wide sketch (two GEMMs per gradient): dY.U^T beside Z^T | Z^T.dY beside G.S^T | sums ---
  const int g_tile = bf16_auto ? choose_tile(tokens, s.R, out, 1) : -1;
  int dx_tile = bf16_auto ? choose_tile(tokens, in, s.R, 1) : -1;
  // beside Z^T.dY the expansion of dX runs on 128 x 128 tiles even where it would take the
  // eight-wave tile on its own: that one leaves no room on a CU to share (measured at
  // BERT-large: 125 us shared against 133 us one after the other)
  if (dx_tile == TILE_256x256_W8) dx_tile = TILE_128x128;
  if (bf16_auto && in_plan == PLAN_TWO_GEMM && plan_first(tokens, s.R, out).splits == 1 &&
      dual_gemm_supported(GEMM_NT, g_tile, GEMM_TT, z_tile) &&
      dual_gemm_supported(du_kind, w.tile, GEMM_NT, dx_tile)) {
    g_hip_error.clear();
    const GemmArgs g = dense_args(dY, out, U_cat, out, ws_in, s.R, tokens, s.R, out, 1.0f, nullptr);
    hipError_t e = launch_dual_gemm_bf16(GEMM_NT, g_tile, g, GEMM_TT, z_tile, z, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (dY.U^T beside x.S)");
    const GemmArgs dx = dense_args(ws_in, s.R, S_cat, s.R, dX, in, tokens, in, s.R, scale, nullptr);
    e = launch_dual_gemm_bf16(du_kind, w.tile, du, GEMM_NT, dx_tile, dx, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (Z^T.dY beside G.S^T)");
    if (red.n + red.n2 > 0) {
      e = launch_reduce_splits(red, hs);
      if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd (sum of splits)");
    }
    return SK_OK;
  }

  const sk_status a = sk_linear_bwd_input(dY, S_cat, U_cat, dX, tokens, in, out, l, k, dtype, ws_in,
                                          in_bytes, stream);
  if (a != SK_OK) return a;
  return sk_linear_bwd_weight(x, S_cat, dY, dU_cat, dbias, tokens, in, out, l, k, dtype, ws_w, w_bytes,
                              stream);
}

sk_status sk_linear_bwd_weight_first(const void* x, const void* U_cat, const void* dY, float* dA,
                                     int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                                     int64_t col_begin, int64_t col_count, sk_dtype dtype,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !U_cat || !dY || !dA) return SK_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(U_cat) || !aligned16(dY) || !aligned16(dA) || !aligned16(workspace))
    return SK_ERR_INVALID_ARG;
  Shape s;
  const sk_status st = check_shape(tokens, in, out, l, k, dtype, s);
  if (st != SK_OK) return st;
  if (col_begin < 0 || col_count < 16 || col_begin % 16 != 0 || col_count % 16 != 0 ||
      col_begin + col_count > s.R)
    return SK_ERR_INVALID_ARG;
  const int64_t nc = col_count;
  if (!workspace || workspace_bytes < first_stage_bytes(s, nc)) return SK_ERR_WORKSPACE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const float scale = 1.0f / (float)l;
  g_hip_error.clear();

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  void* G = ws;
  float* part = reinterpret_cast<float*>(ws + align_up((size_t)s.T * nc * s.esize));
  const unsigned char* U_sub = static_cast<const unsigned char*>(U_cat) + (size_t)col_begin * out * s.esize;

  // G = dY . U_sub^T, rounded to the storage type like the input gradient's intermediate
  hipError_t e = first_gemm(s, GEMM_NT, GEMM_NT_F32,
                            dense_args(dY, out, U_sub, out, G, nc, tokens, nc, out, 1.0f, nullptr), part, hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight_first (dY.U^T)");

  // dA = scale * x^T . G, the token axis split in order
  const TokenPlan t = plan_tokens(in, nc, tokens, dtype, false);
  GemmArgs a{};
  a.A = x; a.lda = in;
  a.B = G; a.ldb = nc;
  a.ldc = nc;
  a.M = (int)in; a.N = (int)nc; a.K = (int)tokens;
  a.splits = t.splits; a.k_per_split = t.k_per_split;
  a.bias = nullptr; a.colsum = nullptr;
  if (t.splits == 1) { a.C = dA; a.scale = scale; }
  else { a.C = part; a.scale = 1.0f; }
  e = dtype == SK_BF16 ? launch_gemm_bf16(GEMM_TN_F32_PLAIN, t.tile, a, hs)
                       : launch_gemm_f32(GEMM_TN_F32, a, hs);
  if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight_first (x^T.G)");
  if (t.splits > 1) {
    ReduceArgs r{};
    r.part = part; r.out = dA; r.n = (int64_t)in * nc; r.scale = scale;
    r.n2 = 0; r.splits = t.splits; r.splits2 = 1;
    e = launch_reduce_splits(r, hs);
    if (e != hipSuccess) return hip_fail(e, "sk_linear_bwd_weight_first (sum of splits)");
  }
  return SK_OK;
}

}  // extern "C"
