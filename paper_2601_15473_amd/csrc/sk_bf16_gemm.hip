// bf16 MFMA GEMM with fp32 accumulation for gfx950: the contraction every
// two-pass plan of the SKLinear forward/backward is made of.
//
//   C[M, N] = scale * (A . B) (+ bias[n]),   or raw fp32 split-K partial slabs.
//
// One work-group of WAVES_M x WAVES_N waves (2 x 2, or 2 x 4 for the eight-wave
// 256 x 256 tile) owns a BM x BN tile; each wave a (BM/WAVES_M) x (BN/WAVES_N)
// sub-tile of 32x32 MFMA blocks.  Operands go global -> registers -> LDS (double
// buffered, one barrier per 64-wide k chunk) and are read from LDS directly in the
// MFMA fragment layout; operands whose contiguous dimension is not k are read with
// the LDS transpose read.  Results leave straight from registers: fp32 as 16-byte
// pieces, bf16 after a half-wave exchange that gives each lane eight consecutive
// columns (no LDS re-layout).  Eight-wave launches with more tiles than CUs run as a
// crew of one work-group per CU that walks the tiles.
#include "sk_bf16_tile.h"
#include "sk_launch.h"

namespace sk {

// One tile configuration of the GEMM: its work-group size, its LDS footprint and its body
// (the work of one work-group, given the group's index in the launch and LDS of at
// least LDS_BYTES).  The body is a device function so that one launch can carry the
// work-groups of two independent GEMMs (dual_gemm_kernel below).
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT,
          bool COLSUM, int PF>
struct GemmTile {
  static constexpr int NTH = 64 * WAVES_M * WAVES_N;
  typedef OpTile<BM, A_KC, BK, NTH> TA;
  typedef OpTile<BN, B_KC, BK, NTH> TB;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N, TM = WM / 32, TN = WN / 32;
  static constexpr int STAGE = TA::ELEMS + TB::ELEMS;
  static constexpr int LDS_BYTES = 2 * STAGE * 2;
  // bf16 results leave through a wave-private strip of LDS (32 rows of the wave's sub-tile at
  // a time, see the epilogue), carved out of a main buffer that is idle by then.
  static constexpr int WAVE_STRIP = 32 * WN * 2;
  static_assert((NTH / 64) * WAVE_STRIP <= STAGE * 2, "the waves' strips fit one main buffer");
  // stride > 0: the work-group goes on to tiles block + stride, block + 2 stride, ... below
  // `total` (large tiles only), fetching the next tile's first chunk behind the last
  // MFMAs of the current one.
  static __device__ __forceinline__ void run(const GemmArgs& p, int block, unsigned char* smem,
                                             int stride = 0, int total = 0);
};

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT,
          bool COLSUM, int PF>
__device__ __forceinline__ void
GemmTile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, COLSUM, PF>::run(const GemmArgs& p, int block,
                                                                      unsigned char* const smem,
                                                                      const int stride, const int total) {
  bf16* const lds = reinterpret_cast<bf16*>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  const int tiles = p.tiles_m * p.tiles_n;
  // where work-group index `blk` of the launch works
  struct Where {
    int split, tile_m, m0, n0, k_begin, k_end;
  };
  auto locate = [&](int blk) {
    Where w;
    const int id = xcd_remap(blk, tiles * p.splits);
    w.split = id / tiles;
    int tile_n;
    tile_coords(id - w.split * tiles, p.tiles_m, p.tiles_n, w.tile_m, tile_n);
    w.m0 = w.tile_m * BM;
    w.n0 = tile_n * BN;
    w.k_begin = w.split * p.k_per_split;
    w.k_end = (w.k_begin + p.k_per_split < p.K) ? w.k_begin + p.k_per_split : p.K;
    return w;
  };
  Where here = locate(block);
  int chunk = 0;  // chunks done by this work-group: its parity picks the LDS buffer
  for (bool first_tile = true;; first_tile = false) {
  const bool has_next = PF == 1 && stride > 0 && block + stride < total;
  const Where next = has_next ? locate(block + stride) : here;
  const int split = here.split, tile_m = here.tile_m, m0 = here.m0, n0 = here.n0;
  const int k_begin = here.k_begin, k_end = here.k_end;
  const int nk = (k_end - k_begin + BK - 1) / BK;

  const bf16* __restrict__ A = static_cast<const bf16*>(p.A);
  const bf16* __restrict__ B = static_cast<const bf16*>(p.B);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  f32x16 csum[COLSUM ? TN : 1];
  if (COLSUM) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) csum[j][r] = 0.f;
  }
  // Column sums of B ride on the MFMA: an all-ones fragment in place of A's.
  const bool do_colsum = COLSUM && p.colsum != nullptr && tile_m == 0 && wm == 0;
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (bf16)1.0f;

  // One k step (16 wide): fragments of the four steps of a chunk are read one step
  // ahead of the MFMAs that use them (two fragment sets), so LDS latency hides
  // behind the matrix pipe.
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  auto read = [&](const bf16* As, int ks, bf16x8 (&fa)[TM], bf16x8 (&fb)[TN]) {
    const bf16* Bs = As + TA::ELEMS;
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = read_frag<A_KC, TA::LD>(As, wm * WM + i * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = read_frag<B_KC, TB::LD>(Bs, wn * WN + j * 32, ks, lane);
  };
  auto mma = [&](const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    if (COLSUM) {
      if (do_colsum) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          csum[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], ones, csum[j], 0, 0, 0);
      }
    }
  };
  // Work per chunk and thread: NMMA MFMAs per k step, NDSR fragment reads per k step,
  // NVM global loads and as many LDS stores per chunk.  Each k step is one scheduling
  // phase in which the other instructions are spread evenly between the MFMAs
  // (sched_phase), so they issue in the shadow of the matrix pipe instead of in a
  // burst that stalls it (the texture path takes 16 cycles per 16-byte-per-lane load).
  constexpr int NDSR = (A_KC ? TM : 2 * TM) + (B_KC ? TN : 2 * TN);
  constexpr int NMMA = TM * TN;
  constexpr int NVM = TA::PIECES + TB::PIECES;

  // This lane's bias values (four columns per 8-column group of each 32-column block),
  // fetched before the main loop so the epilogue does not wait for them; through a
  // buffer window of N elements (none without a bias), so no lane needs a branch.
  constexpr bool HAS_BIAS = sizeof(OutT) == 2;
  uint2 bias_r[HAS_BIAS ? TN : 1][4];
  if constexpr (HAS_BIAS) {
    const GWindow bias_w = make_window(p.bias, 0, p.bias != nullptr ? p.N : 0, 2);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
        const int gn = n0 + wn * WN + j * 32 + q * 8 + (lane >> 5) * 4;
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(bias_w.rsrc, gn * 2, 0, 0);
        bias_r[j][q] = make_uint2(v.x, v.y);
      }
  }

  // Iteration shape (PF == 1): the global loads of chunk kc + 1 are issued during k
  // step 0 of chunk kc and stored to the other LDS buffer during k step 3.
  // Chunks past the end of the k range load as zeros: no branch around any load.
  if (PF == 1) {
    uint4 ra[TA::PIECES], rb[TB::PIECES];
    if (first_tile) {
      TA::load(ra, A, p.lda, m0, p.M, k_begin, k_end, p.K, tid);
      TB::load(rb, B, p.ldb, n0, p.N, k_begin, k_end, p.K, tid);
      TA::store(lds, ra, tid);
      TB::store(lds + TA::ELEMS, rb, tid);
      __syncthreads();
    }
    for (int kc = 0; kc < nk; ++kc, ++chunk) {
      const bf16* As = lds + (chunk & 1) * STAGE;
      bf16* An = lds + ((chunk + 1) & 1) * STAGE;
      // the chunk fetched during this one: the next of this tile, or, behind the last
      // one, the first of the work-group's next tile
      const bool into_next = has_next && kc + 1 == nk;
      const int lm0 = into_next ? next.m0 : m0, ln0 = into_next ? next.n0 : n0;
      const int k0 = into_next ? next.k_begin : k_begin + (kc + 1) * BK;
      const int lk_end = into_next ? next.k_end : k_end;
      read(As, 0, fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
      // k step 0: MFMAs + fragment reads of step 1 + all loads of the next chunk (issued
      // as early as possible: they are stored to LDS three k steps later)
      read(As, 1, fa1, fb1);
      TA::load(ra, A, p.lda, lm0, p.M, k0, lk_end, p.K, tid);
      TB::load(rb, B, p.ldb, ln0, p.N, k0, lk_end, p.K, tid);
      mma(fa0, fb0);
      sched_phase<NMMA, NDSR, NVM, 0>();
      // k step 1
      read(As, 2, fa0, fb0);
      mma(fa1, fb1);
      sched_phase<NMMA, NDSR, 0, 0>();
      // k step 2
      read(As, 3, fa1, fb1);
      mma(fa0, fb0);
      sched_phase<NMMA, NDSR, 0, 0>();
      // k step 3: MFMAs + LDS stores of the next chunk.  (Stores and barrier one step
      // earlier, with the next chunk's first fragments read behind this step's MFMAs as
      // the small tiles do below, cost the eight-wave tile 5 %: its loads then have
      // two k steps to land instead of three, and the extra live fragments spill.)
      mma(fa1, fb1);
      TA::store(An, ra, tid);
      TB::store(An + TA::ELEMS, rb, tid);
      sched_phase<NMMA, 0, 0, NVM>();
      __syncthreads();
    }
  } else {
    // Small tiles: an iteration is too short to cover a load's latency, so two
    // register sets keep the loads of chunk kc + 2 in flight while chunk kc + 1,
    // loaded one iteration earlier, is stored.  (Four and six sets were measured on the
    // shapes of this layer and were no faster.)
    uint4 ra0[TA::PIECES], rb0[TB::PIECES], ra1[TA::PIECES], rb1[TB::PIECES];
    TA::load(ra0, A, p.lda, m0, p.M, k_begin, k_end, p.K, tid);
    TB::load(rb0, B, p.ldb, n0, p.N, k_begin, k_end, p.K, tid);
    TA::load(ra1, A, p.lda, m0, p.M, k_begin + BK, k_end, p.K, tid);
    TB::load(rb1, B, p.ldb, n0, p.N, k_begin + BK, k_end, p.K, tid);
    TA::store(lds, ra0, tid);
    TB::store(lds + TA::ELEMS, rb0, tid);
    __syncthreads();
    auto iteration = [&](const bf16* As, bf16* An, uint4 (&la)[TA::PIECES], uint4 (&lb)[TB::PIECES],
                         uint4 (&sa)[TA::PIECES], uint4 (&sb)[TB::PIECES], int k0) {
      // loads into (la, lb) for chunk k0, A's during k step 0 and B's during k step 1 (in
      // one burst they hold the waves at the memory pipe's queue; measured 1 % on the
      // [8192 x 1024..4096] shapes); stores from (sa, sb), loaded an iteration ago
      __builtin_amdgcn_sched_barrier(0);
      read(As, 1, fa1, fb1);
      TA::load(la, A, p.lda, m0, p.M, k0, k_end, p.K, tid);
      mma(fa0, fb0);
      sched_phase<NMMA, NDSR, TA::PIECES, 0>();
      read(As, 2, fa0, fb0);
      TB::load(lb, B, p.ldb, n0, p.N, k0, k_end, p.K, tid);
      mma(fa1, fb1);
      TA::store(An, sa, tid);
      sched_phase<NMMA, NDSR, TB::PIECES, TA::PIECES>();
      read(As, 3, fa1, fb1);
      mma(fa0, fb0);
      TB::store(An + TA::ELEMS, sb, tid);
      sched_phase<NMMA, NDSR, 0, TB::PIECES>();
      // the barrier one k step before the end of the chunk: the first fragments of the
      // next chunk come in behind the last step's MFMAs, not behind the barrier
      __syncthreads();
      read(An, 0, fa0, fb0);
      mma(fa1, fb1);
      sched_phase<NMMA, NDSR, 0, 0>();
    };
    read(lds, 0, fa0, fb0);
    for (int kc = 0; kc < nk; kc += 2) {
      iteration(lds, lds + STAGE, ra0, rb0, ra1, rb1, k_begin + (kc + 2) * BK);
      // an all-zero chunk when nk is odd
      iteration(lds + STAGE, lds, ra1, rb1, ra0, rb0, k_begin + (kc + 3) * BK);
    }
  }

  // ---- epilogue: accumulators -> global ----
  // Lane l owns output row l % 32 of each 32-row block and, for q = 0..3, the four
  // columns 8 q + 4 (l / 32) .. +3 of each 32-column block.
  //   fp32: those 16 bytes are stored as they are (32-byte row segments, merged by the L2).
  //   bf16: the two half-waves exchange the halves of neighbouring column groups
  //     (v_permlane32_swap), after which every lane holds eight consecutive columns; the
  //     wave then turns each 32-row block of its sub-tile over through a strip of LDS that
  //     only it touches (no barrier: one wave's LDS operations execute in order), so that
  //     eight consecutive lanes hold one whole row of the sub-tile and a store instruction
  //     writes complete 128-byte lines.  Stored straight from registers the same data left as
  //     32 scattered 32-byte segments per instruction, which the store path takes four
  //     times as long to work through: with the stores switched off the [8192 x 512] .
  //     [512 x 4096] product of BERT-large took 37 us instead of 50, and most of that gap
  //     stayed when the stores went to a cache-resident scratch target instead, i.e. it was
  //     the instructions, not the bytes.  Pieces are XOR-swizzled by row so that neither the
  //     column-wise writes nor the row-wise reads collide on LDS banks.
  OutT* __restrict__ C = static_cast<OutT*>(p.C) +
                         (sizeof(OutT) == 4 ? (int64_t)split * p.M * p.ldc : (int64_t)0);
  const float scale = p.scale;
  const int wn0 = n0 + wn * WN;  // first global column of this wave
  const int n_store = p.n_store > 0 ? p.n_store : p.N;

  if constexpr (sizeof(OutT) == 4) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int gm = m0 + wm * WM + i * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gn = wn0 + j * 32 + q * 8 + (lane >> 5) * 4;
          if (gm < p.M && gn < n_store)
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + (int64_t)gm * p.ldc + gn) =
                make_float4(acc[i][j][q * 4 + 0] * scale, acc[i][j][q * 4 + 1] * scale,
                            acc[i][j][q * 4 + 2] * scale, acc[i][j][q * 4 + 3] * scale);
        }
    }
  } else {
    constexpr int PPRW = WN / 8;        // 16-byte pieces per row of the wave's sub-tile
    constexpr int RPI = 64 / PPRW;      // rows one store instruction covers
    constexpr int ROW_BYTES = WN * 2;
    // The strips live in the main buffer that is idle now.  Large tiles: the one the last
    // chunk was multiplied out of (everybody passed the barrier behind it; the other buffer
    // may already hold the first chunk of the work-group's next tile).  Small tiles: their
    // last k step still read fragments after the loop's last barrier, so one more comes first.
    if constexpr (PF != 1) __syncthreads();
    unsigned char* const strip = smem + (PF == 1 ? ((chunk + 1) & 1) * STAGE * 2 : 0) + wave * WAVE_STRIP;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row_w = lane & 31;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          uint2 w[2];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int q = 2 * pr + h;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e] * scale;
            const uint2 bb = bias_r[j][q];
            v[0] += bf16_bits_to_float(bb.x & 0xffffu);
            v[1] += bf16_bits_to_float(bb.x >> 16);
            v[2] += bf16_bits_to_float(bb.y & 0xffffu);
            v[3] += bf16_bits_to_float(bb.y >> 16);
            w[h].x = pack_bf16x2(v[0], v[1]);
            w[h].y = pack_bf16x2(v[2], v[3]);
          }
          typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
          const u32x2 s0 = __builtin_amdgcn_permlane32_swap(w[0].x, w[1].x, false, false);
          const u32x2 s1 = __builtin_amdgcn_permlane32_swap(w[0].y, w[1].y, false, false);
          // columns j * 32 + 16 pr + 8 (l / 32) .. + 7 of the sub-tile: piece 4 j + 2 pr + l / 32
          const int piece = j * 4 + pr * 2 + (lane >> 5);
          *reinterpret_cast<uint4*>(strip + row_w * ROW_BYTES + ((piece ^ (row_w & (PPRW - 1))) * 16)) =
              make_uint4(s0.x, s1.x, s0.y, s1.y);
        }
#pragma unroll
      for (int r0 = 0; r0 < 32; r0 += RPI) {
        const int row_r = r0 + lane / PPRW, piece = lane % PPRW;
        const uint4 v = *reinterpret_cast<const uint4*>(strip + row_r * ROW_BYTES + ((piece ^ (row_r & (PPRW - 1))) * 16));
        const int gm = m0 + wm * WM + i * 32 + row_r;
        const int gn = wn0 + piece * 8;
        if (gm < p.M && gn < n_store)
          *reinterpret_cast<uint4*>(reinterpret_cast<bf16*>(C) + (int64_t)gm * p.ldc + gn) = v;
      }
    }
  }

  if (COLSUM) {
    // every D column of csum holds the same sums; lanes 0 and 32 write them out
    if (do_colsum && (lane & 31) == 0) {
      float* out = p.colsum + (int64_t)split * p.N;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gn = wn0 + j * 32 + q * 8 + (lane >> 5) * 4;
          if (gn < p.N)
            *reinterpret_cast<float4*>(out + gn) = make_float4(
                csum[j][q * 4 + 0], csum[j][q * 4 + 1], csum[j][q * 4 + 2], csum[j][q * 4 + 3]);
        }
    }
  }

  if (!has_next) break;
  // (the next tile's first chunk will store into the buffer the strips were in)
  if constexpr (sizeof(OutT) == 2) __syncthreads();
  block += stride;
  here = next;
  }  // tiles of this work-group
}

// The large tiles as a fixed crew of work-groups, one per CU, each walking the tiles
// index, index + crew, ...: the first chunk of a work-group's next tile is fetched behind
// the last MFMAs of its current one instead of in a new work-group's prologue.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT,
          bool COLSUM, int PF>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_crew_kernel(const GemmArgs p,
                                                                                 const int total) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, COLSUM, PF> G;
  __shared__ __attribute__((aligned(16))) unsigned char smem[G::LDS_BYTES];
  G::run(p, blockIdx.x, smem, gridDim.x, total);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT,
          bool COLSUM, int PF>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(const GemmArgs p) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, COLSUM, PF> G;
  __shared__ __attribute__((aligned(16))) unsigned char smem[G::LDS_BYTES];
  G::run(p, blockIdx.x, smem);
}

// Two independent GEMMs in one launch: the first `groups_a` work-groups run GA on `a`, the
// rest run GB on `b`.  For small problems a kernel's fixed cost (launch, first trip to
// memory, drain) is as large as its work, and two kernels that do not depend on each
// other can share it; the chip co-schedules both kinds of work-group on every CU.
template <class GA, class GB>
__global__ __launch_bounds__(256) void dual_gemm_kernel(const GemmArgs a, const GemmArgs b,
                                                        const int groups_a) {
  static_assert(GA::NTH == 256 && GB::NTH == 256, "both halves run 256 threads per work-group");
  constexpr int BYTES = GA::LDS_BYTES > GB::LDS_BYTES ? GA::LDS_BYTES : GB::LDS_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[BYTES];
  if ((int)blockIdx.x < groups_a) GA::run(a, blockIdx.x, smem);
  else GB::run(b, (int)blockIdx.x - groups_a, smem);
}

// Sums the split-K slabs in index order; see ReduceArgs.
// (One piece per thread and no bounds test inside the slab loop: as many work-groups as
// pieces allow matters more here than loads per thread.)
__global__ __launch_bounds__(256) void reduce_splits_kernel(const ReduceArgs p) {
  int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const float* __restrict__ part = p.part;
  float* __restrict__ out = p.out;
  int64_t n = p.n;
  float scale = p.scale;
  int splits = p.splits;
  if (i4 >= n) {  // second segment
    i4 -= n;
    part = p.part2; out = p.out2; n = p.n2; scale = p.scale2; splits = p.splits2;
    if (i4 >= n) return;
  }
  float4 s = *reinterpret_cast<const float4*>(part + i4);
#pragma unroll 8
  for (int k = 1; k < splits; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)k * n + i4);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  s.x *= scale; s.y *= scale; s.z *= scale; s.w *= scale;
  *reinterpret_cast<float4*>(out + i4) = s;
}

// Sum of split-K slabs in index order, rounded once to bf16 (an intermediate that the
// next GEMM reads as an operand).
__global__ __launch_bounds__(256) void reduce_to_bf16_kernel(const float* __restrict__ part,
                                                             bf16* __restrict__ out, int64_t n,
                                                             int splits) {
  const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= n) return;
  float4 s = *reinterpret_cast<const float4*>(part + i4);
#pragma unroll 8
  for (int k = 1; k < splits; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)k * n + i4);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  uint2 w;
  w.x = pack_bf16x2(s.x, s.y);
  w.y = pack_bf16x2(s.z, s.w);
  *reinterpret_cast<uint2*>(out + i4) = w;
}

template <typename OutT>
static std::string out_label() { return sizeof(OutT) == 2 ? "bf16" : "float"; }

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT, bool COLSUM>
static hipError_t launch_cfg(GemmArgs a, hipStream_t s) {
  a.tiles_m = (a.M + BM - 1) / BM;
  a.tiles_n = (a.N + BN - 1) / BN;
  const long long grid = (long long)a.tiles_m * a.tiles_n * a.splits;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  note_gemm(a, A_KC, B_KC, 2, sizeof(OutT), sizeof(OutT) == 4);
  // big per-wave tiles have no registers to spare for a second set of loads in flight
  constexpr int PF = (BM * BN / (WAVES_M * WAVES_N) >= 128 * 64) ? 1 : 2;
  const auto params = {lbl(BM), lbl(BN), lbl(WAVES_M), lbl(WAVES_N), lbl(A_KC), lbl(B_KC), out_label<OutT>(),
                       lbl(COLSUM), lbl(PF)};
  if constexpr (PF == 1 && !COLSUM && WAVES_M * WAVES_N == 8) if (grid > NUM_CUS && grid < 0x7fffffffLL - NUM_CUS) {
    // more tiles than CUs: one work-group per CU (the tile's LDS admits no second) walks them
    static const std::string name = kernel_label("gemm_bf16_crew_kernel", params);
    return launch_kernel(name.c_str(), gemm_work(a, 2, sizeof(OutT), sizeof(OutT) == 4), gemm_bf16_crew_kernel<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, COLSUM, PF>,
                         dim3((unsigned)NUM_CUS), dim3(64 * WAVES_M * WAVES_N), s, a, (int)grid);
  }
  static const std::string name = kernel_label("gemm_bf16_kernel", params);
  return launch_kernel(name.c_str(), gemm_work(a, 2, sizeof(OutT), sizeof(OutT) == 4), gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, COLSUM, PF>,
                       dim3((unsigned)grid), dim3(64 * WAVES_M * WAVES_N), s, a);
}

template <bool A_KC, bool B_KC, typename OutT, bool COLSUM>
static hipError_t launch_tiles(int tile, const GemmArgs& a, hipStream_t s) {
  // the 256 x 256 tiles have no registers left for the column sums
  if (COLSUM && (tile == TILE_256x256 || tile == TILE_256x256_W8)) return hipErrorInvalidValue;
  switch (tile) {
    case TILE_256x256: return launch_cfg<256, 256, 2, 2, A_KC, B_KC, OutT, false>(a, s);
    case TILE_128x128: return launch_cfg<128, 128, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_128x64: return launch_cfg<128, 64, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_64x128: return launch_cfg<64, 128, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_64x64: return launch_cfg<64, 64, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_256x128: return launch_cfg<256, 128, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_128x256: return launch_cfg<128, 256, 2, 2, A_KC, B_KC, OutT, COLSUM>(a, s);
    case TILE_256x256_W8: return launch_cfg<256, 256, 2, 4, A_KC, B_KC, OutT, false>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_gemm_bf16(GemmKind kind, int tile, const GemmArgs& a, hipStream_t s) {
  switch (kind) {
    case GEMM_NN: return launch_tiles<true, false, bf16, false>(tile, a, s);
    case GEMM_NT: return launch_tiles<true, true, bf16, false>(tile, a, s);
    case GEMM_TN_F32: return launch_tiles<false, false, float, true>(tile, a, s);
    case GEMM_TN_F32_PLAIN: return launch_tiles<false, false, float, false>(tile, a, s);
    case GEMM_NN_F32: return launch_tiles<true, false, float, false>(tile, a, s);
    case GEMM_TT: return launch_tiles<false, true, bf16, false>(tile, a, s);
    case GEMM_NN_F32_COLSUM: return launch_tiles<true, false, float, true>(tile, a, s);
    case GEMM_NT_F32: return launch_tiles<true, true, float, false>(tile, a, s);
    case GEMM_TT_F32: return launch_tiles<false, true, float, false>(tile, a, s);
    default: return hipErrorInvalidValue;
  }
}

// Column sums of a dense row-major bf16 matrix [rows, cols] in fp32, the row range cut
// into `splits` runs of rows_per_split (out[s][c] = sum of rows of run s; fixed order).
// One work-group owns 512 columns of one run: a wave reads one whole 1 KB row segment
// per instruction (lane = 8 columns), the four waves stride over the rows, and their
// four partial sums meet in LDS and are added in wave order.
constexpr int COLSUM_COLS = 512;
// The work of one work-group of NW waves at grid position (bx, by); `part` is NW rows of
// COLSUM_COLS + 8 floats of LDS.
template <int NW>
__device__ __forceinline__ void colsum_body(const unsigned short* __restrict__ in, float* __restrict__ out,
                                            int rows, int cols, int rows_per_split, int bx, int by,
                                            float* part) {
  constexpr int PLD = COLSUM_COLS + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = bx * COLSUM_COLS + lane * 8;
  const int r_begin = by * rows_per_split;
  const int r_end = (r_begin + rows_per_split < rows) ? r_begin + rows_per_split : rows;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c < cols) {
#pragma unroll 8
    for (int r = r_begin + wave; r < r_end; r += NW) {
      const uint4 v = *reinterpret_cast<const uint4*>(in + (int64_t)r * cols + c);
      const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += __builtin_bit_cast(float, w[e] << 16);
        acc[2 * e + 1] += __builtin_bit_cast(float, w[e] & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[wave * PLD + lane * 8 + e] = acc[e];
  __syncthreads();
  for (int i = tid; i < COLSUM_COLS; i += 64 * NW) {
    const int gc = bx * COLSUM_COLS + i;
    if (gc < cols) {
      float s = part[i];
#pragma unroll
      for (int w = 1; w < NW; ++w) s += part[w * PLD + i];   // in wave order
      out[(int64_t)by * cols + gc] = s;
    }
  }
}

__global__ __launch_bounds__(256) void colsum_bf16_kernel(const unsigned short* __restrict__ in,
                                                          float* __restrict__ out, int rows,
                                                          int cols, int rows_per_split) {
  __shared__ float part[4 * (COLSUM_COLS + 8)];
  colsum_body<4>(in, out, rows, cols, rows_per_split, blockIdx.x, blockIdx.y, part);
}

// An eight-wave GEMM launch that does not fill the chip, with the column sums riding
// along: work-groups past the GEMM's own run the column-sum body (eight waves each) on
// the CUs the GEMM leaves free -- one streams from HBM while the other multiplies.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, typename OutT, int PF>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_with_colsum_kernel(
    const GemmArgs p, const int gemm_groups, const ColsumArgs c) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, OutT, false, PF> G;
  static_assert(G::NTH == 512, "the column-sum body here runs eight waves");
  static_assert(G::LDS_BYTES >= 8 * (COLSUM_COLS + 8) * 4, "LDS of the GEMM tile covers the partial sums");
  __shared__ __attribute__((aligned(16))) unsigned char smem[G::LDS_BYTES];
  if ((int)blockIdx.x < gemm_groups) {
    G::run(p, blockIdx.x, smem);
  } else {
    const int w = blockIdx.x - gemm_groups;
    colsum_body<8>(static_cast<const unsigned short*>(c.in), c.out, c.rows, c.cols, c.rows_per_split,
                   w % c.col_groups, w / c.col_groups, reinterpret_cast<float*>(smem));
  }
}

namespace {
// The pairs of (kind, tile) the dual kernel is built for: the ones the backward pass's
// plans produce on the benchmark shapes.  `first` should be the longer-running GEMM: its
// work-groups are dispatched first and the other's fill in beside them.
struct DualPair { GemmKind ka; int ta; GemmKind kb; int tb; };
const DualPair kDualPairs[] = {
    {GEMM_NT_F32, TILE_64x128, GEMM_TT, TILE_64x64},           // narrow sketch, R in 65..128
    {GEMM_NT_F32, TILE_64x64, GEMM_TT, TILE_64x64},            // narrow sketch, R <= 64
    {GEMM_NT, TILE_128x128, GEMM_TT, TILE_128x128},            // wide sketch: dY.U^T beside Z^T
    {GEMM_NN_F32_COLSUM, TILE_128x64, GEMM_NT, TILE_128x128},  // wide sketch: Z^T.dY beside G.S^T
    {GEMM_NN_F32_COLSUM, TILE_128x128, GEMM_NT, TILE_128x128},
    {GEMM_NT, TILE_64x64, GEMM_TT, TILE_64x64},                // R = 256..384 at BERT-base width
    {GEMM_NN_F32_COLSUM, TILE_128x64, GEMM_NT, TILE_128x64},
};
int dual_pair_index(GemmKind ka, int ta, GemmKind kb, int tb) {
  for (int i = 0; i < (int)(sizeof(kDualPairs) / sizeof(kDualPairs[0])); ++i)
    if (kDualPairs[i].ka == ka && kDualPairs[i].ta == ta && kDualPairs[i].kb == kb && kDualPairs[i].tb == tb)
      return i;
  return -1;
}
}  // namespace

bool dual_gemm_supported(GemmKind kind_a, int tile_a, GemmKind kind_b, int tile_b) {
  return dual_pair_index(kind_a, tile_a, kind_b, tile_b) >= 0;
}

hipError_t launch_dual_gemm_bf16(GemmKind kind_a, int tile_a, GemmArgs a, GemmKind kind_b, int tile_b,
                                 GemmArgs b, hipStream_t s) {
  const int pair = dual_pair_index(kind_a, tile_a, kind_b, tile_b);
  if (pair < 0) return hipErrorInvalidValue;
  int bm, bn;
  tile_dims(tile_a, bm, bn);
  a.tiles_m = (a.M + bm - 1) / bm;
  a.tiles_n = (a.N + bn - 1) / bn;
  tile_dims(tile_b, bm, bn);
  b.tiles_m = (b.M + bm - 1) / bm;
  b.tiles_n = (b.N + bn - 1) / bn;
  const long long ga = (long long)a.tiles_m * a.tiles_n * a.splits;
  const long long gb = (long long)b.tiles_m * b.tiles_n * b.splits;
  if (ga <= 0 || gb <= 0 || ga + gb > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)(ga + gb)), block(256);
  Work work;
  {
    bool akc, bkc, f32;
    gemm_kind_traits(kind_a, akc, bkc, f32);
    note_gemm(a, akc, bkc, 2, f32 ? 4 : 2, f32);
    work = gemm_work(a, 2, f32 ? 4 : 2, f32);
    gemm_kind_traits(kind_b, akc, bkc, f32);
    note_gemm(b, akc, bkc, 2, f32 ? 4 : 2, f32);
    const Work wb = gemm_work(b, 2, f32 ? 4 : 2, f32);
    work.flops += wb.flops;
    work.bytes += wb.bytes;
  }
  typedef GemmTile<64, 128, 2, 2, true, true, float, false, 2> NTF_64x128;
  typedef GemmTile<64, 64, 2, 2, true, true, float, false, 2> NTF_64x64;
  typedef GemmTile<64, 64, 2, 2, false, true, bf16, false, 2> TT_64x64;
  typedef GemmTile<128, 128, 2, 2, true, true, bf16, false, 2> NT_128x128;
  typedef GemmTile<128, 128, 2, 2, false, true, bf16, false, 2> TT_128x128;
  typedef GemmTile<128, 64, 2, 2, true, false, float, true, 2> NNFC_128x64;
  typedef GemmTile<128, 128, 2, 2, true, false, float, true, 2> NNFC_128x128;
  typedef GemmTile<64, 64, 2, 2, true, true, bf16, false, 2> NT_64x64;
  typedef GemmTile<128, 64, 2, 2, true, true, bf16, false, 2> NT_128x64;
  const char* name = "dual_gemm_kernel";
  switch (pair) {
    case 0: return launch_kernel(name, work, dual_gemm_kernel<NTF_64x128, TT_64x64>, grid, block, s, a, b, (int)ga);
    case 1: return launch_kernel(name, work, dual_gemm_kernel<NTF_64x64, TT_64x64>, grid, block, s, a, b, (int)ga);
    case 2: return launch_kernel(name, work, dual_gemm_kernel<NT_128x128, TT_128x128>, grid, block, s, a, b, (int)ga);
    case 3: return launch_kernel(name, work, dual_gemm_kernel<NNFC_128x64, NT_128x128>, grid, block, s, a, b, (int)ga);
    case 4: return launch_kernel(name, work, dual_gemm_kernel<NNFC_128x128, NT_128x128>, grid, block, s, a, b, (int)ga);
    case 5: return launch_kernel(name, work, dual_gemm_kernel<NT_64x64, TT_64x64>, grid, block, s, a, b, (int)ga);
    case 6: return launch_kernel(name, work, dual_gemm_kernel<NNFC_128x64, NT_128x64>, grid, block, s, a, b, (int)ga);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_gemm_f32slabs_with_colsum(int tile, GemmArgs a, const void* in, float* out, int rows,
                                            int cols, int splits, int rows_per_split, hipStream_t s) {
  if (tile != TILE_256x256_W8) return hipErrorInvalidValue;
  a.tiles_m = (a.M + 255) / 256;
  a.tiles_n = (a.N + 255) / 256;
  ColsumArgs c;
  c.in = in; c.out = out; c.rows = rows; c.cols = cols; c.rows_per_split = rows_per_split;
  c.col_groups = (cols + COLSUM_COLS - 1) / COLSUM_COLS;
  const long long gg = (long long)a.tiles_m * a.tiles_n * a.splits;
  const long long grid = gg + (long long)c.col_groups * splits;
  if (gg <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  note_gemm(a, true, false, 2, 4, true);
  note_matrix(in, rows, cols, cols, 2, false);
  note_matrix(out, splits, cols, cols, 4, true);
  Work work = gemm_work(a, 2, 4, true);
  work.bytes += (double)rows * cols * 2 + (double)splits * cols * 4;
  return launch_kernel("gemm_bf16_with_colsum_kernel<256, 256, 2, 4, true, false, float, 1>", work,
                       gemm_bf16_with_colsum_kernel<256, 256, 2, 4, true, false, float, 1>,
                       dim3((unsigned)grid), dim3(512), s, a, (int)gg, c);
}

hipError_t launch_colsum_bf16(const void* in, float* out, int rows, int cols, int splits,
                              int rows_per_split, hipStream_t s) {
  const dim3 grid((unsigned)((cols + COLSUM_COLS - 1) / COLSUM_COLS), (unsigned)splits);
  note_matrix(in, rows, cols, cols, 2, false);
  note_matrix(out, splits, cols, cols, 4, true);
  return launch_kernel("colsum_bf16_kernel", Work{0.0, (double)rows * cols * 2 + (double)splits * cols * 4},
                       colsum_bf16_kernel, grid, dim3(256), s,
                       static_cast<const unsigned short*>(in), out, rows, cols, rows_per_split);
}

__global__ __launch_bounds__(256) void reduce_splits_2d_kernel(const float* __restrict__ part,
                                                               float* __restrict__ out, int rows, int cols,
                                                               int64_t ld_out, int splits, float scale) {
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  const int r = blockIdx.y;
  if (c >= cols) return;
  const int64_t n = (int64_t)rows * cols, at = (int64_t)r * cols + c;
  float4 s = *reinterpret_cast<const float4*>(part + at);
#pragma unroll 8
  for (int k = 1; k < splits; ++k) {
    const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)k * n + at);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  *reinterpret_cast<float4*>(out + (int64_t)r * ld_out + c) =
      make_float4(s.x * scale, s.y * scale, s.z * scale, s.w * scale);
}

hipError_t launch_reduce_splits_2d(const float* part, float* out, int rows, int cols, int64_t ld_out,
                                   int splits, float scale, hipStream_t s) {
  if (rows < 1 || rows > 65535 || cols < 4 || (cols & 3) != 0 || splits < 1) return hipErrorInvalidValue;
  const dim3 grid((unsigned)((cols / 4 + 255) / 256), (unsigned)rows);
  note_matrix(part, (int64_t)splits * rows, cols, cols, 4, false);
  note_matrix(out, rows, cols, ld_out, 4, true);
  return launch_kernel("reduce_splits_2d_kernel", Work{0.0, 4.0 * rows * cols * (splits + 1)}, reduce_splits_2d_kernel, grid, dim3(256), s, part, out, rows,
                       cols, ld_out, splits, scale);
}

hipError_t launch_reduce_to_bf16(const float* part, void* out, int64_t n, int splits, hipStream_t s) {
  if (n <= 0 || (n & 3) != 0 || splits < 1) return hipErrorInvalidValue;
  const int64_t groups = (n / 4 + 255) / 256;
  if (groups > 0x7fffffffLL) return hipErrorInvalidValue;
  note_matrix(part, splits, n, n, 4, false);
  note_matrix(out, 1, n, n, 2, true);
  return launch_kernel("reduce_to_bf16_kernel", Work{0.0, (double)n * (4.0 * splits + 2.0)}, reduce_to_bf16_kernel, dim3((unsigned)groups), dim3(256), s,
                       part, static_cast<bf16*>(out), n, splits);
}

hipError_t launch_reduce_splits(const ReduceArgs& a, hipStream_t s) {
  const int64_t groups = ((a.n + a.n2) / 4 + 255) / 256;
  if (groups <= 0) return hipSuccess;
  note_reduce(a);
  return launch_kernel("reduce_splits_kernel", reduce_work(a), reduce_splits_kernel, dim3((unsigned)groups), dim3(256), s, a);
}

}  // namespace sk
