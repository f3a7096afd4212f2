// The "expand" half of SKLinear for small sketch widths (bf16, R <= 512), with the
// R-wide intermediate resident on chip, and optionally the "sketch" half fused in
// front of it:
//
//   C[M, N] = scale * Zt . B2 (+ bias),   Zt = the bf16 R-wide intermediate of a
//   64-token tile, either
//     - computed here:  Zt = bf16(A[64 tokens, K1] . B1)            (FUSED), or
//     - read from the workspace: bf16 [M, R], or the sum of fp32 split-K slabs.
//
// A work-group (256 threads, 4 waves) owns one token tile and one slice of the N
// range.  Zt sits in LDS once and every wave lifts the whole of it into registers
// as MFMA fragments; the waves then split each BN-wide tile of N four ways, so a B2
// fragment is read from LDS by exactly one wave and used for all 32-row blocks.
// Two kernels share that plan:
//   chain_small_kernel (R <= 128, the one the automatic plans use): B2 arrives one whole
//     [R x 128] tile at a time, double buffered across tile boundaries, and output rows
//     leave straight from registers as 16-byte pieces (no LDS re-layout);
//   chain_kernel (R <= 512, forced plans only): B2 streams in 64-row chunks and the output
//     tile is re-laid out through LDS into whole rows.
#include "sk_bf16_tile.h"
#include "sk_launch.h"

namespace sk {

constexpr int CH_BM = 64;

template <int RT, int BN, bool B2_KC, bool FUSED, bool B1_KC>
struct ChainLds {
  typedef OpTile<BN, B2_KC> TB2;
  typedef OpTile<CH_BM, true> TA;
  typedef OpTile<RT, B1_KC> TB1;
  static constexpr int Z_LD = RT + 8;
  static constexpr int Z_BYTES = CH_BM * Z_LD * 2;
  static constexpr int OUT_LD = BN * 2 + 8;                       // bytes per staged output row
  static constexpr int S2_BYTES = 2 * TB2::ELEMS * 2 + CH_BM * OUT_LD;
  static constexpr int S1_BYTES = FUSED ? 2 * (TA::ELEMS + TB1::ELEMS) * 2 : 0;
  static constexpr int BYTES = Z_BYTES + (S1_BYTES > S2_BYTES ? S1_BYTES : S2_BYTES);
};

template <int RT, int BN, bool B2_KC, bool FUSED, bool B1_KC>
__global__ __launch_bounds__(256) void chain_kernel(const ChainArgs p) {
  typedef ChainLds<RT, BN, B2_KC, FUSED, B1_KC> L;
  typedef typename L::TB2 TB2;
  constexpr int KC = RT / 64;            // k chunks of stage 2
  constexpr int WN = BN / 4, TN = WN / 32;
  __shared__ __attribute__((aligned(16))) unsigned char smem[L::BYTES];
  bf16* const Zs = reinterpret_cast<bf16*>(smem);
  unsigned char* const work = smem + L::Z_BYTES;
  bf16* const Bbuf = reinterpret_cast<bf16*>(work);
  unsigned char* const ostage = work + 2 * TB2::ELEMS * 2;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // all slices of one token tile run on the same XCD, so its L2 fetches the tile once
  const int wg = xcd_remap(blockIdx.x, p.tiles_m * p.n_slices);
  const int tile_m = wg / p.n_slices, slice = wg % p.n_slices;
  const int m0 = tile_m * CH_BM;

  // this work-group's run of BN-wide tiles
  const int n_tiles = (p.N + BN - 1) / BN;
  const int per_slice = (n_tiles + p.n_slices - 1) / p.n_slices;
  const int t_begin = slice * per_slice;
  const int t_end = (t_begin + per_slice < n_tiles) ? t_begin + per_slice : n_tiles;
  const int my_tiles = t_end - t_begin;
  if (my_tiles <= 0) return;  // uniform over the work-group

  const bf16* __restrict__ B2 = static_cast<const bf16*>(p.B2);
  uint4 rb[TB2::PIECES];
  // first B2 chunk goes in flight before anything else
  TB2::load(rb, B2, p.ldb2, t_begin * BN, p.N, 0, p.R, p.R, tid);

  // ---------------- the intermediate tile Zt -> LDS ----------------
  if (FUSED) {
    typedef typename L::TA TA;
    typedef typename L::TB1 TB1;
    constexpr int STAGE = TA::ELEMS + TB1::ELEMS;
    constexpr int TN1 = RT / 64;  // waves 2 x 2: each 32 rows x RT/2 columns
    bf16* const s1 = reinterpret_cast<bf16*>(work);
    const bf16* __restrict__ A = static_cast<const bf16*>(p.A);
    const bf16* __restrict__ B1 = static_cast<const bf16*>(p.B1);
    const int wm = wave >> 1, wn = wave & 1;
    f32x16 acc1[TN1];
#pragma unroll
    for (int j = 0; j < TN1; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc1[j][r] = 0.f;
    uint4 ra[TA::PIECES], rb1[TB1::PIECES];
    const int nk = (p.K1 + BK - 1) / BK;
    TA::load(ra, A, p.lda, m0, p.M, 0, p.K1, p.K1, tid);
    TB1::load(rb1, B1, p.ldb1, 0, p.R, 0, p.K1, p.K1, tid);
    TA::store(s1, ra, tid);
    TB1::store(s1 + TA::ELEMS, rb1, tid);
    __syncthreads();
    for (int kc = 0; kc < nk; ++kc) {
      const bf16* As = s1 + (kc & 1) * STAGE;
      const bf16* Bs = As + TA::ELEMS;
      const bool more = kc + 1 < nk;
      if (more) {
        TA::load(ra, A, p.lda, m0, p.M, (kc + 1) * BK, p.K1, p.K1, tid);
        TB1::load(rb1, B1, p.ldb1, 0, p.R, (kc + 1) * BK, p.K1, p.K1, tid);
      }
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        const bf16x8 fa = read_frag<true, TA::LD>(As, wm * 32, ks, lane);
#pragma unroll
        for (int j = 0; j < TN1; ++j) {
          const bf16x8 fb = read_frag<B1_KC, TB1::LD>(Bs, wn * (RT / 2) + j * 32, ks, lane);
          acc1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa, acc1[j], 0, 0, 0);
        }
      }
      if (more) {
        bf16* An = s1 + ((kc + 1) & 1) * STAGE;
        TA::store(An, ra, tid);
        TB1::store(An + TA::ELEMS, rb1, tid);
      }
      __syncthreads();
    }
    // round once to bf16: lane owns row l % 32 and 4 consecutive columns per q
#pragma unroll
    for (int j = 0; j < TN1; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = wn * (RT / 2) + j * 32 + q * 8 + (lane >> 5) * 4;
        uint2 w;
        w.x = pack_bf16x2(acc1[j][q * 4 + 0], acc1[j][q * 4 + 1]);
        w.y = pack_bf16x2(acc1[j][q * 4 + 2], acc1[j][q * 4 + 3]);
        *reinterpret_cast<uint2*>(Zs + (wm * 32 + (lane & 31)) * L::Z_LD + c) = w;
      }
  } else if (p.z_splits == 0) {
    // bf16 [M, R] from the workspace; columns >= R and rows >= M read as zero
    const bf16* __restrict__ Z = static_cast<const bf16*>(p.Z);
    constexpr int PPR = RT / 8;
#pragma unroll
    for (int i = 0; i < (CH_BM * PPR) / 256; ++i) {
      const int piece = i * 256 + tid;
      const int r = piece / PPR, c = (piece % PPR) * 8;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (m0 + r < p.M && c < p.R) v = *reinterpret_cast<const uint4*>(Z + (int64_t)(m0 + r) * p.R + c);
      *reinterpret_cast<uint4*>(Zs + r * L::Z_LD + c) = v;
    }
  } else {
    // sum of fp32 split-K slabs, slabs added in index order, rounded once to bf16
    const float* __restrict__ Zp = static_cast<const float*>(p.Z);
    constexpr int PPR = RT / 4;
#pragma unroll 2
    for (int i = 0; i < (CH_BM * PPR) / 256; ++i) {
      const int piece = i * 256 + tid;
      const int r = piece / PPR, c = (piece % PPR) * 4;
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      if (m0 + r < p.M && c < p.R) {
        const float* src = Zp + (int64_t)(m0 + r) * p.R + c;
        s = *reinterpret_cast<const float4*>(src);
        for (int k = 1; k < p.z_splits; ++k) {
          const float4 v = *reinterpret_cast<const float4*>(src + (int64_t)k * p.z_slab);
          s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
      }
      uint2 w;
      w.x = pack_bf16x2(s.x, s.y);
      w.y = pack_bf16x2(s.z, s.w);
      *reinterpret_cast<uint2*>(Zs + r * L::Z_LD + c) = w;
    }
  }
  __syncthreads();  // Zt complete; stage-1 buffers (aliasing Bbuf) are free

  // every wave lifts all of Zt into registers, in MFMA fragment layout
  bf16x8 fa[2][RT / 16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int ks = 0; ks < RT / 16; ++ks)
      fa[i][ks] = read_frag_rowmajor<L::Z_LD>(Zs, i * 32, ks, lane);

  TB2::store(Bbuf, rb, tid);
  __syncthreads();

  // ---------------- stage 2: stream B2, one BN-wide output tile at a time ----------------
  f32x16 acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16* __restrict__ C = static_cast<bf16*>(p.C);
  const bf16* __restrict__ bias = static_cast<const bf16*>(p.bias);
  const float scale = p.scale;
  const int n_it = my_tiles * KC;
  int it = 0;
  for (int jt = 0; jt < my_tiles; ++jt) {
    const int n0 = (t_begin + jt) * BN;
#pragma unroll
    for (int c = 0; c < KC; ++c, ++it) {
      const bf16* Bs = Bbuf + (it & 1) * TB2::ELEMS;
      const bool more = it + 1 < n_it;
      if (more) {
        const int nn0 = (c + 1 < KC) ? n0 : n0 + BN;
        const int k0 = (c + 1 < KC) ? (c + 1) * 64 : 0;
        TB2::load(rb, B2, p.ldb2, nn0, p.N, k0, p.R, p.R, tid);
      }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const bf16x8 fb = read_frag<B2_KC, TB2::LD>(Bs, wave * WN + j * 32, ks, lane);
#pragma unroll
          for (int i = 0; i < 2; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa[i][c * 4 + ks], acc[i][j], 0, 0, 0);
        }
      }
      if (c == KC - 1) {
        // tile finished: scale, bias, round, re-lay out through LDS, store whole rows
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int cc = wave * WN + j * 32 + q * 8 + (lane >> 5) * 4;  // column in the tile
              float v[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                v[e] = acc[i][j][q * 4 + e] * scale;
                acc[i][j][q * 4 + e] = 0.f;
              }
              if (bias != nullptr && n0 + cc < p.N) {
                const uint2 bb = *reinterpret_cast<const uint2*>(bias + n0 + cc);
                v[0] += bf16_bits_to_float(bb.x & 0xffffu);
                v[1] += bf16_bits_to_float(bb.x >> 16);
                v[2] += bf16_bits_to_float(bb.y & 0xffffu);
                v[3] += bf16_bits_to_float(bb.y >> 16);
              }
              uint2 w;
              w.x = pack_bf16x2(v[0], v[1]);
              w.y = pack_bf16x2(v[2], v[3]);
              *reinterpret_cast<uint2*>(ostage + (i * 32 + (lane & 31)) * L::OUT_LD + cc * 2) = w;
            }
        __syncthreads();
        constexpr int PPR = BN / 4;  // 8-byte pieces per output row
#pragma unroll
        for (int s = 0; s < (CH_BM * PPR) / 256; ++s) {
          const int idx = s * 256 + tid;
          const int r = idx / PPR, pc = idx % PPR;
          const int gm = m0 + r, gn = n0 + pc * 4;
          if (gm < p.M && gn < p.N)
            *reinterpret_cast<uint2*>(C + (int64_t)gm * p.ldc + gn) =
                *reinterpret_cast<const uint2*>(ostage + r * L::OUT_LD + pc * 8);
        }
      }
      if (more) TB2::store(Bbuf + ((it + 1) & 1) * TB2::ELEMS, rb, tid);
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------------------
// Narrow sketches (R <= 128): the same chain, shaped for memory-level parallelism.
// These shapes are bound by bytes and latency, not flops, so the kernel keeps two loads
// in flight per thread at all times (two register sets, prefetch distance two).
//   - The token tile is MB = 64 rows, or 128 when the launcher asks for it (many
//     tokens: half the B2 traffic and LDS reads per MFMA in stage 2).
//   - stage 1 (waves 2 x 2) walks K1 in 64-wide chunks (x chunk + B1 chunk per step);
//   - stage 2 takes B2 one whole [R x 128] tile at a time (no k loop inside a tile).
//     A 64-lane LDS instruction costs the CU about 9 cycles, a transposing read
//     twice that per fragment, so the waves split the tile's columns 1 x 4: every
//     wave holds all rows of Zt in registers and each B2 fragment is read from LDS
//     exactly once.  Output rows leave straight from registers.
//   - In both stages each k step is one scheduling phase: fragment reads of the next
//     step, the step's MFMAs, a share of the global loads of the chunk / tile two
//     ahead and of the LDS stores of the next one.  A wave that issues its loads in
//     one burst waits at the memory pipe's queue while LDS and MFMA idle.
// ---------------------------------------------------------------------------
constexpr int CS_BN = 128;

template <int MB, int RT, bool B2_KC, bool FUSED, bool B1_KC>
struct SmallLds {
  typedef OpTile<CS_BN, B2_KC, RT> TB2;
  typedef OpTile<MB, true> TA;
  typedef OpTile<RT, B1_KC> TB1;
  static constexpr int Z_LD = RT + 8;
  static constexpr int Z_BYTES = MB * Z_LD * 2;
  static constexpr int HEAD_BYTES = Z_BYTES;
  static constexpr int S2_BYTES = 2 * TB2::ELEMS * 2;
  static constexpr int S1_BYTES = FUSED ? 2 * (TA::ELEMS + TB1::ELEMS) * 2 : 0;
  static constexpr int BYTES = HEAD_BYTES + (S1_BYTES > S2_BYTES ? S1_BYTES : S2_BYTES);
};

// Scheduling of one stage-2 tile of the narrow kernel: per k step the fragment reads of
// the next step (ND LDS reads), the step's NM MFMAs, one or two of the KS + 4 global loads
// and one of the KS LDS stores.
template <int KS, int ND, int NM, int I = 0>
__device__ __forceinline__ void sched_stage2() {
  if constexpr (I < KS) {
    if constexpr (I + 1 < KS) __builtin_amdgcn_sched_group_barrier(0x100, ND, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
    __builtin_amdgcn_sched_group_barrier(0x020, I < 4 ? 2 : 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
    sched_stage2<KS, ND, NM, I + 1>();
  } else {
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int MB, int RT, bool B2_KC, bool FUSED, bool B1_KC>
__global__ __launch_bounds__(256) void chain_small_kernel(const ChainArgs p) {
  static_assert(MB == 64 || MB == 128, "token tiles are 64 or 128 rows");
  typedef SmallLds<MB, RT, B2_KC, FUSED, B1_KC> L;
  typedef typename L::TB2 TB2;
  constexpr int KS = RT / 16;
  constexpr int MT = MB / 32;   // 32-row blocks of the token tile (stage 2: all of them in every wave)
  // stage 1: waves 2 x 2, each MB/2 rows x RT/2 columns of Zt (a 1 x 4 grid, with fewer
  // LDS reads per MFMA when B1 is read transposed, measured no faster)
  constexpr int WM1 = MB / 2, WN1 = RT / 2;
  constexpr int TM1 = WM1 / 32, TN1 = WN1 / 32;
  __shared__ __attribute__((aligned(16))) unsigned char smem[L::BYTES];
  bf16* const Zs = reinterpret_cast<bf16*>(smem);
  unsigned char* const work = smem + L::HEAD_BYTES;
  bf16* const Bbuf = reinterpret_cast<bf16*>(work);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;  // stage-1 wave grid
  const int wg = xcd_remap(blockIdx.x, p.tiles_m * p.n_slices);
  const int tile_m = wg / p.n_slices, slice = wg % p.n_slices;
  const int m0 = tile_m * MB;

  const int n_tiles = (p.N + CS_BN - 1) / CS_BN;
  const int per_slice = (n_tiles + p.n_slices - 1) / p.n_slices;
  const int t_begin = slice * per_slice;
  const int t_end = (t_begin + per_slice < n_tiles) ? t_begin + per_slice : n_tiles;
  const int my_tiles = t_end - t_begin;
  // The reduction this launch carries along goes to the work-groups with the least tile
  // work: those of the slices that got fewer tiles than the rest (often none at all, when
  // the tiles do not divide over the slices), or to everybody when all slices are equal.
  const bool has_tail = p.tail.n + p.tail.n2 > 0;
  const int first_light = n_tiles / per_slice;           // slices below this one are full
  const int n_light = p.n_slices - first_light;
  const bool tail_here = has_tail && (n_light == 0 || slice >= first_light);
  const int tail_rank = n_light == 0 ? wg : tile_m * n_light + (slice - first_light);
  const int tail_ranks = p.tiles_m * (n_light == 0 ? p.n_slices : n_light);
  if (my_tiles <= 0) {  // uniform over the work-group
    if (tail_here) reduce_splits_part(p.tail, tail_rank, tail_ranks, tid);
    return;
  }

  const bf16* __restrict__ B2 = static_cast<const bf16*>(p.B2);
  uint4 rb0[TB2::PIECES], rb1[TB2::PIECES];
  // B2 tile jt of this work-group; tiles past its run load as zeros (all lanes masked)
  auto load_b2 = [&](uint4 (&r)[TB2::PIECES], int jt) {
    TB2::load(r, B2, p.ldb2, (t_begin + jt) * CS_BN, jt < my_tiles ? p.N : 0, 0, p.R, p.R, tid);
  };
  // The first two B2 tiles go in flight early: before anything else when the intermediate
  // comes from memory, behind the first two chunks of stage 1 when it is computed here
  // (their 64 KB per work-group would hold up the start of stage 1 by ~0.7 us otherwise).
  if (!FUSED) {
    load_b2(rb0, 0);
    load_b2(rb1, 1);
  }

  // bias through a buffer window of N elements (zero elements when there is no bias:
  // every load then returns zero)
  const GWindow bias_w = make_window(p.bias, 0, p.bias != nullptr ? p.N : 0, 2);
  // this lane's 4 x 4 bias values of tile jt; always fetched one tile ahead of its use
  // (a tile's MFMAs are shorter than a trip to L2)
  auto load_bias = [&](uint2 (&bv)[4], int jt) {
    const int n0 = (t_begin + jt) * CS_BN;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int cc = wave * 32 + q * 8 + (lane >> 5) * 4;
      typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
      const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(bias_w.rsrc, (n0 + cc) * 2, 0, 0);
      bv[q] = make_uint2(v.x, v.y);
    }
  };
  uint2 bv0[4], bv1[4];
  load_bias(bv0, 0);

  // this work-group's share of the carried reduction, while its own first loads are in flight
  if (tail_here) reduce_splits_part(p.tail, tail_rank, tail_ranks, tid);

  // ---------------- the intermediate tile Zt -> LDS ----------------
  if (FUSED) {
    typedef typename L::TA TA;
    typedef typename L::TB1 TB1;
    constexpr int STAGE = TA::ELEMS + TB1::ELEMS;
    bf16* const s1 = reinterpret_cast<bf16*>(work);
    const bf16* __restrict__ A = static_cast<const bf16*>(p.A);
    const bf16* __restrict__ B1 = static_cast<const bf16*>(p.B1);
    f32x16 acc1[TM1][TN1];
#pragma unroll
    for (int i = 0; i < TM1; ++i)
#pragma unroll
      for (int j = 0; j < TN1; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[i][j][r] = 0.f;
    uint4 xa0[TA::PIECES], xb0[TB1::PIECES], xa1[TA::PIECES], xb1[TB1::PIECES];
    const int nk = (p.K1 + BK - 1) / BK;
    // chunks past K1 load as zeros, so the loop needs no branch around its loads
    auto load_a = [&](uint4 (&r)[TA::PIECES], int kc) {
      TA::load(r, A, p.lda, m0, p.M, kc * BK, p.K1, p.K1, tid);
    };
    constexpr int HB = TB1::PIECES / 2;
    auto load_b_lo = [&](uint4 (&r)[TB1::PIECES], int kc) {
      TB1::template load<0, HB>(r, B1, p.ldb1, 0, p.R, kc * BK, p.K1, p.K1, tid);
    };
    auto load_b_hi = [&](uint4 (&r)[TB1::PIECES], int kc) {
      TB1::template load<HB, TB1::PIECES>(r, B1, p.ldb1, 0, p.R, kc * BK, p.K1, p.K1, tid);
    };
    bf16x8 fa0[TM1], fa1[TM1], fb0[TN1], fb1[TN1];
    auto rd = [&](const bf16* As, int ks, bf16x8 (&fa)[TM1], bf16x8 (&fb)[TN1]) {
#pragma unroll
      for (int i = 0; i < TM1; ++i) fa[i] = read_frag<true, TA::LD>(As, wm * WM1 + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TN1; ++j)
        fb[j] = read_frag<B1_KC, TB1::LD>(As + TA::ELEMS, wn * WN1 + j * 32, ks, lane);
    };
    auto mm = [&](const bf16x8 (&fa)[TM1], const bf16x8 (&fb)[TN1]) {
#pragma unroll
      for (int i = 0; i < TM1; ++i)
#pragma unroll
        for (int j = 0; j < TN1; ++j)
          acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc1[i][j], 0, 0, 0);
    };
    // LDS read instructions of one k step: one per x fragment, one (k-contiguous B1) or
    // two (transposing reads) per B1 fragment
    constexpr int NDS = TM1 + TN1 * (B1_KC ? 1 : 2);
    constexpr int NM1 = TM1 * TN1;
    // One chunk: MFMAs on the chunk in `As`, the loads of the chunk two ahead (into la,
    // lb) and the LDS stores of the next chunk (from sa, sb, loaded an iteration ago)
    // spread between them -- issued in one burst the loads hold every wave at the
    // memory pipe's queue while LDS and MFMA sit idle.
    auto iteration = [&](const bf16* As, bf16* An, uint4 (&la)[TA::PIECES], uint4 (&lb)[TB1::PIECES],
                         uint4 (&sa)[TA::PIECES], uint4 (&sb)[TB1::PIECES], int kc_load) {
      rd(As, 0, fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
      rd(As, 1, fa1, fb1);
      load_a(la, kc_load);
      mm(fa0, fb0);
      sched_phase<NM1, NDS, TA::PIECES, 0>();
      rd(As, 2, fa0, fb0);
      load_b_lo(lb, kc_load);
      mm(fa1, fb1);
      sched_phase<NM1, NDS, HB, 0>();
      rd(As, 3, fa1, fb1);
      load_b_hi(lb, kc_load);
      mm(fa0, fb0);
      TA::store(An, sa, tid);
      sched_phase<NM1, NDS, TB1::PIECES - HB, TA::PIECES>();
      mm(fa1, fb1);
      TB1::store(An + TA::ELEMS, sb, tid);
      sched_phase<NM1, 0, 0, TB1::PIECES>();
      __syncthreads();
    };
    load_a(xa0, 0);
    load_b_lo(xb0, 0);
    load_b_hi(xb0, 0);
    load_a(xa1, 1);
    load_b_lo(xb1, 1);
    load_b_hi(xb1, 1);
    load_b2(rb0, 0);
    load_b2(rb1, 1);
    TA::store(s1, xa0, tid);
    TB1::store(s1 + TA::ELEMS, xb0, tid);
    __syncthreads();
    for (int kc = 0; kc < nk; kc += 2) {
      // chunk kc sits in buffer 0; set 1 holds chunk kc + 1 (in flight or landed)
      iteration(s1, s1 + STAGE, xa0, xb0, xa1, xb1, kc + 2);
      iteration(s1 + STAGE, s1, xa1, xb1, xa0, xb0, kc + 3);  // an all-zero chunk when nk is odd
    }
#pragma unroll
    for (int i = 0; i < TM1; ++i)
#pragma unroll
      for (int j = 0; j < TN1; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = wn * WN1 + j * 32 + q * 8 + (lane >> 5) * 4;
          uint2 w;
          w.x = pack_bf16x2(acc1[i][j][q * 4 + 0], acc1[i][j][q * 4 + 1]);
          w.y = pack_bf16x2(acc1[i][j][q * 4 + 2], acc1[i][j][q * 4 + 3]);
          *reinterpret_cast<uint2*>(Zs + (wm * WM1 + i * 32 + (lane & 31)) * L::Z_LD + c) = w;
        }
  } else if (p.z_splits == 0) {
    const bf16* __restrict__ Z = static_cast<const bf16*>(p.Z);
    constexpr int PPR = RT / 8;
#pragma unroll
    for (int i = 0; i < (MB * PPR) / 256; ++i) {
      const int piece = i * 256 + tid;
      const int r = piece / PPR, c = (piece % PPR) * 8;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (m0 + r < p.M && c < p.R) v = *reinterpret_cast<const uint4*>(Z + (int64_t)(m0 + r) * p.R + c);
      *reinterpret_cast<uint4*>(Zs + r * L::Z_LD + c) = v;
    }
  } else {
    // Sum of the fp32 split-K slabs in index order, rounded once to bf16.  The loads
    // are branch free (buffer windows, one per slab; a masked lane reads zero) and go
    // out four slabs x all pieces of the thread at a time, so the whole tile costs one
    // or two trips to memory instead of one per piece.
    const float* __restrict__ Zp = static_cast<const float*>(p.Z);
    constexpr int PPR = RT / 4;
    constexpr int NP = (64 * PPR) / 256;  // pieces of four floats per thread and 64 rows
    constexpr int MAXS = 8, GROUP = 4;
    for (int h = 0; h < MB / 64; ++h) {  // 64 rows at a time: bounds the registers in flight
    unsigned off[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int piece = i * 256 + tid;
      const int r = h * 64 + piece / PPR, c = (piece % PPR) * 4;
      off[i] = c < p.R ? (unsigned)(r * p.R + c) * 4u : OOB_OFFSET;  // rows past M fall outside
    }
    float4 sum[NP];
#pragma unroll
    for (int g = 0; g < MAXS / GROUP; ++g) {
      if (g * GROUP < p.z_splits) {  // uniform
        f32x4 v[GROUP][NP];
#pragma unroll
        for (int k = 0; k < GROUP; ++k) {
          const int sp = g * GROUP + k;
          // slabs past z_splits: an empty window, every lane reads zero
          const int64_t origin = (int64_t)sp * p.z_slab + (int64_t)m0 * p.R;
          const GWindow w = make_window(Zp, origin, sp < p.z_splits ? (int64_t)sp * p.z_slab + (int64_t)p.M * p.R : origin, 4);
#pragma unroll
          for (int i = 0; i < NP; ++i)
            v[k][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(w.rsrc, (int)off[i], 0, 0));
        }
#pragma unroll
        for (int i = 0; i < NP; ++i) {
#pragma unroll
          for (int k = 0; k < GROUP; ++k) {
            if (g == 0 && k == 0) sum[i] = make_float4(v[0][i].x, v[0][i].y, v[0][i].z, v[0][i].w);
            else { sum[i].x += v[k][i].x; sum[i].y += v[k][i].y; sum[i].z += v[k][i].z; sum[i].w += v[k][i].w; }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int piece = i * 256 + tid;
      const int r = h * 64 + piece / PPR, c = (piece % PPR) * 4;
      uint2 w;
      w.x = pack_bf16x2(sum[i].x, sum[i].y);
      w.y = pack_bf16x2(sum[i].z, sum[i].w);
      *reinterpret_cast<uint2*>(Zs + r * L::Z_LD + c) = w;
    }
    }  // h
  }
  __syncthreads();  // Zt complete; stage-1 buffers (aliasing Bbuf) are free

  // all rows of Zt, as MFMA fragments, in every wave for the rest of the kernel
  bf16x8 fa[MT][KS];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fa[i][ks] = read_frag_rowmajor<L::Z_LD>(Zs, i * 32, ks, lane);

  TB2::store(Bbuf, rb0, tid);
  __syncthreads();

  bf16* __restrict__ C = static_cast<bf16*>(p.C);
  const float scale = p.scale;

  // One [MB x 128] output tile (wave w owns columns 32 w .. 32 w + 31 of it) from the B2
  // tile in `Bs`.  Between its MFMAs go the loads of the tile two ahead (into rl), the
  // next tile's bias (into bvn) and the LDS stores of the next tile (from rs, loaded one
  // step ago, into Bn): issued in one burst, the loads hold every wave at the memory
  // pipe's queue while LDS and MFMA sit idle.
  auto step = [&](int jt, const bf16* Bs, bf16* Bn, const uint2 (&bv)[4], uint2 (&bvn)[4],
                  uint4 (&rl)[TB2::PIECES], uint4 (&rs)[TB2::PIECES]) {
    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    bf16x8 fb = read_frag<B2_KC, TB2::LD>(Bs, wave * 32, 0, lane);
    __builtin_amdgcn_sched_barrier(0);
    load_bias(bvn, jt + 1);
    load_b2(rl, jt + 2);
    // (an LDS store may not pass an LDS read in the compiler's eyes, so each k step's
    // store sits where the schedule wants it: after the reads of the step that follows;
    // reading the fragments two steps ahead instead of one measured no faster)
    static_for<0, KS>([&](auto ksc) {
      constexpr int ks = decltype(ksc)::value;
      bf16x8 fbn = fb;
      if (ks + 1 < KS) fbn = read_frag<B2_KC, TB2::LD>(Bs, wave * 32, ks + 1, lane);
#pragma unroll
      for (int i = 0; i < MT; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb, fa[i][ks], acc[i], 0, 0, 0);
      TB2::template store<ks, ks + 1>(Bn, rs, tid);
      fb = fbn;
    });
    sched_stage2<KS, B2_KC ? 1 : 2, MT>();
    // Result rows leave straight from registers.  A lane holds, per 8-column group q, the
    // four columns 8 q + 4 (l / 32) .. +3 of its row; exchanging the upper half-wave's part
    // of an even group with the lower half-wave's part of the odd group next to it
    // (v_permlane32_swap) leaves every lane with eight consecutive columns -- 16 bytes --
    // so no trip through LDS, and no barrier, is needed to form whole pieces.
    const int n0 = (t_begin + jt) * CS_BN + wave * 32;
    const int n_lim = jt < my_tiles ? p.N : 0;
    auto rows_out = [&](const f32x16& acc, int row0) {
      const int gm = m0 + row0 + (lane & 31);
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        uint2 w[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int q = 2 * pr + h;
          const float b0 = bf16_bits_to_float(bv[q].x & 0xffffu), b1 = bf16_bits_to_float(bv[q].x >> 16);
          const float b2 = bf16_bits_to_float(bv[q].y & 0xffffu), b3 = bf16_bits_to_float(bv[q].y >> 16);
          w[h].x = pack_bf16x2(acc[q * 4 + 0] * scale + b0, acc[q * 4 + 1] * scale + b1);
          w[h].y = pack_bf16x2(acc[q * 4 + 2] * scale + b2, acc[q * 4 + 3] * scale + b3);
        }
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(w[0].x, w[1].x, false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(w[0].y, w[1].y, false, false);
        const int gn = n0 + 16 * pr + 8 * (lane >> 5);
        if (gm < p.M && gn < n_lim)
          *reinterpret_cast<uint4*>(C + (int64_t)gm * p.ldc + gn) = make_uint4(s0.x, s1.x, s0.y, s1.y);
      }
    };
#pragma unroll
    for (int i = 0; i < MT; ++i) rows_out(acc[i], i * 32);
    __syncthreads();
  };

  for (int jt = 0; jt < my_tiles; jt += 2) {
    // tile jt sits in buffer 0; set 1 holds tile jt + 1
    step(jt, Bbuf, Bbuf + TB2::ELEMS, bv0, bv1, rb0, rb1);
    // (computes on zeros and stores nothing past the run)
    step(jt + 1, Bbuf + TB2::ELEMS, Bbuf, bv1, bv0, rb1, rb0);
  }
}

bool chain_supported(int R) { return R >= 16 && R <= 512; }

// Flops and bytes of a chain launch: both contractions when the first one is fused in,
// otherwise the second one with the intermediate (or its slabs) read from memory; the
// reduction it may carry along counts by its bytes.
static Work chain_work(const ChainArgs& a, bool fused) {
  Work w;
  w.flops = 2.0 * a.M * a.R * ((fused ? a.K1 : 0) + (double)a.N);
  w.bytes = 2.0 * ((double)a.R * a.N + (double)a.M * a.N) + (a.bias != nullptr ? 2.0 * a.N : 0.0);
  if (fused) w.bytes += 2.0 * ((double)a.M * a.K1 + (double)a.K1 * a.R);
  else w.bytes += (double)a.M * a.R * (a.z_splits == 0 ? 2.0 : 4.0 * a.z_splits);
  w.bytes += reduce_work(a.tail).bytes;
  return w;
}

template <int RT, int BN, bool B2_KC, bool FUSED, bool B1_KC>
static hipError_t launch_one(const ChainArgs& a, hipStream_t s) {
  const long long grid = (long long)a.tiles_m * a.n_slices;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  static const std::string name =
      kernel_label("chain_kernel", {lbl(RT), lbl(BN), lbl(B2_KC), lbl(FUSED), lbl(B1_KC)});
  return launch_kernel(name.c_str(), chain_work(a, FUSED), chain_kernel<RT, BN, B2_KC, FUSED, B1_KC>, dim3((unsigned)grid), dim3(256),
                       s, a);
}

template <int MB, int RT, bool B2_KC, bool FUSED, bool B1_KC>
static hipError_t launch_small_mb(const ChainArgs& a, hipStream_t s) {
  const long long grid = (long long)a.tiles_m * a.n_slices;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  static const std::string name =
      kernel_label("chain_small_kernel", {lbl(MB), lbl(RT), lbl(B2_KC), lbl(FUSED), lbl(B1_KC)});
  return launch_kernel(name.c_str(), chain_work(a, FUSED), chain_small_kernel<MB, RT, B2_KC, FUSED, B1_KC>, dim3((unsigned)grid),
                       dim3(256), s, a);
}

template <int RT, bool B2_KC, bool FUSED, bool B1_KC>
static hipError_t launch_small(const ChainArgs& a, hipStream_t s) {
  return a.bm == 128 ? launch_small_mb<128, RT, B2_KC, FUSED, B1_KC>(a, s)
                     : launch_small_mb<64, RT, B2_KC, FUSED, B1_KC>(a, s);
}

template <bool B_KC, bool FUSED>
static hipError_t launch_rt(const ChainArgs& a, hipStream_t s) {
  constexpr int BN = 128;
  if (a.z_splits > 8) return hipErrorInvalidValue;
  if (a.R <= 64) return launch_small<64, B_KC, FUSED, B_KC>(a, s);
  if (a.R <= 128) return launch_small<128, B_KC, FUSED, B_KC>(a, s);
  if (a.R <= 192) return launch_one<192, BN, B_KC, FUSED, B_KC>(a, s);
  if (a.R <= 256) return launch_one<256, BN, B_KC, FUSED, B_KC>(a, s);
  if (!FUSED) {  // the fused form needs LDS for both stages: R <= 256 only
    if (a.R <= 384) return launch_one<384, BN, B_KC, false, B_KC>(a, s);
    if (a.R <= 512) return launch_one<512, BN, B_KC, false, B_KC>(a, s);
  }
  return hipErrorInvalidValue;
}

int chain_bn(int R) { return R <= 128 ? CS_BN : 128; }

hipError_t launch_chain_bf16(bool b_kc, bool fused, ChainArgs a, hipStream_t s) {
  if (!chain_supported(a.R) || a.n_slices < 1 || (fused && a.R > CHAIN_FUSED_MAX_R))
    return hipErrorInvalidValue;
  if (a.bm == 0) a.bm = CH_BM;
  if (a.bm != CH_BM && !(a.bm == 128 && a.R <= 128)) return hipErrorInvalidValue;
  a.tiles_m = (a.M + a.bm - 1) / a.bm;
  if (tracing()) {
    if (fused) {
      note_matrix(a.A, a.M, a.K1, a.lda, 2, false);
      note_matrix(a.B1, b_kc ? a.R : a.K1, b_kc ? a.K1 : a.R, a.ldb1, 2, false);
    } else if (a.z_splits == 0) {
      note_matrix(a.Z, a.M, a.R, a.R, 2, false);
    } else {   // fp32 slabs [M, R], z_slab elements apart
      note_matrix(a.Z, 1, (int64_t)(a.z_splits - 1) * a.z_slab + (int64_t)a.M * a.R, 0, 4, false);
    }
    note_matrix(a.B2, b_kc ? a.N : a.R, b_kc ? a.R : a.N, a.ldb2, 2, false);
    if (a.bias != nullptr) note_matrix(a.bias, 1, a.N, a.N, 2, false);
    note_matrix(a.C, a.M, a.N, a.ldc, 2, true);
    note_reduce(a.tail);
  }
  if (b_kc) return fused ? launch_rt<true, true>(a, s) : launch_rt<true, false>(a, s);
  return fused ? launch_rt<false, true>(a, s) : launch_rt<false, false>(a, s);
}

}  // namespace sk
