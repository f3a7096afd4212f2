// Backward pass of SKLinear for narrow sketches (bf16, R <= 32) in one pass over x and dY.
//
// The two gradients contract dY along different axes -- G = dY . U_cat^T over the output
// columns, dU_cat = Z^T . dY over the tokens -- so a kernel that wants each dY tile only
// once has to own whole rows of dY (for G, and through it dX) and leave one partial sum of
// dU_cat per token tile behind.  For a narrow sketch over a layer of moderate width that
// partial sum is small, and this kernel does it: a work-group owns 32 or 64 tokens and
//   1. recomputes its Z tile = x_tile . S_cat (tokens x R; never read from a saved copy):
//      S_cat sits in LDS whole and the four waves split the contraction four ways.  A wave
//      loads its quarter of the x tile as whole 128-byte row segments and turns them into
//      MFMA fragments through an LDS strip of its own, so this stage needs no barrier
//      (fragments fetched straight from global memory -- 16 contiguous bytes per lane, but
//      32 different rows per instruction -- issued four times slower); the four partial
//      tiles meet in LDS and are rounded to bf16 once;
//   2. walks its rows of dY in 128-column chunks, each loaded once and stored in LDS in two
//      layouts (k-contiguous for the product over columns, as it is for the product over
//      tokens), and from every chunk forms
//        - its term of G = dY . U_cat^T (accumulated in registers over all chunks),
//        - the chunk's 128 columns of Z_tile^T . dY_tile, kept in registers,
//        - the chunk's column sums of dY (the bias gradient's term), kept in LDS;
//      after every PASS chunks (and after the last) the registers and the sums are flushed
//      to the token tile's fp32 slab.  The loop itself holds no global store: loads and
//      stores retire through one in-order counter, so a store between the prefetches would
//      make every wait for a chunk a wait for everything issued before that store;
//   3. rounds G to bf16 and expands dX_tile = scale . G . S_cat^T, the S_cat fragments again
//      straight from global memory (rows of S_cat are k-contiguous for this product).
// Every wave does the same work in every stage (no divergent roles), every load that does
// not depend on an earlier stage is issued before the first wait, the LDS reads of a step
// are issued together ahead of its MFMAs, and results leave through wave-private LDS strips
// as whole 128-byte lines.  A second, small kernel sums the token
// tiles' slabs into dU_cat and dbias in a fixed order, so results are bit-reproducible.
#include "sk_bf16_tile.h"
#include "sk_launch.h"

namespace sk {

// NI = 32-token blocks per work-group: a work-group owns TMK = 32 NI tokens (32 or 64).
template <int NI>
struct NarrowLds {
  static constexpr int RT = 32;             // sketch columns the kernel is built for (R <= RT)
  static constexpr int TMK = 32 * NI;       // tokens per work-group
  static constexpr int CW = 128;            // columns of dY per chunk
  // Row stride of the two tiles that are read with the LDS transpose read (S_cat and Z, both
  // [k][R]): 24 dwords modulo 32, so the four k rows a 16-lane group reads (8 dwords each)
  // sit in disjoint banks.
  static constexpr int S_LD = 48;
  static constexpr int S_CAP = 81920;       // bytes reserved for S_cat
  static constexpr int MAX_IN = S_CAP / (2 * S_LD) / 16 * 16;
  static constexpr int S_PIECES = (MAX_IN * (RT / 8) + 255) / 256;   // 16-byte pieces of S_cat per thread
  static constexpr int X_STEPS = ((MAX_IN / 16) + 3) / 4;            // k steps of stage 1 per wave
  static constexpr int X_SUBS = (X_STEPS + 3) / 4;                   // 64-wide sub-tiles of x per wave
  static constexpr int DX_GROUPS = ((MAX_IN + 63) / 64 + 3) / 4;     // 64-column groups of dX per wave
  static constexpr int Z_LD = S_LD;
  static constexpr int G_LD = RT + 8;       // G tile, [tokens][R] row-major (read_frag_rowmajor's padding)
  typedef OpTile<TMK, true, CW, 256> TDK;   // dY chunk, [tokens][columns], columns = k of G
  typedef OpTile<CW, false, TMK, 256> TDN;  // dY chunk, [tokens = k of dU][columns]
  typedef OpTile<RT, true, CW, 256> TU;     // U_cat chunk, [R rows][columns = k of G]
  static constexpr int CHUNK_BYTES = (TDK::ELEMS + TDN::ELEMS + TU::ELEMS) * 2;
  static constexpr int PASS = 8;            // chunks between flushes: PASS x 16 accumulators
  static constexpr int NSET = 4;            // chunks in flight (register sets); divides PASS
  // G = dY . U^T: each of the NI token blocks has KP partial sums over parts of a chunk's
  // columns (one per wave), added when the chunks are done.
  static constexpr int KP = 4 / NI;
  static constexpr int GK = (CW / 16) / KP; // k steps of G per chunk and wave
  // LDS map: Z tile | column sums of a pass | an 8 KB strip per wave (x sub-tiles, then the dU
  // flush, then dX) | work.
  // work: S_cat (stages 0-1); then two chunk buffers, the partial Z tiles on top of the
  // second one (dead before it is first filled); at the end the partial sums of G and G.
  static constexpr int Z_BYTES = TMK * Z_LD * 2;
  static constexpr int DB_BYTES = PASS * CW * 4;
  static constexpr int STRIP_BYTES = 4 * 8192;
  static constexpr int ZPART_OFF = CHUNK_BYTES;
  static constexpr int ZPART_BYTES = 4 * TMK * RT * 4;
  static constexpr int AFTER_S = ZPART_OFF + (ZPART_BYTES > CHUNK_BYTES ? ZPART_BYTES : CHUNK_BYTES);
  static constexpr int WORK_BYTES = S_CAP > AFTER_S ? S_CAP : AFTER_S;
  static constexpr int BYTES = Z_BYTES + DB_BYTES + STRIP_BYTES + WORK_BYTES;
  static constexpr int GX_BYTES = 16384;
  static_assert(BYTES <= 160 * 1024, "over the LDS of a compute unit");
  static_assert((KP - 1) * NI * 64 * 16 * 4 <= GX_BYTES && GX_BYTES + TMK * G_LD * 2 <= WORK_BYTES,
                "stage 3: partial sums of G, G tile");
  static_assert(PASS % NSET == 0 && NSET % 2 == 0, "register sets and LDS buffers rotate with the pass");
  static_assert(TMK * 128 <= 8192 && TMK * 64 * 2 <= 8192, "the wave's strip holds a dX block and an x sub-tile");
};

// The largest `in` whose S_cat fits the kernel's LDS budget for this sketch width.
int narrow_bwd_max_in(int R) { return R <= NarrowLds<2>::RT ? NarrowLds<2>::MAX_IN : 0; }

template <int NI>
__global__ __launch_bounds__(256) void bwd_narrow_kernel(const NarrowBwdArgs p) {
  typedef NarrowLds<NI> L;
  typedef typename L::TDK TDK;
  typedef typename L::TDN TDN;
  typedef typename L::TU TU;
  constexpr int RT = L::RT, TMK = L::TMK;
  constexpr int NSET = L::NSET, PASS = L::PASS, CW = L::CW;
  __shared__ __attribute__((aligned(16))) unsigned char smem[L::BYTES];
  bf16* const Zs = reinterpret_cast<bf16*>(smem);
  float* const dbs = reinterpret_cast<float*>(smem + L::Z_BYTES);
  unsigned char* const work = smem + L::Z_BYTES + L::DB_BYTES + L::STRIP_BYTES;
  bf16* const Ss = reinterpret_cast<bf16*>(work);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned char* const strip = smem + L::Z_BYTES + L::DB_BYTES + wave * 8192;   // this wave's own
  const int tile_m = blockIdx.x;
  const int m0 = tile_m * TMK;

  const bf16* __restrict__ X = static_cast<const bf16*>(p.x);
  const bf16* __restrict__ S = static_cast<const bf16*>(p.S);
  const bf16* __restrict__ DY = static_cast<const bf16*>(p.dY);
  const bf16* __restrict__ U = static_cast<const bf16*>(p.U);
  const GWindow sw = make_window(S, 0, (int64_t)p.K1 * p.R, 2);
  const int n_chunks = (p.N + CW - 1) / CW;

  // ---------------- every independent load, issued before the first barrier ----------------
  // S_cat, whole
  constexpr int PPR = RT / 8;
  const int s_pieces = p.K1 * PPR;
  uint4 sv[L::S_PIECES];
#pragma unroll
  for (int u = 0; u < L::S_PIECES; ++u) {
    const int q = u * 256 + tid;
    const int k = q / PPR, c = (q % PPR) * 8;
    sv[u] = window_load16(sw, (q < s_pieces && c < p.R) ? (unsigned)(k * p.R + c) * 2u : OOB_OFFSET);
  }
  // this wave's quarter of the x tile: 64-wide sub-tiles, whole row segments
  const int steps = p.K1 / 16;
  const int per_wave = (steps + 3) / 4;
  const int s_begin = wave * per_wave;
  const int s_end = (s_begin + per_wave < steps) ? s_begin + per_wave : steps;
  constexpr int XP = TMK * 8 / 64;   // 16-byte pieces of a sub-tile per lane
  uint4 xv[L::X_SUBS][XP];
  {
    const GWindow xw = make_window(X, (int64_t)m0 * p.K1, (int64_t)p.M * p.K1, 2);
#pragma unroll
    for (int t = 0; t < L::X_SUBS; ++t)
#pragma unroll
      for (int u = 0; u < XP; ++u) {
        const int q = u * 64 + lane;
        const int row = q >> 3, k = (s_begin + t * 4) * 16 + (q & 7) * 8;
        // (rows past M fall outside the window by themselves)
        xv[t][u] = window_load16(xw, k < s_end * 16 ? (unsigned)(row * p.K1 + k) * 2u : OOB_OFFSET);
      }
  }
  // the first chunks of dY and U_cat
  uint4 rd[NSET][TDK::PIECES], ru[NSET][TU::PIECES];
  auto load_chunk = [&](uint4 (&d)[TDK::PIECES], uint4 (&u)[TU::PIECES], int c) {
    // chunks past the last load as zeros (every lane masked)
    const int lim = c < n_chunks ? p.N : 0;
    TDK::load(d, DY, p.N, m0, p.M, c * CW, lim, p.N, tid);
    TU::load(u, U, p.N, 0, p.R, c * CW, lim, p.N, tid);
  };

  // ---------------- S_cat -> LDS ----------------
#pragma unroll
  for (int u = 0; u < L::S_PIECES; ++u) {
    const int q = u * 256 + tid;
    const int k = q / PPR, c = (q % PPR) * 8;
    if (q < s_pieces) *reinterpret_cast<uint4*>(Ss + k * L::S_LD + c) = sv[u];
  }
  // (the chunk loads go out only now: a wave issues in order, and S_cat cannot be stored
  // before everything in front of that store has been issued -- about 16 cycles a load)
  static_for<0, NSET>([&](auto j) { load_chunk(rd[j.value], ru[j.value], j.value); });
  __syncthreads();

  // ---------------- stage 1: Z tile, the contraction split over the four waves ----------------
  {
    f32x16 accz[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) accz[i][r] = 0.f;
    bf16* const xt = reinterpret_cast<bf16*>(strip);   // [TMK rows][64 k], pieces swizzled by row
#pragma unroll
    for (int t = 0; t < L::X_SUBS; ++t) {
      if (s_begin + t * 4 >= s_end) break;   // (the loops are sized for the longest input)
#pragma unroll
      for (int u = 0; u < XP; ++u) {
        const int q = u * 64 + lane;
        const int row = q >> 3;
        *reinterpret_cast<uint4*>(xt + row * 64 + kc_piece<64>(row, q & 7) * 8) = xv[t][u];
      }
      bf16x8 fx[4][NI], fb[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        // (past the wave's range the x fragments are zero; any valid k step serves for S_cat)
        const int kg = s_begin + t * 4 + ks < s_end ? s_begin + t * 4 + ks : 0;
        fb[ks] = read_frag<false, L::S_LD>(Ss, 0, kg, lane);
#pragma unroll
        for (int i = 0; i < NI; ++i) fx[ks][i] = read_frag<true, 64>(xt, i * 32, ks, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int i = 0; i < NI; ++i)
          accz[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks], fx[ks][i], accz[i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();   // everybody is done with S_cat: part of its region now takes the partial tiles
    float* const Zpart = reinterpret_cast<float*>(work + L::ZPART_OFF);
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = i * 32 + (lane & 31), col = q * 8 + (lane >> 5) * 4;
        *reinterpret_cast<float4*>(Zpart + (wave * TMK + row) * RT + col) =
            make_float4(accz[i][q * 4 + 0], accz[i][q * 4 + 1], accz[i][q * 4 + 2], accz[i][q * 4 + 3]);
      }
    __syncthreads();
    // the four partial tiles summed in wave order, rounded once to bf16
#pragma unroll
    for (int u = 0; u < (TMK * RT / 4) / 256; ++u) {
      const int q = u * 256 + tid;
      const int row = q / (RT / 4), c = (q % (RT / 4)) * 4;
      float4 s = *reinterpret_cast<const float4*>(Zpart + row * RT + c);
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float4 v = *reinterpret_cast<const float4*>(Zpart + (w * TMK + row) * RT + c);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      uint2 o;
      o.x = pack_bf16x2(s.x, s.y);
      o.y = pack_bf16x2(s.z, s.w);
      *reinterpret_cast<uint2*>(Zs + row * L::Z_LD + c) = o;
    }
  }
  __syncthreads();   // Z tile complete
  constexpr int UK = TMK / 16;   // k steps (tokens) of the dU product
  bf16x8 fz[UK];                 // the Z tile's fragments (rows r, k = tokens) serve every chunk
#pragma unroll
  for (int ks = 0; ks < UK; ++ks) fz[ks] = read_frag<false, L::Z_LD>(Zs, 0, ks, lane);

  // ---------------- stage 2: the rows of dY, one 128-column chunk at a time ----------------
  auto store_chunk = [&](int buf, const uint4 (&d)[TDK::PIECES], const uint4 (&u)[TU::PIECES]) {
    bf16* b = reinterpret_cast<bf16*>(work + buf * L::CHUNK_BYTES);
    TDK::store(b, d, tid);                       // the same pieces in both layouts
    TDN::store(b + TDK::ELEMS, d, tid);
    TU::store(b + TDK::ELEMS + TDN::ELEMS, u, tid);
  };

  // A wave's share of a chunk.
  //   G [TMK tokens x R]: the 32-token block gi over part kp of the chunk's columns (KP
  //   partial sums per block, added at the end);
  //   dU [R x 128 columns]: the 32 columns uc = wave.
  constexpr int GK = L::GK, KP = L::KP;
  const int gi = wave % NI, kp = wave / NI, gk0 = kp * GK;
  const int uc = wave;
  f32x16 accg;
#pragma unroll
  for (int r = 0; r < 16; ++r) accg[r] = 0.f;
  bf16x8 ones;
#pragma unroll
  for (int j = 0; j < 8; ++j) ones[j] = (bf16)1.0f;
  const bool do_colsum = p.db_slabs != nullptr;
  f32x16 accu[PASS];
  const GWindow duw = make_window(p.du_slabs, (int64_t)tile_m * p.R * p.N, ((int64_t)tile_m + 1) * p.R * p.N, 4);

  for (int c0 = 0; c0 < n_chunks; c0 += PASS) {
#pragma unroll
    for (int cp = 0; cp < PASS; ++cp)
#pragma unroll
      for (int r = 0; r < 16; ++r) accu[cp][r] = 0.f;
    // LDS buffers alternate; a register set is reloaded as soon as it has been stored, so
    // NSET - 1 chunks are in flight behind the one being multiplied.  One barrier per chunk:
    // a wave that stores into a buffer has passed the barrier that every wave reaches only
    // after its last read of that buffer.
    static_for<0, PASS>([&](auto cpc) {
      constexpr int cp = cpc.value, set = cp % NSET, buf = cp & 1;
      if (c0 + cp >= n_chunks) return;   // (uniform over the work-group)
      store_chunk(buf, rd[set], ru[set]);
      load_chunk(rd[set], ru[set], c0 + cp + NSET);   // (past the last chunk: every lane masked)
      __syncthreads();
      const bf16* dk = reinterpret_cast<const bf16*>(work + buf * L::CHUNK_BYTES);
      const bf16* dn = dk + TDK::ELEMS;
      const bf16* uk = dn + TDN::ELEMS;
      bf16x8 fa[GK], fb[GK], fd[UK];
#pragma unroll
      for (int ks = 0; ks < GK; ++ks) {
        fa[ks] = read_frag<true, TDK::LD>(dk, gi * 32, gk0 + ks, lane);
        fb[ks] = read_frag<true, TU::LD>(uk, 0, gk0 + ks, lane);
      }
#pragma unroll
      for (int ks = 0; ks < UK; ++ks) fd[ks] = read_frag<false, TDN::LD>(dn, uc * 32, ks, lane);   // columns, k = tokens
      __builtin_amdgcn_sched_barrier(0);
      f32x16 csum;
#pragma unroll
      for (int r = 0; r < 16; ++r) csum[r] = 0.f;
      // three independent accumulation chains, interleaved
#pragma unroll
      for (int ks = 0; ks < (GK > UK ? GK : UK); ++ks) {
        if (ks < GK) accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks], fa[ks], accg, 0, 0, 0);
        if (ks < UK) {
          accu[cp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[ks], fz[ks], accu[cp], 0, 0, 0);
          csum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[ks], ones, csum, 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // every row of csum holds the same column sums; lanes 0 and 32 keep them
      if ((lane & 31) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<float4*>(dbs + cp * CW + uc * 32 + q * 8 + (lane >> 5) * 4) =
              make_float4(csum[q * 4 + 0], csum[q * 4 + 1], csum[q * 4 + 2], csum[q * 4 + 3]);
      }
    });

    // ---- flush the pass: dU blocks through the wave's strip as whole lines, then the sums ----
    // (per block: all four reads first, then four branch-free stores -- rows past R and
    // columns past N are pointed outside the slab's window.  Writing block cp + 1 into a second
    // slot of the strip before block cp is read back measured no faster.)
    static_for<0, PASS>([&](auto cpc) {
      constexpr int cp = cpc.value;
      if (c0 + cp >= n_chunks) return;
      const int col0 = (c0 + cp) * CW + uc * 32;
      const int row = lane & 31;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int piece = q * 2 + (lane >> 5);
        *reinterpret_cast<float4*>(strip + row * 128 + ((piece ^ (row & 7)) * 16)) =
            make_float4(accu[cp][q * 4 + 0], accu[cp][q * 4 + 1], accu[cp][q * 4 + 2], accu[cp][q * 4 + 3]);
      }
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int r = u * 8 + (lane >> 3), piece = lane & 7;
        v[u] = *reinterpret_cast<const uint4*>(strip + r * 128 + ((piece ^ (r & 7)) * 16));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int r = u * 8 + (lane >> 3), gn = col0 + (lane & 7) * 4;
        window_store16(duw, (r < p.R && gn < p.N) ? (unsigned)(r * p.N + gn) * 4u : OOB_OFFSET, v[u]);
      }
    });
    if (do_colsum) {
      __syncthreads();
      for (int q = tid; q < PASS * CW / 4; q += 256) {
        const int gn = c0 * CW + q * 4;
        if (gn < p.N) *reinterpret_cast<float4*>(p.db_slabs + (int64_t)tile_m * p.N + gn) = *reinterpret_cast<const float4*>(dbs + q * 4);
      }
      __syncthreads();
    }
  }

  // ---------------- stage 3: dX tile = scale . G . S_cat^T ----------------
  // A wave takes every fourth group of 64 input columns.  Its S_cat fragments: row n of
  // S_cat, 8 consecutive sketch columns -- 16 contiguous bytes, straight from global
  // memory, all of them requested before G is assembled.
  constexpr int KS = RT / 16;
  const int n_groups = (p.K1 + 63) / 64;
  uint4 fs[L::DX_GROUPS][2][KS];
#pragma unroll
  for (int t = 0; t < L::DX_GROUPS; ++t)
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int g = wave + 4 * t;
        const int n = g * 64 + jb * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
        fs[t][jb][ks] = window_load16(sw, (g < n_groups && n < p.K1 && k < p.R) ? (unsigned)(n * p.R + k) * 2u : OOB_OFFSET);
      }
  // G, rounded to bf16, row-major, once the partial sums of each block are added (in order)
  float* const Gx = reinterpret_cast<float*>(work);                    // [KP - 1][NI blocks][64 lanes][16]
  bf16* const Gs = reinterpret_cast<bf16*>(work + L::GX_BYTES);
  __syncthreads();   // the chunk buffers are idle
  if (kp > 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float4*>(Gx + ((((kp - 1) * NI + gi) * 64 + lane) * 16 + q * 4)) =
          make_float4(accg[q * 4 + 0], accg[q * 4 + 1], accg[q * 4 + 2], accg[q * 4 + 3]);
  }
  __syncthreads();
  if (kp == 0) {
    const int row = gi * 32 + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 a = make_float4(accg[q * 4 + 0], accg[q * 4 + 1], accg[q * 4 + 2], accg[q * 4 + 3]);
#pragma unroll
      for (int k2 = 1; k2 < KP; ++k2) {
        const float4 b = *reinterpret_cast<const float4*>(Gx + ((((k2 - 1) * NI + gi) * 64 + lane) * 16 + q * 4));
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
      }
      const int col = q * 8 + (lane >> 5) * 4;
      uint2 o;
      o.x = pack_bf16x2(a.x, a.y);
      o.y = pack_bf16x2(a.z, a.w);
      *reinterpret_cast<uint2*>(Gs + row * L::G_LD + col) = o;
    }
  }
  __syncthreads();   // G complete
  bf16x8 fg[NI][KS];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fg[i][ks] = read_frag_rowmajor<L::G_LD>(Gs, i * 32, ks, lane);
  const GWindow dxw = make_window(p.dX, (int64_t)m0 * p.K1, (int64_t)p.M * p.K1, 2);
#pragma unroll
  for (int t = 0; t < L::DX_GROUPS; ++t) {
    const int g = wave + 4 * t;
    if (g >= n_groups) break;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fs[t][jb][ks]), fg[i][ks], acc, 0, 0, 0);
        const int row = i * 32 + (lane & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 o;
          o.x = pack_bf16x2(acc[q * 4 + 0] * p.scale, acc[q * 4 + 1] * p.scale);
          o.y = pack_bf16x2(acc[q * 4 + 2] * p.scale, acc[q * 4 + 3] * p.scale);
          const int piece = jb * 4 + q;
          *reinterpret_cast<uint2*>(strip + row * 128 + ((piece ^ (row & 7)) * 16) + (lane >> 5) * 8) = o;
        }
      }
    uint4 v[TMK / 8];
#pragma unroll
    for (int u = 0; u < TMK / 8; ++u) {
      const int row = u * 8 + (lane >> 3), piece = lane & 7;
      v[u] = *reinterpret_cast<const uint4*>(strip + row * 128 + ((piece ^ (row & 7)) * 16));
    }
#pragma unroll
    for (int u = 0; u < TMK / 8; ++u) {
      const int row = u * 8 + (lane >> 3), gn = g * 64 + (lane & 7) * 8;
      // rows past M fall outside the window; columns past the end are pointed there
      window_store16(dxw, gn < p.K1 ? (unsigned)(row * p.K1 + gn) * 2u : OOB_OFFSET, v[u]);
    }
  }
}

// Sum of per-token-tile slabs (both segments of a ReduceArgs) in a fixed order: a work-group
// takes 32 16-byte pieces; eight thread groups each sum every eighth slab in index order
// (up to eight loads in flight per thread), and the eight partial sums are added in group
// order.
__global__ __launch_bounds__(256) void reduce_tiles_kernel(const ReduceArgs p) {
  __shared__ float4 partial[8][32];
  const int pl = threadIdx.x & 31, sg = threadIdx.x >> 5;
  const int64_t n1 = p.n / 4, n2 = p.n2 / 4;
  int64_t q = (int64_t)blockIdx.x * 32 + pl;
  const float* __restrict__ src = p.part;
  float* __restrict__ dst = p.out;
  int64_t n = p.n;
  int splits = p.splits;
  float scale = p.scale;
  bool valid = q < n1 + n2;
  if (q >= n1) { q -= n1; src = p.part2; dst = p.out2; n = p.n2; splits = p.splits2; scale = p.scale2; }
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (valid) {
    for (int k0 = sg; k0 < splits; k0 += 64) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + u * 8;
        v[u] = k < splits ? *reinterpret_cast<const float4*>(src + (int64_t)k * n + q * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
  }
  partial[sg][pl] = s;
  __syncthreads();
  if (sg == 0 && valid) {
#pragma unroll
    for (int g = 1; g < 8; ++g) {
      const float4 v = partial[g][pl];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4*>(dst + q * 4) = make_float4(s.x * scale, s.y * scale, s.z * scale, s.w * scale);
  }
}

hipError_t launch_reduce_tiles(const ReduceArgs& a, hipStream_t s) {
  const int64_t groups = ((a.n + a.n2) / 4 + 31) / 32;
  if (groups <= 0) return hipSuccess;
  if (groups > 0x7fffffffLL || (a.n & 3) || (a.n2 & 3)) return hipErrorInvalidValue;
  note_reduce(a);
  return launch_kernel("reduce_tiles_kernel", reduce_work(a), reduce_tiles_kernel, dim3((unsigned)groups), dim3(256), s, a);
}

hipError_t launch_bwd_narrow_bf16(NarrowBwdArgs a, hipStream_t s) {
  typedef NarrowLds<2> L;
  if (a.R < 16 || a.R > L::RT || a.K1 > L::MAX_IN || a.M < 1 || (a.tm != 32 && a.tm != 64)) return hipErrorInvalidValue;
  a.tiles_m = (a.M + a.tm - 1) / a.tm;
  if (tracing()) {
    note_matrix(a.x, a.M, a.K1, a.K1, 2, false);
    note_matrix(a.S, a.K1, a.R, a.R, 2, false);
    note_matrix(a.dY, a.M, a.N, a.N, 2, false);
    note_matrix(a.U, a.R, a.N, a.N, 2, false);
    note_matrix(a.dX, a.M, a.K1, a.K1, 2, true);
    note_matrix(a.du_slabs, (int64_t)a.tiles_m * a.R, a.N, a.N, 4, true);
    if (a.db_slabs != nullptr) note_matrix(a.db_slabs, a.tiles_m, a.N, a.N, 4, true);
  }
  Work w;
  w.flops = 2.0 * a.M * a.R * (2.0 * a.K1 + 2.0 * a.N);
  w.bytes = 2.0 * ((double)a.M * (2.0 * a.K1 + a.N) + (double)a.R * (a.K1 + a.N)) +
            4.0 * ((double)a.tiles_m * a.R * a.N + (double)a.tiles_m * a.N);
  if (a.tm == 32)
    return launch_kernel("bwd_narrow_kernel<1>", w, bwd_narrow_kernel<1>, dim3((unsigned)a.tiles_m), dim3(256), s, a);
  return launch_kernel("bwd_narrow_kernel<2>", w, bwd_narrow_kernel<2>, dim3((unsigned)a.tiles_m), dim3(256), s, a);
}

}  // namespace sk
