// fp32 GEMM on v_mfma_f32_32x32x2_f32 for gfx950 (storage type SK_F32), the accuracy path
// of the library.  Same contract as the bf16 GEMM.  4 waves as 2 x 2; a wave owns TB x TB
// MFMA blocks of 32 x 32, so the tile is 64 x 64 (TB = 1: small problems) or 128 x 128
// (TB = 2, once those tiles fill the chip: each operand value read from LDS then feeds two
// MFMAs instead of one, which is what the LDS pipe needs to keep up with the matrix
// pipe).  k chunks of 16, LDS double-buffered, the next chunk's global loads in flight
// during the MFMAs of the current one.
//
// Lane layout of v_mfma_f32_32x32x2_f32 (D = P . Q), lane l:
//   P: row l % 32, k = l / 32;   Q: col l % 32, k = l / 32;
//   D: col l % 32, rows 8 * (r / 4) + 4 * (l / 32) + r % 4, r = 0..15.
#include "sk_launch.h"

namespace sk {

// One [BMN x 16] operand chunk, global -> registers (TB float4 per thread), zero outside
// the matrix or the k range, then registers -> LDS stored [k][m or n] with rows LD apart.
template <int TB, bool KC>
struct F32Chunk {
  static constexpr int BMN = 64 * TB;
  static constexpr int LD = BMN + 4;  // 16-byte aligned rows, k rows 4 banks apart
  static __device__ __forceinline__ void load(float4 (&r)[TB], const float* __restrict__ g, int64_t ld,
                                              int e0, int e_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int v = 0; v < TB; ++v) {
      const int q = v * 256 + tid;
      r[v] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (KC) {  // source [ext, K]: 4 consecutive k of one row
        const int e = q >> 2, k4 = (q & 3) * 4;
        if (e0 + e < e_total && k0 + k4 < k_end)
          r[v] = *reinterpret_cast<const float4*>(g + (int64_t)(e0 + e) * ld + k0 + k4);
      } else {   // source [K, ext]: 4 consecutive m/n of one k row
        const int kk = q / (BMN / 4), e4 = (q % (BMN / 4)) * 4;
        if (e0 + e4 < e_total && k0 + kk < k_end)
          r[v] = *reinterpret_cast<const float4*>(g + (int64_t)(k0 + kk) * ld + e0 + e4);
      }
    }
  }
  static __device__ __forceinline__ void store(float* tile, const float4 (&r)[TB], int tid) {
#pragma unroll
    for (int v = 0; v < TB; ++v) {
      const int q = v * 256 + tid;
      if (KC) {  // scattered into 4 LDS rows
        const int e = q >> 2, k4 = (q & 3) * 4;
        tile[(k4 + 0) * LD + e] = r[v].x;
        tile[(k4 + 1) * LD + e] = r[v].y;
        tile[(k4 + 2) * LD + e] = r[v].z;
        tile[(k4 + 3) * LD + e] = r[v].w;
      } else {
        const int kk = q / (BMN / 4), e4 = (q % (BMN / 4)) * 4;
        *reinterpret_cast<float4*>(tile + kk * LD + e4) = r[v];
      }
    }
  }
};

template <int TB, bool A_KC, bool B_KC, bool COLSUM>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs p) {
  typedef F32Chunk<TB, A_KC> CA;
  typedef F32Chunk<TB, B_KC> CB;
  constexpr int BMN = 64 * TB, LD = CA::LD, WT = 32 * TB;  // WT: rows / columns per wave
  __shared__ __attribute__((aligned(16))) float As[2][F32_BK * LD];
  __shared__ __attribute__((aligned(16))) float Bs[2][F32_BK * LD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles = p.tiles_m * p.tiles_n;
  const int id = blockIdx.x;
  const int split = id / tiles;
  const int t = id - split * tiles;
  const int m0 = (t % p.tiles_m) * BMN, n0 = (t / p.tiles_m) * BMN;
  const int k_begin = split * p.k_per_split;
  const int k_end = (k_begin + p.k_per_split < p.K) ? k_begin + p.k_per_split : p.K;
  const float* __restrict__ A = static_cast<const float*>(p.A);
  const float* __restrict__ B = static_cast<const float*>(p.B);

  f32x16 acc[TB][TB], csum[TB];
#pragma unroll
  for (int i = 0; i < TB; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) csum[i][r] = 0.f;
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  }
  const bool do_colsum = COLSUM && p.colsum != nullptr && m0 == 0 && wm == 0;

  float4 ra[TB], rb[TB];
  CA::load(ra, A, p.lda, m0, p.M, k_begin, k_end, tid);
  CB::load(rb, B, p.ldb, n0, p.N, k_begin, k_end, tid);
  CA::store(As[0], ra, tid);
  CB::store(Bs[0], rb, tid);
  __syncthreads();
  int buf = 0;
  for (int k0 = k_begin; k0 < k_end; k0 += F32_BK, buf ^= 1) {
    // the next chunk (zeros past the end of the range) while this one is multiplied
    CA::load(ra, A, p.lda, m0, p.M, k0 + F32_BK, k_end, tid);
    CB::load(rb, B, p.ldb, n0, p.N, k0 + F32_BK, k_end, tid);
    const float* __restrict__ as = As[buf];
    const float* __restrict__ bs = Bs[buf];
#pragma unroll
    for (int ks = 0; ks < F32_BK; ks += 2) {
      float a[TB], b[TB];
#pragma unroll
      for (int i = 0; i < TB; ++i) a[i] = as[(ks + (lane >> 5)) * LD + wm * WT + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < TB; ++j) b[j] = bs[(ks + (lane >> 5)) * LD + wn * WT + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < TB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
      if (COLSUM) {
        if (do_colsum) {
#pragma unroll
          for (int j = 0; j < TB; ++j) csum[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(1.0f, b[j], csum[j], 0, 0, 0);
        }
      }
    }
    CA::store(As[buf ^ 1], ra, tid);
    CB::store(Bs[buf ^ 1], rb, tid);
    __syncthreads();
  }

  float* __restrict__ C = static_cast<float*>(p.C) + (int64_t)split * p.M * p.ldc;
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
#pragma unroll
  for (int j = 0; j < TB; ++j) {
    const int gn = n0 + wn * WT + j * 32 + (lane & 31);
    if (gn < p.N) {
      const float bv = bias != nullptr ? bias[gn] : 0.f;
#pragma unroll
      for (int i = 0; i < TB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int gm = m0 + wm * WT + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (gm < p.M) C[(int64_t)gm * p.ldc + gn] = acc[i][j][r] * p.scale + bv;
        }
      if (COLSUM) {
        if (do_colsum && lane < 32) p.colsum[(int64_t)split * p.N + gn] = csum[j][0];
      }
    }
  }
}

template <bool A_KC, bool B_KC, bool COLSUM>
static hipError_t launch_one(GemmArgs a, hipStream_t s) {
  // 128 x 128 tiles once they give every CU a work-group, 64 x 64 otherwise
  const long long big = (long long)((a.M + 127) / 128) * ((a.N + 127) / 128) * a.splits;
  const int bmn = big >= NUM_CUS ? 128 : F32_BM;
  a.tiles_m = (a.M + bmn - 1) / bmn;
  a.tiles_n = (a.N + bmn - 1) / bmn;
  const long long grid = (long long)a.tiles_m * a.tiles_n * a.splits;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  // (the result is always addressed as slabs [M, ldc], one per k range: one slab when not split)
  note_gemm(a, A_KC, B_KC, 4, 4, true);
  if (bmn == 128) {
    static const std::string name = kernel_label("gemm_f32_kernel", {lbl(2), lbl(A_KC), lbl(B_KC), lbl(COLSUM)});
    return launch_kernel(name.c_str(), gemm_work(a, 4, 4, true), gemm_f32_kernel<2, A_KC, B_KC, COLSUM>, dim3((unsigned)grid), dim3(256), s, a);
  }
  static const std::string name = kernel_label("gemm_f32_kernel", {lbl(1), lbl(A_KC), lbl(B_KC), lbl(COLSUM)});
  return launch_kernel(name.c_str(), gemm_work(a, 4, 4, true), gemm_f32_kernel<1, A_KC, B_KC, COLSUM>, dim3((unsigned)grid), dim3(256), s, a);
}

hipError_t launch_gemm_f32(GemmKind kind, const GemmArgs& a, hipStream_t s) {
  switch (kind) {
    case GEMM_NN: return launch_one<true, false, false>(a, s);
    case GEMM_NT: return launch_one<true, true, false>(a, s);
    case GEMM_TN_F32: return launch_one<false, false, true>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sk
