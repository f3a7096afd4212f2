// fp32 GEMM on v_mfma_f32_32x32x2_f32 for gfx950 (storage type SK_F32).
// Same contract as the bf16 GEMM; one tile shape (64 x 64 x 16), 4 waves as
// 2 x 2, each wave one 32 x 32 MFMA block.  fp32 is the accuracy path of the
// library (small parity workloads), so it is kept simple: single-buffered LDS.
//
// Lane layout of v_mfma_f32_32x32x2_f32 (D = P . Q), lane l:
//   P: row l % 32, k = l / 32;   Q: col l % 32, k = l / 32;
//   D: col l % 32, rows 8 * (r / 4) + 4 * (l / 32) + r % 4, r = 0..15.
#include "sk_launch.h"

namespace sk {

constexpr int F32_LD = F32_BM + 4;  // 272-byte rows: 16-byte aligned, k rows 16 banks apart

// One 64 x 16 operand chunk: global -> LDS stored [k][m or n].
template <bool KC>
__device__ __forceinline__ void f32_stage(float* tile, const float* __restrict__ g, int64_t ld,
                                          int e0, int e_total, int k0, int k_end, int tid) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (KC) {  // source [ext, K]: 4 consecutive k of one row, scattered into 4 LDS rows
    const int e = tid >> 2, k4 = (tid & 3) * 4;
    if (e0 + e < e_total && k0 + k4 < k_end)
      v = *reinterpret_cast<const float4*>(g + (int64_t)(e0 + e) * ld + k0 + k4);
    tile[(k4 + 0) * F32_LD + e] = v.x;
    tile[(k4 + 1) * F32_LD + e] = v.y;
    tile[(k4 + 2) * F32_LD + e] = v.z;
    tile[(k4 + 3) * F32_LD + e] = v.w;
  } else {   // source [K, ext]: 4 consecutive m/n of one k row
    const int kk = tid >> 4, e4 = (tid & 15) * 4;
    if (e0 + e4 < e_total && k0 + kk < k_end)
      v = *reinterpret_cast<const float4*>(g + (int64_t)(k0 + kk) * ld + e0 + e4);
    *reinterpret_cast<float4*>(tile + kk * F32_LD + e4) = v;
  }
}

template <bool A_KC, bool B_KC, bool COLSUM>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs p) {
  __shared__ __attribute__((aligned(16))) float As[F32_BK * F32_LD];
  __shared__ __attribute__((aligned(16))) float Bs[F32_BK * F32_LD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles = p.tiles_m * p.tiles_n;
  const int id = blockIdx.x;
  const int split = id / tiles;
  const int t = id - split * tiles;
  const int m0 = (t % p.tiles_m) * F32_BM, n0 = (t / p.tiles_m) * F32_BN;
  const int k_begin = split * p.k_per_split;
  const int k_end = (k_begin + p.k_per_split < p.K) ? k_begin + p.k_per_split : p.K;
  const float* __restrict__ A = static_cast<const float*>(p.A);
  const float* __restrict__ B = static_cast<const float*>(p.B);

  f32x16 acc, csum;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[r] = 0.f; csum[r] = 0.f; }
  const bool do_colsum = COLSUM && p.colsum != nullptr && m0 == 0 && wm == 0;

  for (int k0 = k_begin; k0 < k_end; k0 += F32_BK) {
    f32_stage<A_KC>(As, A, p.lda, m0, p.M, k0, k_end, tid);
    f32_stage<B_KC>(Bs, B, p.ldb, n0, p.N, k0, k_end, tid);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < F32_BK; ks += 2) {
      const float a = As[(ks + (lane >> 5)) * F32_LD + wm * 32 + (lane & 31)];
      const float b = Bs[(ks + (lane >> 5)) * F32_LD + wn * 32 + (lane & 31)];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
      if (COLSUM) {
        if (do_colsum) csum = __builtin_amdgcn_mfma_f32_32x32x2f32(1.0f, b, csum, 0, 0, 0);
      }
    }
    __syncthreads();
  }

  float* __restrict__ C = static_cast<float*>(p.C) + (int64_t)split * p.M * p.ldc;
  const float* __restrict__ bias = static_cast<const float*>(p.bias);
  const int gn = n0 + wn * 32 + (lane & 31);
  if (gn < p.N) {
    const float bv = bias != nullptr ? bias[gn] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int gm = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (gm < p.M) C[(int64_t)gm * p.ldc + gn] = acc[r] * p.scale + bv;
    }
    if (COLSUM) {
      if (do_colsum && lane < 32) p.colsum[(int64_t)split * p.N + gn] = csum[0];
    }
  }
}

template <bool A_KC, bool B_KC, bool COLSUM>
static hipError_t launch_one(GemmArgs a, hipStream_t s) {
  a.tiles_m = (a.M + F32_BM - 1) / F32_BM;
  a.tiles_n = (a.N + F32_BN - 1) / F32_BN;
  const long long grid = (long long)a.tiles_m * a.tiles_n * a.splits;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((gemm_f32_kernel<A_KC, B_KC, COLSUM>), dim3((unsigned)grid), dim3(256), 0, s, a);
  return hipGetLastError();
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
