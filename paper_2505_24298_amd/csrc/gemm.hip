// bf16 x bf16 -> float32 GEMM on the gfx950 matrix cores.
//   C[M,N] (+)= A[M,K] * W[N,K]^T      (both operands K-contiguous)
// Work-group tile BM x BN x 64 staged through LDS with register prefetch of
// the next K-slab; four wavefronts in a 2 x 2 grid, each computing
// (BM/2) x (BN/2) with v_mfma_f32_32x32x16_bf16.
#include "kernels.hpp"

namespace areal {

namespace {

constexpr int BK = 64;
constexpr int LDS_K = BK + 8;   // row stride in elements (144 B): conflict-free 16-B reads

// Row `b` of the W tile -> pointer to that row of the (segmented) weight, or
// null when it lies outside the matrix.
template <int BN, int MODE>
__device__ __forceinline__ const bf16* w_row_ptr(const GemmW& W, int tile_n, int b, int N, int K) {
  if (MODE == GEMM_SWIGLU_BF16) {
    // the wave column owns BN/2 tile rows: first half gate rows, second half up rows
    const int wn = b / (BN / 2), rb = b % (BN / 2);
    const int isup = rb / (BN / 4), c = rb % (BN / 4);
    const int f = tile_n * (BN / 2) + wn * (BN / 4) + c;
    return f < N ? W.ptr[isup] + (int64_t)f * K : nullptr;
  } else {
    const int n = tile_n * BN + b;
    if (n >= N) return nullptr;
    if (n < W.end[0]) return W.ptr[0] + (int64_t)n * K;
    if (n < W.end[1]) return W.ptr[1] + (int64_t)(n - W.end[0]) * K;
    return W.ptr[2] + (int64_t)(n - W.end[1]) * K;
  }
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

template <int BM, int BN, int MODE>
__global__ __launch_bounds__(256) void gemm_kernel(const bf16* __restrict__ A, GemmW W,
                                                   void* __restrict__ Cv, int M, int N, int K,
                                                   int ldc) {
  constexpr int TM = BM / 64, TN = BN / 64;      // 32x32 MFMA tiles per wave
  constexpr int ACH = BM / 32, BCH = BN / 32;    // 16-B chunks per thread per slab
  __shared__ __attribute__((aligned(16))) bf16 sA[2][BM * LDS_K];
  __shared__ __attribute__((aligned(16))) bf16 sB[2][BN * LDS_K];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile_n = blockIdx.x, m0 = blockIdx.y * BM;
  const int kc = tid & 7, r0 = tid >> 3;         // chunk column, first chunk row

  const bf16* pa[ACH];
  const bf16* pb[BCH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int m = m0 + r0 + 32 * i;
    pa[i] = m < M ? A + (int64_t)m * K + kc * 8 : nullptr;
  }
#pragma unroll
  for (int i = 0; i < BCH; ++i) {
    const bf16* p = w_row_ptr<BN, MODE>(W, tile_n, r0 + 32 * i, N, K);
    pb[i] = p ? p + kc * 8 : nullptr;
  }

  bf16x8 ra[ACH], rb[BCH];
  const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto load_slab = [&](int k0) {
    const bool kin = k0 + kc * 8 < K;            // K % 8 == 0: a chunk is all in or all out
#pragma unroll
    for (int i = 0; i < ACH; ++i) ra[i] = (pa[i] && kin) ? ld8(pa[i] + k0) : zero8;
#pragma unroll
    for (int i = 0; i < BCH; ++i) rb[i] = (pb[i] && kin) ? ld8(pb[i] + k0) : zero8;
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int i = 0; i < ACH; ++i)
      *reinterpret_cast<bf16x8*>(&sA[buf][(r0 + 32 * i) * LDS_K + kc * 8]) = ra[i];
#pragma unroll
    for (int i = 0; i < BCH; ++i)
      *reinterpret_cast<bf16x8*>(&sB[buf][(r0 + 32 * i) * LDS_K + kc * 8]) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (K + BK - 1) / BK;
  load_slab(0);
  store_slab(0);
  __syncthreads();
  const int fr = lane & 31, fh = lane >> 5;      // fragment row, K half
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_slab((kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(
            &sA[buf][(wm * (BM / 2) + i * 32 + fr) * LDS_K + kk * 16 + fh * 8]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(
            &sB[buf][(wn * (BN / 2) + j * 32 + fr) * LDS_K + kk * 16 + fh * 8]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_slab(buf ^ 1);
    __syncthreads();
  }

  // D layout of the 32x32 tile: lane (fh, fr) holds column fr, rows 8*(v/4) + 4*fh + v%4.
  if (MODE == GEMM_SWIGLU_BF16) {
    bf16* C = reinterpret_cast<bf16*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN / 2; ++j) {
        const int f = tile_n * (BN / 2) + wn * (BN / 4) + j * 32 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && f < N)
            C[(int64_t)m * ldc + f] = f2bf(silu_f(acc[i][j][v]) * acc[i][j + TN / 2][v]);
        }
      }
  } else {
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = tile_n * BN + wn * (BN / 2) + j * 32 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && n < N) {
            float* p = C + (int64_t)m * ldc + n;
            if (MODE == GEMM_ADD_F32) *p += acc[i][j][v]; else *p = acc[i][j][v];
          }
        }
      }
  }
}

template <int BM, int BN, int MODE>
hipError_t run(hipStream_t s, const bf16* A, const GemmW& W, void* C, int M, int N, int K, int ldc) {
  const int n_out_per_tile = MODE == GEMM_SWIGLU_BF16 ? BN / 2 : BN;
  dim3 grid((N + n_out_per_tile - 1) / n_out_per_tile, (M + BM - 1) / BM);
  gemm_kernel<BM, BN, MODE><<<grid, 256, 0, s>>>(A, W, C, M, N, K, ldc);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(hipStream_t s, const bf16* A, GemmW W, void* C, int M, int N, int K, int ldc,
                       GemmMode mode) {
  if (M <= 0 || N <= 0 || K <= 0 || K % 8 || ldc < N || !A || !C || !W.ptr[0]) return hipErrorInvalidValue;
  if (((uintptr_t)A | (uintptr_t)W.ptr[0] | (uintptr_t)W.ptr[1] | (uintptr_t)W.ptr[2]) & 15)
    return hipErrorInvalidValue;
  switch (mode) {
    case GEMM_STORE_F32:
      if (W.end[0] > N || (W.end[0] < N && (!W.ptr[1] || W.end[1] > N)) ||
          (W.end[0] < N && W.end[1] < N && (!W.ptr[2] || W.end[2] != N)))
        return hipErrorInvalidValue;
      return run<128, 128, GEMM_STORE_F32>(s, A, W, C, M, N, K, ldc);
    case GEMM_ADD_F32:
      if (W.end[0] != N) return hipErrorInvalidValue;
      return run<128, 128, GEMM_ADD_F32>(s, A, W, C, M, N, K, ldc);
    case GEMM_SWIGLU_BF16:
      if (!W.ptr[1]) return hipErrorInvalidValue;
      return run<128, 128, GEMM_SWIGLU_BF16>(s, A, W, C, M, N, K, ldc);
  }
  return hipErrorInvalidValue;
}

}  // namespace areal
