// f16 x f16 -> float32 GEMM on the gfx950 matrix cores.
//   C[M,N] (+)= A[M,K] * W[N,K]^T      (both operands K-contiguous)
// Work-group tile BM x BN x 64 staged through LDS with register prefetch of
// the next K-slab; WM x WN wavefronts, each computing (BM/WM) x (BN/WN) with
// v_mfma_f32_32x32x16_f16.  The K range can be split over work-groups
// (float32 atomic accumulation into C) so that skinny decode-shape products
// still fill 256 compute units; the block id -> tile map keeps the row tiles
// that share a weight panel on one XCD (one L2).
#include <algorithm>

#include "kernels.hpp"
#include <cstdlib>

namespace areal {

namespace {

constexpr int BK = 64;
constexpr int LDS_K = BK + 8;   // row stride in elements (144 B): conflict-free 16-B reads

// Row `b` of the W tile -> pointer to that row of the (segmented) weight, or
// null when it lies outside the matrix.
template <int BN, int MODE>
__device__ __forceinline__ const f16* w_row_ptr(const GemmW& W, int tile_n, int b, int N, int K) {
  if (MODE == GEMM_SWIGLU_F16) {
    // every 64 tile rows = 32 gate rows then 32 up rows of the same 32 features
    const int grp = b >> 6, within = b & 63;
    const int isup = within >> 5, c = within & 31;
    const int f = tile_n * (BN / 2) + grp * 32 + c;
    return f < N ? W.ptr[isup] + (int64_t)f * K : nullptr;
  } else {
    const int n = tile_n * BN + b;
    if (n >= N) return nullptr;
    if (n < W.end[0]) return W.ptr[0] + (int64_t)n * K;
    if (n < W.end[1]) return W.ptr[1] + (int64_t)(n - W.end[0]) * K;
    return W.ptr[2] + (int64_t)(n - W.end[1]) * K;
  }
}

// Block id -> (row tile, column tile, K split).  Work-groups are handed to the 8
// XCDs round-robin, so ids equal mod 8 share one L2.
//  * Many row tiles (prefill): inside an XCD consecutive work-groups walk
//    super-tiles of 8 row tiles x 4 column tiles (column tile = 8*g + xcd): the 32
//    work-groups resident on an XCD's 32 compute units then share each A slab 4
//    ways and each W slab 8 ways in that L2.
//  * At most 8 row tiles (decode): a unit = (column tile, K split) with all its
//    row tiles, so that the work-groups that read one W slab run side by side on
//    one XCD; units go to the XCDs round-robin, which keeps the XCDs evenly
//    loaded whatever the number of column tiles (1536 columns = 12 tiles).
constexpr int SUPER_M = 8, SUPER_N = 4;
__host__ __device__ __forceinline__ int grid_blocks(int m_tiles, int n_tiles, int splits) {
  if (m_tiles <= SUPER_M) return 8 * ((n_tiles * splits + 7) / 8) * m_tiles;
  const int n_groups = (n_tiles + 7) / 8;
  const int mb = (m_tiles + SUPER_M - 1) / SUPER_M, nb = (n_groups + SUPER_N - 1) / SUPER_N;
  return 8 * splits * nb * mb * SUPER_M * SUPER_N;
}
__device__ __forceinline__ bool tile_of_block(int id, int m_tiles, int n_tiles, int& tile_m, int& tile_n,
                                              int& split) {
  const int xcd = id & 7, q = id >> 3;
  if (m_tiles <= SUPER_M) {
    const int unit = (q / m_tiles) * 8 + xcd;
    tile_m = q % m_tiles;
    tile_n = unit % n_tiles;
    split = unit / n_tiles;   // the up to 7 padding units get split >= the split count: an empty
    return true;              // K range, on which the kernels return before touching memory
  }
  const int n_groups = (n_tiles + 7) >> 3;
  const int mb = (m_tiles + SUPER_M - 1) / SUPER_M, nb = (n_groups + SUPER_N - 1) / SUPER_N;
  const int within = q % (SUPER_M * SUPER_N), sq = q / (SUPER_M * SUPER_N);
  const int m_blk = sq % mb, rest = sq / mb;
  tile_m = m_blk * SUPER_M + within % SUPER_M;
  tile_n = ((rest % nb) * SUPER_N + within / SUPER_M) * 8 + xcd;
  split = rest / nb;
  return tile_m < m_tiles && tile_n < n_tiles;
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

template <int BM, int BN, int WM, int WN, int MODE, bool RAGGED_K>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(const f16* __restrict__ A, GemmW W,
                                                            void* __restrict__ Cv, int M, int N, int K,
                                                            int ldc, int m_tiles, int n_tiles,
                                                            int slabs_per_split, int atomic) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave
  constexpr int ACH = BM * 8 / NT, BCH = BN * 8 / NT;   // 16-B chunks per thread per slab
  static_assert(TM >= 1 && TN >= 1 && ACH >= 1 && BCH >= 1, "tile too small for the wave grid");
  static_assert(MODE != GEMM_SWIGLU_F16 || (TN % 2 == 0), "SwiGLU needs gate+up in one wave tile");
  __shared__ __attribute__((aligned(16))) f16 sA[2][BM * LDS_K];
  __shared__ __attribute__((aligned(16))) f16 sB[2][BN * LDS_K];

  // block id -> (row tile, column tile, K split): ids that differ by a multiple
  // of 8 sit on the same XCD; the row tiles of one weight panel are adjacent there.
  int tile_m, tile_n, split;
  if (!tile_of_block(blockIdx.x, m_tiles, n_tiles, tile_m, tile_n, split)) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = tile_m * BM;
  const int kc = tid & 7, r0 = tid >> 3;         // chunk column, first chunk row
  constexpr int RSTEP = NT / 8;                  // rows covered per chunk round

  // Rows outside the matrix are clamped to a valid row: they only feed
  // accumulator rows / columns that are never stored.
  const f16* pa[ACH];
  const f16* pb[BCH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int m = min(m0 + r0 + RSTEP * i, M - 1);
    pa[i] = A + (int64_t)m * K + kc * 8;
  }
#pragma unroll
  for (int i = 0; i < BCH; ++i) {
    const f16* p = w_row_ptr<BN, MODE>(W, tile_n, r0 + RSTEP * i, N, K);
    if (!p) p = w_row_ptr<BN, MODE>(W, 0, 0, N, K);
    pb[i] = p + kc * 8;
  }

  struct Slab { f16x8 a[ACH], b[BCH]; };
  // RAGGED_K (K % 64 != 0; K % 8 == 0 always): a 16-byte chunk is all inside or
  // all outside the row; outside chunks are fetched from the row start and zeroed.
  auto load_slab = [&](Slab& r, int k0) {
    if (RAGGED_K) {
      const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
      const bool kin = k0 + kc * 8 < K;
      const int ko = kin ? k0 : -kc * 8;
#pragma unroll
      for (int i = 0; i < BCH; ++i) { const f16x8 v = ld8(pb[i] + ko); r.b[i] = kin ? v : zero8; }
#pragma unroll
      for (int i = 0; i < ACH; ++i) { const f16x8 v = ld8(pa[i] + ko); r.a[i] = kin ? v : zero8; }
    } else {
#pragma unroll
      for (int i = 0; i < BCH; ++i) r.b[i] = ld8(pb[i] + k0);
#pragma unroll
      for (int i = 0; i < ACH; ++i) r.a[i] = ld8(pa[i] + k0);
    }
  };
  auto store_slab = [&](const Slab& r, int buf) {
#pragma unroll
    for (int i = 0; i < ACH; ++i)
      *reinterpret_cast<f16x8*>(&sA[buf][(r0 + RSTEP * i) * LDS_K + kc * 8]) = r.a[i];
#pragma unroll
    for (int i = 0; i < BCH; ++i)
      *reinterpret_cast<f16x8*>(&sB[buf][(r0 + RSTEP * i) * LDS_K + kc * 8]) = r.b[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int fr = lane & 31, fh = lane >> 5;      // fragment row, K half
  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      f16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const f16x8*>(
            &sA[buf][(wm * (BM / WM) + i * 32 + fr) * LDS_K + kk * 16 + fh * 8]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const f16x8*>(
            &sB[buf][(wn * (BN / WN) + j * 32 + fr) * LDS_K + kk * 16 + fh * 8]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  // Software pipeline, two slabs of global loads in flight: while slab kt is
  // multiplied out of LDS, slab kt+1 sits in one register set (already
  // requested) and slab kt+2 is requested into the other.
  const int nk_all = (K + BK - 1) / BK;
  const int kt0 = split * slabs_per_split;
  const int kt1 = min(nk_all, kt0 + slabs_per_split);
  if (kt0 >= kt1) return;
  Slab r0s, r1s;
  // Loads are issued unconditionally (past the end they re-read the last slab)
  // so that no branch separates a load from the wait that consumes it: the
  // wait counters then let two slabs stay in flight.
  const int k_last = (kt1 - 1) * BK;
  load_slab(r0s, kt0 * BK);
  load_slab(r1s, min((kt0 + 1) * BK, k_last));
  store_slab(r0s, 0);
  __syncthreads();
  for (int kt = kt0; kt < kt1; kt += 2) {
    // even step: LDS buffer 0 holds slab kt, r1s holds slab kt+1
    load_slab(r0s, min((kt + 2) * BK, k_last));
    compute(0);
    store_slab(r1s, 1);
    __syncthreads();
    if (kt + 1 >= kt1) break;
    // odd step: LDS buffer 1 holds slab kt+1, r0s holds slab kt+2
    load_slab(r1s, min((kt + 3) * BK, k_last));
    compute(1);
    store_slab(r0s, 0);
    __syncthreads();
  }

  // D layout of the 32x32 tile: lane (fh, fr) holds column fr, rows 8*(v/4) + 4*fh + v%4.
  if (MODE == GEMM_SWIGLU_F16) {
    f16* C = reinterpret_cast<f16*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
        // wave columns [wn*BN/WN + j*32, +64) = gate | up of 32 features
        const int f = tile_n * (BN / 2) + (wn * (BN / WN) + j * 32) / 2 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && f < N)
            C[(int64_t)m * ldc + f] = f2h_sat(silu_f(acc[i][j][v]) * acc[i][j + 1][v]);
        }
      }
  } else {
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = tile_n * BN + wn * (BN / WN) + j * 32 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && n < N) {
            float* p = C + (int64_t)m * ldc + n;
            if (atomic) unsafeAtomicAdd(p, acc[i][j][v]);
            else if (MODE == GEMM_ADD_F32) *p += acc[i][j][v];
            else *p = acc[i][j][v];
          }
        }
      }
  }
}


// Epilogue of the direct-to-LDS kernels: the wave's accumulators to C.
template <int BM, int BN, int WM, int WN, int MODE>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[BM / WM / 32][BN / WN / 32], void* __restrict__ Cv,
                                           int M, int N, int ldc, int tile_m, int tile_n, int wm, int wn,
                                           int fr, int fh, int atomic) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  const int m0 = tile_m * BM;
  if (MODE == GEMM_SWIGLU_F16) {
    f16* C = reinterpret_cast<f16*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
        const int f = tile_n * (BN / 2) + (wn * (BN / WN) + j * 32) / 2 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && f < N)
            C[(int64_t)m * ldc + f] = f2h_sat(silu_f(acc[i][j][v]) * acc[i][j + 1][v]);
        }
      }
  } else {
    float* C = reinterpret_cast<float*>(Cv);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = tile_n * BN + wn * (BN / WN) + j * 32 + fr;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / WM) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (m < M && n < N) {
            float* p = C + (int64_t)m * ldc + n;
            if (atomic) unsafeAtomicAdd(p, acc[i][j][v]);
            else if (MODE == GEMM_ADD_F32) *p += acc[i][j][v];
            else *p = acc[i][j][v];
          }
        }
      }
  }
}

constexpr int GEMM_LSE = 3;     // internal mode of the direct-to-LDS kernel: launch_gemm_lse

__device__ __forceinline__ void lse_pair_combine(float& m, float& s, float m2, float s2) {
  const float mn = fmaxf(m, m2);
  const float mu = mn == -INFINITY ? 0.f : mn;
  s = s * __expf(m - mu) + s2 * __expf(m2 - mu);
  m = mn;
}

// Epilogue of launch_gemm_lse: nothing of the tile is stored but, per row, the (max, sum of
// exponentials) pair over the tile's columns and the value at the row's target column.  The
// ring's LDS is reused (all its loads have landed and all waves are past their last read).
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void store_tile_lse(const f32x16 (&acc)[BM / WM / 32][BN / WN / 32], char* lds,
                                               float2* __restrict__ part, int ld_rows, int M, int N, int tile_m,
                                               int tile_n, int wm, int wn, int fr, int fh, const GemmLse& lse) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NT = WM * WN * 64;
  float2* red = reinterpret_cast<float2*>(lds);                       // [BM][WN]
  int32_t* tgt = reinterpret_cast<int32_t*>(lds + BM * WN * 8);       // [BM]
  const int m0 = tile_m * BM;
  wait_vmcnt(0);
  __syncthreads();
  for (int r = threadIdx.x; r < BM; r += NT) tgt[r] = m0 + r < M ? lse.target[m0 + r] : -1;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = wm * (BM / WM) + i * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
      const int t = tgt[rl];
      float z[TN], m = -INFINITY;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = tile_n * BN + wn * (BN / WN) + j * 32 + fr;
        z[j] = n < N ? acc[i][j][v] * lse.inv_t : -INFINITY;
        if (n == t) lse.target_z[m0 + rl] = z[j];
        m = fmaxf(m, z[j]);
      }
      // the row's maximum over the wave's columns first (lanes of equal fh hold one row), then the
      // exponentials once, against that maximum
#pragma unroll
      for (int o = 1; o < 32; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
      const float mu = m == -INFINITY ? 0.f : m;
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < TN; ++j) sum += __expf(z[j] - mu);
#pragma unroll
      for (int o = 1; o < 32; o <<= 1) sum += __shfl_xor(sum, o);
      if (fr == 0) red[rl * WN + wn] = float2{m, sum};
    }
  __syncthreads();
  for (int r = threadIdx.x; r < BM; r += NT) {
    if (m0 + r >= M) continue;
    float m = -INFINITY, sum = 0.f;
#pragma unroll
    for (int w = 0; w < WN; ++w) lse_pair_combine(m, sum, red[r * WN + w].x, red[r * WN + w].y);
    part[(int64_t)tile_n * ld_rows + m0 + r] = float2{m, sum};
  }
}

// ---- direct-to-LDS variant ---------------------------------------------------
// Same tiling, but the K-slabs travel HBM -> LDS with global_load_lds_dwordx4
// (no register staging) into a ring of STAGES slab buffers, so STAGES-1 slabs
// of loads stay in flight per work-group.  One wavefront instruction moves a
// group of 8 tile rows x 128 B; lane s of the group lands at byte s*16 of the
// group's 1 KiB window, and fetches chunk (s&7) ^ (row&7) of row s>>3, an XOR
// swizzle that makes the later 16-byte fragment reads bank-conflict free.
// Requires K % 64 == 0.
constexpr int GROUP_BYTES = 1024 + 128;   // 8 rows x 128 B, + 128 B skew between groups

// One tile over the K slabs [kt0, kt1), through the ring in `lds` (STAGES * STAGE_BYTES bytes).
template <int BM, int BN, int WM, int WN, int STAGES, int MODE>
__device__ __forceinline__ void dma_tile(const f16* __restrict__ A, const GemmW& W, void* __restrict__ Cv, int M,
                                         int N, int K, int ldc, int tile_m, int tile_n, int kt0, int kt1,
                                         int atomic, const GemmLse& lse, char* lds) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int GA = BM / 8, GB = BN / 8;              // row groups per slab
  constexpr int LPS = (GA + GB) / NW;                  // load instructions per wave per slab
  static_assert((GA + GB) % NW == 0 && GA % NW == 0, "row groups must divide over the waves");
  static_assert(MODE != GEMM_SWIGLU_F16 || (TN % 2 == 0), "SwiGLU needs gate+up in one wave tile");
  constexpr int STAGE_BYTES = (GA + GB) * GROUP_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = tile_m * BM;

  // this wave's share of the row groups: GA/NW groups of A, then GB/NW of B
  const f16* src[LPS];
  int dst_off[LPS];
  {
    const int rin = lane >> 3;                          // row inside the group
#pragma unroll
    for (int i = 0; i < LPS; ++i) {
      const bool is_a = i < GA / NW;
      const int gi = is_a ? wave * (GA / NW) + i : wave * (GB / NW) + (i - GA / NW);
      const int row = gi * 8 + rin;
      const int chunk = (lane & 7) ^ (row & 7);
      if (is_a) {
        const int m = min(m0 + row, M - 1);
        src[i] = A + (int64_t)m * K + chunk * 8;
        dst_off[i] = gi * GROUP_BYTES;
      } else {
        const f16* p = w_row_ptr<BN, MODE>(W, tile_n, row, N, K);
        if (!p) p = w_row_ptr<BN, MODE>(W, 0, 0, N, K);
        src[i] = p + chunk * 8;
        dst_off[i] = (GA + gi) * GROUP_BYTES;
      }
    }
  }
  auto issue = [&](int stage, int k0) {
#pragma unroll
    for (int i = 0; i < LPS; ++i)
      dma16(src[i] + k0, lds + stage * STAGE_BYTES + dst_off[i]);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int fr = lane & 31, fh = lane >> 5;
  // fragment addressing: tile row R -> group R>>3, slot (R&7)*8 + (chunk ^ (R&7))
  int a_base[TM], b_base[TN], koff[BK / 16];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int R = wm * (BM / WM) + i * 32 + fr;
    a_base[i] = (R >> 3) * GROUP_BYTES + (R & 7) * 128;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int R = wn * (BN / WN) + j * 32 + fr;
    b_base[j] = (GA + (R >> 3)) * GROUP_BYTES + (R & 7) * 128;
  }
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) koff[kk] = ((kk * 2 + fh) ^ (fr & 7)) << 4;

  // Fragment reads run one K-step ahead of the MFMAs that consume them, so the
  // LDS latency is covered by a full K-step of matrix work.
  struct Frags { f16x8 a[TM], b[TN]; };
  auto read_frags = [&](Frags& f, const char* base, int kk) {
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = *reinterpret_cast<const f16x8*>(base + a_base[i] + koff[kk]);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = *reinterpret_cast<const f16x8*>(base + b_base[j] + koff[kk]);
  };
  auto mma = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
  };
  auto compute = [&](int stage) {
    const char* base = lds + stage * STAGE_BYTES;
    Frags f0, f1;
    read_frags(f0, base, 0);
    read_frags(f1, base, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(f0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f0, base, 2);
    __builtin_amdgcn_sched_barrier(0);
    mma(f1);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f1, base, 3);
    __builtin_amdgcn_sched_barrier(0);
    mma(f0);
    __builtin_amdgcn_sched_barrier(0);
    mma(f1);
  };

  if (kt0 >= kt1) return;
  const int k_last = (kt1 - 1) * BK;
  // prologue: STAGES-1 slabs in flight (past the end: re-read the last slab, never consumed)
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue(s, min((kt0 + s) * BK, k_last));
  for (int kt = kt0; kt < kt1; kt += STAGES) {
#pragma unroll
    for (int u = 0; u < STAGES; ++u) {
      if (kt + u < kt1) {
        // slab kt+u sits in stage u; the STAGES-2 slabs requested after it may still be in flight
        wait_vmcnt((STAGES - 2) * LPS);
        // plain barrier (no fence: a fence would drain every outstanding load): every wave's
        // part of slab kt+u has landed, and every wave has finished reading stage u-1
        __builtin_amdgcn_s_barrier();
        issue((u + STAGES - 1) % STAGES, min((kt + u + STAGES - 1) * BK, k_last));
        compute(u);
      }
    }
  }
  // (all remaining in-flight loads target LDS only; the epilogue does not touch LDS)

  if constexpr (MODE == GEMM_LSE)
    store_tile_lse<BM, BN, WM, WN>(acc, lds, reinterpret_cast<float2*>(Cv), ldc, M, N, tile_m, tile_n, wm, wn, fr,
                                   fh, lse);
  else
    store_tile<BM, BN, WM, WN, MODE>(acc, Cv, M, N, ldc, tile_m, tile_n, wm, wn, fr, fh, atomic);
  // drain the loads that were requested past the end before the LDS is released
  wait_vmcnt(0);
}

template <int BM, int BN, int WM, int WN, int STAGES, int MODE>
__global__ __launch_bounds__(WM * WN * 64) void gemm_dma_kernel(const f16* __restrict__ A, GemmW W,
                                                                void* __restrict__ Cv, int M, int N,
                                                                int K, int ldc, int m_tiles,
                                                                int n_tiles, int slabs_per_split,
                                                                int atomic, GemmLse lse) {
  __shared__ __attribute__((aligned(16))) char lds[STAGES * (BM / 8 + BN / 8) * GROUP_BYTES];
  int tile_m, tile_n, split;
  if (!tile_of_block(blockIdx.x, m_tiles, n_tiles, tile_m, tile_n, split)) return;
  const int kt0 = split * slabs_per_split;
  dma_tile<BM, BN, WM, WN, STAGES, MODE>(A, W, Cv, M, N, K, ldc, tile_m, tile_n, kt0,
                                         min(K / BK, kt0 + slabs_per_split), atomic, lse, lds);
}

// The same tiles with the last, partly filled round of work-groups evened out (one work-group
// per compute unit; the residual-add products only, whose pieces add into C with float32 atomics).
// XCD x takes the x-th eighth of the tiles (numbered row tile slowest: a block of neighbouring
// tiles, so its work-groups share A and W panels in one L2).  Its G work-groups take whole
// tiles G at a time; the `rem` tiles left over (rem < G) are cut along K: work-group j < rem walks
// the first S = ceil(rem nk / G) slabs of tile j, side by side with the others at the same K, and
// the work-groups j >= rem walk S-slab pieces of what is left of those tiles.  For shapes whose
// tile count leaves compute units idle in the last round (1,536 output columns: 192 tiles of
// 256 x 256 at 8,192 rows on 256 units).
template <int BM, int BN, int WM, int WN, int STAGES>
__global__ __launch_bounds__(WM * WN * 64) void gemm_dma_even_kernel(const f16* __restrict__ A, GemmW W,
                                                                     float* __restrict__ C, int M, int N, int K,
                                                                     int ldc, int n_tiles, int tiles) {
  __shared__ __attribute__((aligned(16))) char lds[STAGES * (BM / 8 + BN / 8) * GROUP_BYTES];
  const int nk = K / BK;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, G = gridDim.x >> 3;
  const int t0 = (int)((int64_t)tiles * xcd / 8), t1 = (int)((int64_t)tiles * (xcd + 1) / 8);
  const int rounds = (t1 - t0) / G, rem = (t1 - t0) % G;
  const GemmLse none{nullptr, nullptr, 1.f};
  auto piece = [&](int tile, int kt0, int kt1) {
    dma_tile<BM, BN, WM, WN, STAGES, GEMM_ADD_F32>(A, W, C, M, N, K, ldc, tile / n_tiles, tile % n_tiles, kt0, kt1,
                                                   1, none, lds);
    __syncthreads();            // every wave is done with the ring before the next piece refills it
  };
  for (int r = 0; r < rounds; ++r) piece(t0 + r * G + j, 0, nk);
  if (rem == 0) return;
  const int last = t0 + rounds * G;
  const int S = (rem * nk + G - 1) / G;                  // slabs per work-group in the last round, < nk
  if (j < rem) {
    piece(last + j, 0, S);
  } else {
    const int tail = nk - S;                             // slabs left of each of the rem tiles
    int u = (j - rem) * S;
    const int u_end = min((j - rem + 1) * S, rem * tail);
    while (u < u_end) {
      const int t = u / tail, k0 = S + u % tail;
      const int k1 = min(nk, k0 + (u_end - u));
      piece(last + t, k0, k1);
      u += k1 - k0;
    }
  }
}

template <int BM, int BN, int WM, int WN, int STAGES>
hipError_t run_dma_even(hipStream_t s, const f16* A, const GemmW& W, float* C, int M, int N, int K, int ldc,
                        int n_groups) {
  if (K % BK || n_groups <= 0 || n_groups % 8) return hipErrorInvalidValue;
  const int n_tiles = (N + BN - 1) / BN, m_tiles = (M + BM - 1) / BM;
  gemm_dma_even_kernel<BM, BN, WM, WN, STAGES><<<n_groups, WM * WN * 64, 0, s>>>(A, W, C, M, N, K, ldc, n_tiles,
                                                                               n_tiles * m_tiles);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int STAGES, int MODE>
hipError_t run_dma(hipStream_t s, const f16* A, const GemmW& W, void* C, int M, int N, int K, int ldc,
                   int splits, GemmLse lse = GemmLse{nullptr, nullptr, 1.f}) {
  if (K % BK) return hipErrorInvalidValue;
  constexpr int n_out_per_tile = MODE == GEMM_SWIGLU_F16 ? BN / 2 : BN;
  const int n_tiles = (N + n_out_per_tile - 1) / n_out_per_tile, m_tiles = (M + BM - 1) / BM;
  const int nk = K / BK;
  splits = std::max(1, std::min(splits, nk));
  const int sps = (nk + splits - 1) / splits;
  splits = (nk + sps - 1) / sps;
  const int grid = grid_blocks(m_tiles, n_tiles, splits);
  gemm_dma_kernel<BM, BN, WM, WN, STAGES, MODE><<<grid, WM * WN * 64, 0, s>>>(
      A, W, C, M, N, K, ldc, m_tiles, n_tiles, sps, (splits > 1 || MODE == GEMM_ADD_F32) ? 1 : 0, lse);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, int MODE>
hipError_t run(hipStream_t s, const f16* A, const GemmW& W, void* C, int M, int N, int K, int ldc,
               int splits) {
  constexpr int n_out_per_tile = MODE == GEMM_SWIGLU_F16 ? BN / 2 : BN;
  const int n_tiles = (N + n_out_per_tile - 1) / n_out_per_tile, m_tiles = (M + BM - 1) / BM;
  const int nk = (K + BK - 1) / BK;
  splits = std::max(1, std::min(splits, nk));
  const int sps = (nk + splits - 1) / splits;
  splits = (nk + sps - 1) / sps;
  const int grid = grid_blocks(m_tiles, n_tiles, splits);
  if (K % BK)
    gemm_kernel<BM, BN, WM, WN, MODE, true><<<grid, WM * WN * 64, 0, s>>>(A, W, C, M, N, K, ldc, m_tiles,
                                                                          n_tiles, sps, (splits > 1 || MODE == GEMM_ADD_F32) ? 1 : 0);
  else
    gemm_kernel<BM, BN, WM, WN, MODE, false><<<grid, WM * WN * 64, 0, s>>>(A, W, C, M, N, K, ldc, m_tiles,
                                                                           n_tiles, sps, (splits > 1 || MODE == GEMM_ADD_F32) ? 1 : 0);
  return hipGetLastError();
}

template <int MODE>
hipError_t dispatch(hipStream_t s, int cfg, const f16* A, const GemmW& W, void* C, int M, int N, int K,
                    int ldc, int splits) {
  switch (cfg) {
    case 0: return run<128, 128, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 1: return run<256, 128, 4, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 2: return run<64, 128, 1, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 3: return run<256, 64, 4, 1, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 4: return run<32, 128, 1, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 5: return run<128, 64, 2, 1, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 6: return run<64, 64, 1, 1, MODE>(s, A, W, C, M, N, K, ldc, splits);
    // direct-to-LDS ring (K % 64 == 0)
    case 7: return run_dma<128, 128, 2, 2, 3, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 8: return run_dma<128, 128, 2, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 9: return run_dma<256, 128, 4, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 10: return run_dma<64, 128, 1, 2, 3, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 11: return run_dma<64, 128, 1, 2, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 12: return run_dma<32, 128, 1, 2, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 13: return run_dma<128, 64, 2, 1, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 14: return run_dma<256, 64, 4, 1, 3, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 15: return run_dma<128, 128, 2, 2, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 16: return run_dma<256, 256, 2, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 17: return run_dma<256, 128, 2, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 18: return run_dma<256, 256, 4, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 19: return run_dma<256, 256, 2, 4, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 20: return run_dma<128, 128, 4, 2, 2, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 21: return run_dma<128, 128, 4, 2, 3, MODE>(s, A, W, C, M, N, K, ldc, splits);
    case 22:   // one 32-column panel per wave: no room for a gate/up pair
      if constexpr (MODE != GEMM_SWIGLU_F16) return run_dma<32, 128, 1, 4, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
      else return hipErrorInvalidValue;
    case 23:
      if constexpr (MODE != GEMM_SWIGLU_F16) return run_dma<64, 128, 2, 4, 3, MODE>(s, A, W, C, M, N, K, ldc, splits);
      else return hipErrorInvalidValue;
    case 24:   // 256 x 256 tiles, last round of work-groups evened out along K (residual-add products)
      if constexpr (MODE == GEMM_ADD_F32)
        return run_dma_even<256, 256, 2, 4, 2>(s, A, W, reinterpret_cast<float*>(C), M, N, K, ldc, 256);
      else return hipErrorInvalidValue;
    case 25:   // 64-column tiles, one 32-column panel per wave (twice the work-groups of 22)
      if constexpr (MODE != GEMM_SWIGLU_F16) return run_dma<32, 64, 1, 2, 4, MODE>(s, A, W, C, M, N, K, ldc, splits);
      else return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int gemm_num_configs() { return 26; }

// Tile configuration and K split for a product of this shape: rules read off
// sweeps over every configuration on the MI355X at the decoder's shapes
// (`cfg` / `splits` >= 0 in launch_gemm_cfg override them).
// Upper limit of the K split (tuning knob for sweeps: AREAL_GEMM_MAX_SPLITS, read once).
static int max_splits() {
  static const int v = [] {
    const char* e = getenv("AREAL_GEMM_MAX_SPLITS");
    const int x = e ? atoi(e) : 0;
    return (x >= 1 && x <= 64) ? x : 12;
  }();
  return v;
}

// Largest K split that keeps every XCD at one round of work-groups (32 CUs, one
// work-group each): units of (column tile, split) go to the XCDs round-robin, each with
// m_tiles work-groups.  Each split keeps at least 3 slabs.  Beyond 8 (12 with a single
// row tile) the atomic adds outweigh the shorter K walk.
static int split_for(int M, int bm, int n_tiles, int nk) {
  const int m_tiles = (M + bm - 1) / bm;
  const int cap = std::min(std::max(1, nk / 3), std::min(m_tiles == 1 ? 12 : 8, max_splits()));
  static const int steps[] = {12, 8, 6, 4, 3, 2, 1};
  for (int cand : steps) {
    if (cand > cap) continue;
    if (((n_tiles * cand + 7) / 8) * m_tiles <= 32 || cand == 1) return cand;
  }
  return 1;
}

void gemm_choose(int M, int N, int K, GemmMode mode, int* cfg, int* splits) {
  const bool dma_ok = (K % BK) == 0;
  const int n_tiles = mode == GEMM_SWIGLU_F16 ? (N + 63) / 64 : (N + 127) / 128;
  const int nk = (K + BK - 1) / BK;
  int c, bm;
  if (!dma_ok) {                       // register-staged path (ragged K)
    if (M <= 32) { c = 4; bm = 32; }
    else if (M <= 64) { c = 2; bm = 64; }
    else { c = 0; bm = 128; }
  } else if (M > 256) {                // prefill: MFMA-bound, large tiles
    const int t256 = (mode == GEMM_SWIGLU_F16 ? (N + 127) / 128 : (N + 255) / 256) * ((M + 255) / 256);
    // down projection (few column tiles, long K): whole 256 x 256 tiles leave compute units idle in
    // the last round (192 tiles on 256 units at 8,192 rows of the 1.5B shape, 448 at the 7B shape);
    // the evened-out launch: 927 against 778 TFLOP/s, 1,063 against 973
    if (mode == GEMM_ADD_F32 && K >= 4096 && t256 >= 96) { *cfg = 24; *splits = 1; return; }
    if (t256 >= 224) { *cfg = 19; *splits = 1; return; }     // 256x256, 8 waves: 940 TFLOP/s
    if (mode == GEMM_ADD_F32 && K >= 4096) {             // down projection: few column tiles, long K
      if (t256 >= 128) { *cfg = 19; *splits = 1; }       // 8192 rows: 760-980 TFLOP/s
      else if (t256 >= 64) { *cfg = 19; *splits = 2; }
      else { *cfg = 20; *splits = 2; }
      return;
    }
    const int t128 = n_tiles * ((M + 127) / 128);
    if (t128 > 256) { *cfg = 20; *splits = 1; return; }  // O projection at 8192 rows
    *cfg = 21; *splits = 1;                              // a last, short pass: 128x128, 8 waves, 3 stages
    return;
  } else if (n_tiles >= 100) {         // wide outputs: one work-group per column panel
    if (M <= 32) { c = 12; bm = 32; }
    else if (M <= 64) { c = 10; bm = 64; }
    else if (M <= 128) { c = 21; bm = 128; }
    else { c = 20; bm = 128; }         // two 128-row work-groups per CU beat one 256-row tile
    if (mode != GEMM_SWIGLU_F16 && c == 12) c = 22;       // output projection: one more wave pair
    if (mode != GEMM_SWIGLU_F16 && c == 10) c = 23;
    if (mode != GEMM_SWIGLU_F16 && c == 20) { c = 19; bm = 256; }   // output projection above 128 rows
    // gate/up with a long K (7B shape, 56 slabs): the register-staged tiles come out 8-10 % ahead
    if (mode == GEMM_SWIGLU_F16 && K >= 3072 && c == 12) c = 4;
    if (mode == GEMM_SWIGLU_F16 && K >= 3072 && c == 10) c = 6;
    if (mode == GEMM_SWIGLU_F16 && K >= 3072 && c == 21) c = 20;
  } else if (mode == GEMM_SWIGLU_F16) { // narrow gate/up (small models): no K split
    if (M <= 32) { c = 12; bm = 32; }
    else if (M <= 64) { c = 10; bm = 64; }
    else { c = 21; bm = 128; }
  } else if (mode == GEMM_ADD_F32 && M <= 32 && K >= 4096 && N <= 2048) {
    // down projection at few rows: 64-column tiles, 8 splits = twice the work-groups of the
    // 128-column tile at 12 splits (8.1 / 8.9 us against 8.7 / 9.8 at 16 / 32 rows of the 1.5B shape)
    *cfg = 25;
    *splits = std::min(8, max_splits());
    return;
  } else {
    // Narrow outputs (QKV, O, down): row tiles of 32 / 64 / 128 with a K split.  Every
    // (tile height, split) with the split no larger than what keeps each XCD at one round
    // of work-groups is priced in microseconds -- a fixed part, the K slabs one work-group
    // walks, and the atomic adds of all splits -- with constants fitted to the sweeps at
    // the 1.5B and 7B shapes; the cheapest wins.
    static const int cand_cfg[3] = {22, 23, 21}, cand_bm[3] = {32, 64, 128};
    static const float slab_us[3] = {0.38f, 0.55f, 0.75f}, fixed_us[3] = {2.f, 2.f, 3.f};
    const float atomic_us = 3.3e-6f * (float)M * (float)N;        // per split
    static const int steps[] = {12, 8, 6, 4, 3, 2, 1};
    float best = 1e30f;
    c = 22; bm = 32;
    int best_sp = 1;
    for (int k = 0; k < 3; ++k) {
      const int sp_max = split_for(M, cand_bm[k], n_tiles, nk);
      for (int sp_k : steps) {
        if (sp_k > sp_max) continue;
        const float cost = fixed_us[k] + (float)((nk + sp_k - 1) / sp_k) * slab_us[k] + atomic_us * (float)sp_k;
        if (cost < best) { best = cost; c = cand_cfg[k]; bm = cand_bm[k]; best_sp = sp_k; }
      }
    }
    *cfg = c;
    *splits = best_sp;
    return;
  }
  int sp = 1;
  if (mode != GEMM_SWIGLU_F16 && M <= 256) sp = split_for(M, bm, n_tiles, nk);
  *cfg = c;
  *splits = sp;
}

hipError_t launch_gemm_cfg(hipStream_t s, const f16* A, GemmW W, void* C, int M, int N, int K, int ldc,
                           GemmMode mode, int cfg, int splits) {
  if (M <= 0 || N <= 0 || K <= 0 || K % 8 || ldc < N || !A || !C || !W.ptr[0]) return hipErrorInvalidValue;
  if (((uintptr_t)A | (uintptr_t)W.ptr[0] | (uintptr_t)W.ptr[1] | (uintptr_t)W.ptr[2]) & 15)
    return hipErrorInvalidValue;
  int c0, s0;
  gemm_choose(M, N, K, mode, &c0, &s0);
  if (cfg < 0) cfg = c0;
  if (splits < 0) splits = s0;
  switch (mode) {
    case GEMM_STORE_F32:
      if (W.end[0] > N || (W.end[0] < N && (!W.ptr[1] || W.end[1] > N)) ||
          (W.end[0] < N && W.end[1] < N && (!W.ptr[2] || W.end[2] != N)))
        return hipErrorInvalidValue;
      return dispatch<GEMM_STORE_F32>(s, cfg, A, W, C, M, N, K, ldc, splits);
    case GEMM_ADD_F32:
      if (W.end[0] != N) return hipErrorInvalidValue;
      return dispatch<GEMM_ADD_F32>(s, cfg, A, W, C, M, N, K, ldc, splits);
    case GEMM_SWIGLU_F16:
      if (!W.ptr[1]) return hipErrorInvalidValue;
      return dispatch<GEMM_SWIGLU_F16>(s, cfg, A, W, C, M, N, K, ldc, 1);
  }
  return hipErrorInvalidValue;
}

// Column tiles of launch_gemm_lse: 256 wide above 256 rows (the 256 x 256 tile), else 128.
int gemm_lse_tiles(int M, int N) { return M > 256 ? (N + 255) / 256 : (N + 127) / 128; }

hipError_t launch_gemm_lse(hipStream_t s, const f16* A, GemmW W, int M, int N, int K, void* part, int ld_rows,
                           GemmLse lse) {
  if (M <= 0 || N <= 0 || K <= 0 || K % BK || ld_rows < M || !A || !part || !W.ptr[0] || W.end[0] != N ||
      !lse.target || !lse.target_z || !(lse.inv_t > 0.f) ||
      (((uintptr_t)A | (uintptr_t)W.ptr[0]) & 15) || ((uintptr_t)part & 7))
    return hipErrorInvalidValue;
  if (M > 256) return run_dma<256, 256, 2, 4, 2, GEMM_LSE>(s, A, W, part, M, N, K, ld_rows, 1, lse);
  return run_dma<128, 128, 4, 2, 3, GEMM_LSE>(s, A, W, part, M, N, K, ld_rows, 1, lse);
}

hipError_t launch_gemm(hipStream_t s, const f16* A, GemmW W, void* C, int M, int N, int K, int ldc,
                       GemmMode mode) {
  // GEMM_STORE_F32 callers that did not zero C get no K split
  int cfg, splits;
  gemm_choose(M, N, K, mode, &cfg, &splits);
  if (mode == GEMM_STORE_F32) splits = 1;
  return launch_gemm_cfg(s, A, W, C, M, N, K, ldc, mode, cfg, splits);
}

}  // namespace areal
