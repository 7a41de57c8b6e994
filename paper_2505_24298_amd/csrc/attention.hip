// Grouped-query causal attention over the paged KV cache.
//
// One wavefront owns 16 "rows" (decode: the <=16 query heads that share one
// KV head, for one sequence; prefill: 16 consecutive query positions of one
// head) and walks KV blocks of 16 tokens with an online softmax:
//   S^T[token, row] = K_tile . Q^T      v_mfma_f32_16x16x32_f16, K straight
//                                       from HBM in its row-major tile layout
//   P = exp2(S^T - m)                   float32, per-row running max / sum
//   O[row, :] += P . V_tile             v_mfma_f32_16x16x16_f16; the 
//                                       accumulator layout of S^T is already
//                                       the A-operand layout of this product,
//                                       and the V tile is stored in its
//                                       B-operand layout, so nothing is
//                                       transposed or staged through LDS.
#include "kernels.hpp"

namespace areal {
namespace {

constexpr int NB = 2;   // KV blocks per softmax update (32 tokens)

template <int D>
struct KvFrag {
  f16x8 k[NB][D / 32];
  f16x8 v[NB][D / 32];
};

__device__ __forceinline__ f32x4 mfma_qk(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_pv(f16x4 p, f16x4 v, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(p, v, c, 0, 0, 0);
}

// Issue the loads of NB blocks starting at logical block `b` (blocks >= b_end
// are skipped and read as zero).
template <int D>
__device__ __forceinline__ void load_group(KvFrag<D>& f, const f16* __restrict__ arena,
                                           const KvGeom& geom, const int32_t* __restrict__ table,
                                           int b, int b_end, int kvh, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    if (b + u < b_end) {
      const int blk = table[b + u];
      const f16* kt = arena + kv_tile_off(geom, blk, kvh, 0) + j * D + g * (D / 4);
      const f16* vt = arena + kv_tile_off(geom, blk, kvh, 1) + lane * (D / 4);
#pragma unroll
      for (int c = 0; c < D / 32; ++c) {
        f.k[u][c] = ld8(kt + c * 8);
        f.v[u][c] = ld8(vt + c * 8);
      }
    } else {
#pragma unroll
      for (int c = 0; c < D / 32; ++c) {
        f.k[u][c] = zero8;
        f.v[u][c] = zero8;
      }
    }
  }
}

// One online-softmax update over the NB blocks held in `f`.
//   qf     : this lane's slice of its row's query (row = lane & 15)
//   row_pos: last visible token position of this lane's row
//   m, l   : running max (log2 domain) and this lane's share of the running sum
//   o      : accumulator, lane (g, jj) holds rows 4g+v, dims 16n+jj
template <int D>
__device__ __forceinline__ void attend_group(const KvFrag<D>& f, const f16x8 (&qf)[D / 32], int b,
                                             int row_pos, float scale_log2, float& m, float& l,
                                             f32x4 (&o)[D / 16], int lane) {
  const int g = lane >> 4;
  float s[NB][4];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < D / 32; ++c) acc = mfma_qk(f.k[u][c], qf[c], acc);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int t = (b + u) * kBlockTokens + 4 * g + v;
      s[u][v] = t <= row_pos ? acc[v] * scale_log2 : -INFINITY;
      mx = fmaxf(mx, s[u][v]);
    }
  }
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  const float m_use = m_new == -INFINITY ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(m - m_use);   // m = -inf -> 0
  m = m_new;
  float psum = 0.f;
  f16x4 p[NB];
#pragma unroll
  for (int u = 0; u < NB; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float e = __builtin_amdgcn_exp2f(s[u][v] - m_use);
      psum += e;
      p[u][v] = f2h(e);
    }
  l = l * alpha + psum;
  // rescale the accumulator rows: row 4g+v needs the alpha held by lanes with (lane&15)==4g+v
  float ao[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) ao[v] = __shfl(alpha, 4 * g + v);
#pragma unroll
  for (int n = 0; n < D / 16; ++n)
#pragma unroll
    for (int v = 0; v < 4; ++v) o[n][v] *= ao[v];
#pragma unroll
  for (int u = 0; u < NB; ++u)
#pragma unroll
    for (int n = 0; n < D / 16; ++n) {
      const f16x8 vv = f.v[u][n >> 1];
      f16x4 vh;
      if (n & 1) vh = f16x4{vv[4], vv[5], vv[6], vv[7]}; else vh = f16x4{vv[0], vv[1], vv[2], vv[3]};
      o[n] = mfma_pv(p[u], vh, o[n]);
    }
}

// ------------------------------------------------------------------ decode
// Block ids of a split, fetched once: lane l of every wave holds the ids of
// blocks b0 + l and b0 + 64 + l (a split spans at most 128 blocks).
struct BlockIds { int lo, hi; };
__device__ __forceinline__ int block_id(const BlockIds& t, int rel) {
  const int v = rel < 64 ? t.lo : t.hi;
  return __shfl(v, rel & 63);
}

template <int D>
__device__ __forceinline__ void load_group_ids(KvFrag<D>& f, const f16* __restrict__ arena,
                                               const KvGeom& geom, const BlockIds& ids, int b0, int b,
                                               int b_end, int kvh, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    if (b + u < b_end) {                               // wave-uniform
      const int blk = block_id(ids, b + u - b0);
      const f16* kt = arena + kv_tile_off(geom, blk, kvh, 0) + j * D + g * (D / 4);
      const f16* vt = arena + kv_tile_off(geom, blk, kvh, 1) + lane * (D / 4);
#pragma unroll
      for (int c = 0; c < D / 32; ++c) {
        f.k[u][c] = ld8(kt + c * 8);
        f.v[u][c] = ld8(vt + c * 8);
      }
    } else {
#pragma unroll
      for (int c = 0; c < D / 32; ++c) {
        f.k[u][c] = zero8;
        f.v[u][c] = zero8;
      }
    }
  }
}

// One work-group per (split, kv head, sequence); the partials of a sequence cut
// into several splits are combined by attn_merge_kernel.
template <int D>
__global__ __launch_bounds__(256) void attn_decode_kernel(
    const f16* __restrict__ q, RowMeta rm, SeqState st, const f16* __restrict__ arena, KvGeom geom,
    int nq, int chunk, int n_splits, float scale_log2, float* __restrict__ part_o,
    float* __restrict__ part_ml, f16* __restrict__ out) {
  __shared__ float sm[4][16], sl[4][16];
  __shared__ float so[4][16][D];
  const int i = blockIdx.z, kvh = blockIdx.y, split = blockIdx.x;
  const int pos = rm.pos[i], ctx = pos + 1;
  const int t0 = split * chunk;
  if (t0 >= ctx) return;
  const int t1 = min(ctx, t0 + chunk);
  const int b0 = t0 / kBlockTokens, b1 = (t1 + kBlockTokens - 1) / kBlockTokens;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int G = nq / geom.n_kv_heads;
  const int32_t* table = st.table + (int64_t)rm.slot[i] * st.max_blocks;
  BlockIds ids;
  ids.lo = b0 + lane < b1 ? table[b0 + lane] : 0;
  ids.hi = b0 + 64 + lane < b1 ? table[b0 + 64 + lane] : 0;

  f16x8 qf[D / 32];
  {
    const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    const f16* qp = q + ((int64_t)i * nq + kvh * G + j) * D + g * (D / 4);
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qf[c] = j < G ? ld8(qp + c * 8) : zero8;
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[D / 16];
#pragma unroll
  for (int n = 0; n < D / 16; ++n) o[n] = f32x4{0.f, 0.f, 0.f, 0.f};

  // wave w takes block groups w, w+4, ... of this split
  int b = b0 + wave * NB;
  KvFrag<D> cur, nxt;
  if (b < b1) load_group_ids<D>(cur, arena, geom, ids, b0, b, b1, kvh, lane);
  while (b < b1) {
    const int bn = b + 4 * NB;
    if (bn < b1) load_group_ids<D>(nxt, arena, geom, ids, b0, bn, b1, kvh, lane);
    attend_group<D>(cur, qf, b, pos, scale_log2, m, l, o, lane);
    cur = nxt;
    b = bn;
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  if (g == 0) { sm[wave][j] = m; sl[wave][j] = l; }
#pragma unroll
  for (int n = 0; n < D / 16; ++n)
#pragma unroll
    for (int v = 0; v < 4; ++v) so[wave][4 * g + v][16 * n + j] = o[n][v];
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int h = idx / D, dd = idx - h * D;
    float M = fmaxf(fmaxf(sm[0][h], sm[1][h]), fmaxf(sm[2][h], sm[3][h]));
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float sc = __builtin_amdgcn_exp2f(sm[w][h] - M);   // idle wave: m = -inf -> 0
      L += sl[w][h] * sc;
      O += so[w][h][dd] * sc;
    }
    const int head = kvh * G + h;
    if (n_splits == 1) {
      out[((int64_t)i * nq + head) * D + dd] = f2h(O / L);
    } else {
      const int64_t pi = ((int64_t)i * nq + head) * n_splits + split;
      part_o[pi * D + dd] = O;
      if (dd == 0) { part_ml[pi * 2] = M; part_ml[pi * 2 + 1] = L; }
    }
  }
}

// Combine the split partials of one (row, head): out = sum_s O_s 2^(M_s-M) / sum_s L_s 2^(M_s-M).
template <int D>
__global__ __launch_bounds__(D) void attn_merge_kernel(const float* __restrict__ part_o,
                                                       const float* __restrict__ part_ml, RowMeta rm,
                                                       int nq, int chunk, int n_splits,
                                                       f16* __restrict__ out) {
  const int i = blockIdx.x / nq;
  const int ctx = rm.pos[i] + 1;
  const int ns = min(n_splits, (ctx + chunk - 1) / chunk);
  const int64_t base = (int64_t)blockIdx.x * n_splits;
  float M = -INFINITY;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, part_ml[(base + s) * 2]);
  float L = 0.f, O = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float sc = __builtin_amdgcn_exp2f(part_ml[(base + s) * 2] - M);
    L += part_ml[(base + s) * 2 + 1] * sc;
    O += part_o[(base + s) * D + threadIdx.x] * sc;
  }
  out[(int64_t)blockIdx.x * D + threadIdx.x] = f2h(O / L);
}

// ----------------------------------------------------------------- prefill
template <int D>
__global__ __launch_bounds__(256) void attn_prefill_kernel(
    const f16* __restrict__ q, const AttnWork* __restrict__ work, SeqState st,
    const f16* __restrict__ arena, KvGeom geom, int nq, float scale_log2, f16* __restrict__ out) {
  const AttnWork wk = work[blockIdx.x];
  const int head = blockIdx.y, kvh = head / (nq / geom.n_kv_heads);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int r_first = wave * 16;
  if (r_first >= wk.n_rows) return;
  const int my_r = r_first + j;                       // row within the work item
  const bool row_ok = my_r < wk.n_rows;
  const int my_pos = wk.pos0 + my_r;                  // absolute position of this lane's row
  const int last_pos = wk.pos0 + min(wk.n_rows, r_first + 16) - 1;
  const int b1 = last_pos / kBlockTokens + 1;
  const int32_t* table = st.table + (int64_t)wk.slot * st.max_blocks;

  f16x8 qf[D / 32];
  {
    const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    const f16* qp = q + ((int64_t)(wk.row0 + my_r) * nq + head) * D + g * (D / 4);
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qf[c] = row_ok ? ld8(qp + c * 8) : zero8;
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[D / 16];
#pragma unroll
  for (int n = 0; n < D / 16; ++n) o[n] = f32x4{0.f, 0.f, 0.f, 0.f};

  int b = 0;
  KvFrag<D> cur, nxt;
  load_group<D>(cur, arena, geom, table, b, b1, kvh, lane);
  while (b < b1) {
    const int bn = b + NB;
    if (bn < b1) load_group<D>(nxt, arena, geom, table, bn, b1, kvh, lane);
    attend_group<D>(cur, qf, b, row_ok ? my_pos : last_pos, scale_log2, m, l, o, lane);
    cur = nxt;
    b = bn;
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  float lo[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) lo[v] = __shfl(l, 4 * g + v);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int r = r_first + 4 * g + v;
    if (r < wk.n_rows) {
      f16* op = out + ((int64_t)(wk.row0 + r) * nq + head) * D;
      const float inv = 1.0f / lo[v];
#pragma unroll
      for (int n = 0; n < D / 16; ++n) op[16 * n + j] = f2h(o[n][v] * inv);
    }
  }
}

}  // namespace

static bool geom_ok(const KvGeom& g, int nq) {
  const int d = g.head_dim;
  if (d != 32 && d != 64 && d != 128) return false;
  if (g.n_kv_heads <= 0 || nq % g.n_kv_heads || nq / g.n_kv_heads > 16) return false;
  return true;
}

hipError_t launch_attn_decode(hipStream_t s, const f16* q, int M, RowMeta rm, SeqState st,
                              const f16* arena_layer, KvGeom geom, int n_q_heads, int chunk,
                              int n_splits, float* part_o, float* part_ml, f16* out) {
  if (M <= 0 || !geom_ok(geom, n_q_heads) || chunk <= 0 || chunk % (4 * NB * kBlockTokens) ||
      chunk > 128 * kBlockTokens || n_splits <= 0 || (n_splits > 1 && (!part_o || !part_ml)))
    return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)geom.head_dim);
  dim3 grid(n_splits, geom.n_kv_heads, M);
#define AREAL_DEC(DD)                                                                              \
  attn_decode_kernel<DD><<<grid, 256, 0, s>>>(q, rm, st, arena_layer, geom, n_q_heads, chunk,      \
                                               n_splits, scale_log2, part_o, part_ml, out);        \
  if (n_splits > 1)                                                                                \
    attn_merge_kernel<DD><<<M * n_q_heads, DD, 0, s>>>(part_o, part_ml, rm, n_q_heads, chunk,      \
                                                       n_splits, out);
  switch (geom.head_dim) {
    case 32: AREAL_DEC(32) break;
    case 64: AREAL_DEC(64) break;
    default: AREAL_DEC(128) break;
  }
#undef AREAL_DEC
  return hipGetLastError();
}

hipError_t launch_attn_prefill(hipStream_t s, const f16* q, const AttnWork* work, int n_work,
                               SeqState st, const f16* arena_layer, KvGeom geom, int n_q_heads,
                               f16* out) {
  if (n_work <= 0 || !geom_ok(geom, n_q_heads)) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)geom.head_dim);
  dim3 grid(n_work, n_q_heads);
  switch (geom.head_dim) {
    case 32: attn_prefill_kernel<32><<<grid, 256, 0, s>>>(q, work, st, arena_layer, geom, n_q_heads, scale_log2, out); break;
    case 64: attn_prefill_kernel<64><<<grid, 256, 0, s>>>(q, work, st, arena_layer, geom, n_q_heads, scale_log2, out); break;
    default: attn_prefill_kernel<128><<<grid, 256, 0, s>>>(q, work, st, arena_layer, geom, n_q_heads, scale_log2, out); break;
  }
  return hipGetLastError();
}

}  // namespace areal
