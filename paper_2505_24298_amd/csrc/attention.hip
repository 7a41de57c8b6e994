// Grouped-query causal attention over the paged KV cache.
//
// One wavefront owns 16 "rows" (decode: the <=16 query heads that share one
// KV head, for one sequence; prefill: 16 consecutive query positions of one
// head) and walks KV blocks of 16 tokens with an online softmax:
//   S^T[token, row] = K_tile . Q^T      v_mfma_f32_16x16x32_f16, K straight
//                                       from HBM (tiles stored in operand order)
//   P = exp2(S^T - m)                   float32, per-row running max / sum
//   O[row, :] += P . V_tile             v_mfma_f32_16x16x16_f16; the 
//                                       accumulator layout of S^T is already
//                                       the A-operand layout of this product,
//                                       and the V tile is stored in its
//                                       B-operand layout, so nothing is
//                                       transposed or staged through LDS.
#include "kernels.hpp"
#include <cstdlib>
#include <type_traits>

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
  const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    if (b + u < b_end) {                               // wave-uniform
      const int blk = block_id(ids, b + u - b0);
      // both tiles are stored chunk-major in operand order: load c of a wave reads 1 KiB in a row
      const f16* kt = arena + kv_tile_off(geom, blk, kvh, 0) + lane * 8;
      const f16* vt = arena + kv_tile_off(geom, blk, kvh, 1) + lane * 8;
#pragma unroll
      for (int c = 0; c < D / 32; ++c) {
        f.k[u][c] = ld8(kt + c * 512);
        f.v[u][c] = ld8(vt + c * 512);
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

// Bias, rotate-half RoPE and rounding to half of one head vector of the float32
// QKV row, delivered as this lane's MFMA fragments: lane group g gets dims
// [32c + 8g, +8) for c = 0 .. D/32-1.  For D >= 64 a lane holds both members of
// every rotation pair (dims x and x + D/2 sit in chunks c and c + D/64); for
// D = 32 the partner sits in lane ^ 32.  Loading and rotating are separate steps
// so that the caller can put other loads in flight between them.
template <int D>
struct RawHead {
  float x[D / 32][8];
};
template <int D>
struct RopeAngles {                       // cos / sin of this lane's rotation pairs
  float c[D >= 64 ? D / 64 : 1][8], s[D >= 64 ? D / 64 : 1][8];
};

template <int D>
__device__ __forceinline__ void load_raw(RawHead<D>& r, const float* __restrict__ src, int g) {
#pragma unroll
  for (int c = 0; c < D / 32; ++c) {
    const float4 a = *reinterpret_cast<const float4*>(src + 32 * c + 8 * g);
    const float4 b = *reinterpret_cast<const float4*>(src + 32 * c + 8 * g + 4);
    r.x[c][0] = a.x; r.x[c][1] = a.y; r.x[c][2] = a.z; r.x[c][3] = a.w;
    r.x[c][4] = b.x; r.x[c][5] = b.y; r.x[c][6] = b.z; r.x[c][7] = b.w;
  }
}
template <int D>
__device__ __forceinline__ void load_angles(RopeAngles<D>& a, const float* __restrict__ ct,
                                            const float* __restrict__ sn, int g) {
  constexpr int HC = D >= 64 ? D / 64 : 1;
#pragma unroll
  for (int c = 0; c < HC; ++c) {
    const int j0 = D >= 64 ? 32 * c + 8 * g : (8 * g) & 15;
    const float4 c0 = *reinterpret_cast<const float4*>(ct + j0), c1 = *reinterpret_cast<const float4*>(ct + j0 + 4);
    const float4 s0 = *reinterpret_cast<const float4*>(sn + j0), s1 = *reinterpret_cast<const float4*>(sn + j0 + 4);
    a.c[c][0] = c0.x; a.c[c][1] = c0.y; a.c[c][2] = c0.z; a.c[c][3] = c0.w;
    a.c[c][4] = c1.x; a.c[c][5] = c1.y; a.c[c][6] = c1.z; a.c[c][7] = c1.w;
    a.s[c][0] = s0.x; a.s[c][1] = s0.y; a.s[c][2] = s0.z; a.s[c][3] = s0.w;
    a.s[c][4] = s1.x; a.s[c][5] = s1.y; a.s[c][6] = s1.z; a.s[c][7] = s1.w;
  }
}
template <int D>
__device__ __forceinline__ void rotate(RawHead<D>& r, const f16* __restrict__ bias, const RopeAngles<D>& a,
                                       int g, f16x8 (&out)[D / 32]) {
  if (bias) {
#pragma unroll
    for (int c = 0; c < D / 32; ++c) {
      const f16x8 bb = ld8(bias + 32 * c + 8 * g);
#pragma unroll
      for (int e = 0; e < 8; ++e) r.x[c][e] += h2f(bb[e]);
    }
  }
  if constexpr (D >= 64) {
    constexpr int HC = D / 64;
#pragma unroll
    for (int c = 0; c < HC; ++c)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x1 = r.x[c][e], x2 = r.x[c + HC][e];
        out[c][e] = f2h_sat(x1 * a.c[c][e] - x2 * a.s[c][e]);
        out[c + HC][e] = f2h_sat(x2 * a.c[c][e] + x1 * a.s[c][e]);
      }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float xp = __shfl_xor(r.x[0][e], 32);
      out[0][e] = f2h_sat(g < 2 ? r.x[0][e] * a.c[0][e] - xp * a.s[0][e] : r.x[0][e] * a.c[0][e] + xp * a.s[0][e]);
    }
  }
}

// The leading KV blocks that a set of rows has in common (work-groups blockIdx.x >= n_splits of
// the decode launch: x - n_splits = chunk of the shared part, y = kv head, z = set).  Wave w
// owns tile w of the set: 16 MFMA rows = floor(16 / G) sequences x their G query heads, so
// every lane has its own sequence, position and query head.  Each wave walks all blocks of the
// chunk (the four waves read the same tiles: one fetch from L2 per work-group) and writes
// its rows' partial (max, sum, accumulator) into slot n_splits + chunk of those rows; the
// merge kernel folds them into the rows' own partials.  Every shared position precedes every
// row's position, so nothing is masked but the tail of the last block pair.  Block ids: row
// M + set of the per-step table.
template <int D>
__device__ __forceinline__ void decode_shared_set(
    const float* __restrict__ qkv, const RowMeta& rm, const f16* __restrict__ bq,
    const float* __restrict__ cos_tab, const float* __restrict__ sin_tab,
    const f16* __restrict__ arena, const KvGeom& geom, int nq, int n_splits, int n_slots,
    float scale_log2, float* __restrict__ part_o, float* __restrict__ part_ml,
    const int32_t* __restrict__ step_table, int step_stride, const DecodeGroups& grp, int M) {
  const int set = blockIdx.z, kvh = blockIdx.y, u = (int)blockIdx.x - n_splits;
  if (set >= grp.n_sets) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int nkv = geom.n_kv_heads, G = nq / nkv, P = 16 / G;
  const int chunk = grp.sh_chunk;
  const int t0 = u * chunk, b0 = t0 / kBlockTokens;
  const int32_t* table = step_table + (int64_t)(M + set) * step_stride;
  const int b_cap = min(b0 + chunk / kBlockTokens, step_stride);
  BlockIds ids;
  ids.lo = b0 + lane < b_cap ? table[b0 + lane] : 0;
  ids.hi = b0 + 64 + lane < b_cap ? table[b0 + 64 + lane] : 0;
  const int sq = j / G;                                  // sequence of this lane's row inside the tile
  const int r = sq < P ? grp.set_rows[((int64_t)set * kGroupTiles + wave) * 16 + sq] : -1;
  const int ts = grp.set_start[set];
  if (t0 >= ts) return;
  if (__ballot(r >= 0) == 0) return;                     // no tile for this wave
  const int t1 = min(ts, t0 + chunk);
  const int b1 = (t1 + kBlockTokens - 1) / kBlockTokens;
  const int rr = max(r, 0);                              // empty rows read row 0 and are zeroed below
  const int pos = rm.pos[rr];
  const int head = kvh * G + (j - sq * G);
  RawHead<D> qraw;
  load_raw<D>(qraw, qkv + ((int64_t)rr * (nq + 2 * nkv) + head) * D, g);
  RopeAngles<D> ang;
  load_angles<D>(ang, cos_tab + (int64_t)pos * (D / 2), sin_tab + (int64_t)pos * (D / 2), g);
  int b = b0;
  KvFrag<D> cur, nxt;
  load_group_ids<D>(cur, arena, geom, ids, b0, b, b1, kvh, lane);
  f16x8 qf[D / 32];
  rotate<D>(qraw, bq ? bq + head * D : nullptr, ang, g, qf);
  if (r < 0) {
    const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qf[c] = zero8;
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[D / 16];
#pragma unroll
  for (int n = 0; n < D / 16; ++n) o[n] = f32x4{0.f, 0.f, 0.f, 0.f};
  while (b < b1) {
    const int bn = b + NB;
    if (bn < b1) load_group_ids<D>(nxt, arena, geom, ids, b0, bn, b1, kvh, lane);
    attend_group<D>(cur, qf, b, t1 - 1, scale_log2, m, l, o, lane);
    cur = nxt;
    b = bn;
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  const int slot = n_splits + u;
  if (g == 0 && r >= 0) {
    const int64_t pi = ((int64_t)r * nq + head) * n_slots + slot;
    part_ml[pi * 2] = m;
    part_ml[pi * 2 + 1] = l;
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {                          // accumulator row 4g+v belongs to lane 4g+v's row
    const int r_v = __shfl(r, 4 * g + v), head_v = __shfl(head, 4 * g + v);
    if (r_v >= 0) {
      const int64_t pi = ((int64_t)r_v * nq + head_v) * n_slots + slot;
#pragma unroll
      for (int n = 0; n < D / 16; ++n) part_o[pi * D + 16 * n + j] = o[n][v];
    }
  }
}

// One work-group per (split, kv head, sequence); the partials of a sequence cut
// into several splits are combined by attn_merge_kernel.  The row's query heads
// are taken from the float32 QKV row (bias, RoPE, rounding done here).  The
// cached positions 0 .. pos-1 come from the paged arena; the token being
// appended (position pos) is handled by the work-group whose split contains
// pos: it rotates and rounds the new key, stores key and value into the
// sequence's block for later steps, and folds the new token into its softmax
// state as one more (score, value) pair.
template <int D>
__global__ __launch_bounds__(256) void attn_decode_kernel(
    const float* __restrict__ qkv, RowMeta rm, SeqState st, const f16* __restrict__ bq,
    const f16* __restrict__ bk, const f16* __restrict__ bv, const float* __restrict__ cos_tab,
    const float* __restrict__ sin_tab, f16* __restrict__ arena, KvGeom geom, int nq, int chunk,
    int n_splits, float scale_log2, float* __restrict__ part_o, float* __restrict__ part_ml,
    f16* __restrict__ out, const int32_t* __restrict__ step_table, int step_stride, DecodeGroups grp) {
  __shared__ float sm[4][16], sl[4][16];
  __shared__ float so[4][16][D];
  __shared__ float s_new[16], v_new[D];
  const int n_slots = n_splits + grp.n_shared;           // partial slots per (row, head)
  if ((int)blockIdx.x >= n_splits) {                     // the shared leading blocks of a set of rows
    if ((int)blockIdx.x >= n_slots) return;             // padding column (the launch keeps gridDim.x odd)
    decode_shared_set<D>(qkv, rm, bq, cos_tab, sin_tab, arena, geom, nq, n_splits, n_slots,
                         scale_log2, part_o, part_ml, step_table, step_stride, grp, (int)gridDim.z);
    return;
  }
  const int i = blockIdx.z, kvh = blockIdx.y, split = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int nkv = geom.n_kv_heads, G = nq / nkv;
  // Token and block indices below are relative to the first position this row's own
  // work-groups cover (t_start, a multiple of the block size; the row of the per-step table
  // starts at that block too), so that no address depends on t_start.
  const int t0 = split * chunk;
  const int b0 = t0 / kBlockTokens;
  // the table entries of the whole split are requested at once with the row's position (entries
  // past the sequence's last block are stale but inside the table row, and never used)
  // (with the per-step table, row i of which lists the blocks of this launch's row i, the
  // address depends on the block index alone: one load fewer in front of the first tile)
  const int32_t* table = step_table ? step_table + (int64_t)i * step_stride
                                    : st.table + (int64_t)rm.slot[i] * st.max_blocks;
  const int b_cap = min(b0 + chunk / kBlockTokens, step_table ? step_stride : st.max_blocks);
  BlockIds ids;
  ids.lo = b0 + lane < b_cap ? table[b0 + lane] : 0;
  ids.hi = b0 + 64 + lane < b_cap ? table[b0 + 64 + lane] : 0;
  const int pos_abs = rm.pos[i];
  const int pos = pos_abs - (grp.t_start ? grp.t_start[i] : 0);
  if (t0 > pos) return;
  const bool owner = pos < t0 + chunk;                 // this split holds the appended position
  const int t1 = min(pos, t0 + chunk);                 // cached tokens [t0, t1)
  const int b1 = (t1 + kBlockTokens - 1) / kBlockTokens;

  // Loads go out in dependency order (the query row needs nothing, the angles need pos,
  // the K/V tiles need the block ids) and the rotation runs while the tiles are in flight.
  const float* row = qkv + (int64_t)i * (nq + 2 * nkv) * D;
  const int head = kvh * G + min(j, G - 1);
  RawHead<D> qraw;
  load_raw<D>(qraw, row + head * D, g);
  RopeAngles<D> ang;
  load_angles<D>(ang, cos_tab + (int64_t)pos_abs * (D / 2), sin_tab + (int64_t)pos_abs * (D / 2), g);

  // wave w takes block groups w, w+4, ... of this split
  int b = b0 + wave * NB;
  KvFrag<D> cur, nxt;
  if (b < b1) load_group_ids<D>(cur, arena, geom, ids, b0, b, b1, kvh, lane);

  f16x8 qf[D / 32];
  rotate<D>(qraw, bq ? bq + head * D : nullptr, ang, g, qf);
  if (j >= G) {
    const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qf[c] = zero8;
  }
  if (owner && wave == 0) {                            // wave-uniform
    RawHead<D> kraw;
    load_raw<D>(kraw, row + (nq + kvh) * D, g);
    f16x8 kf[D / 32];
    rotate<D>(kraw, bk ? bk + kvh * D : nullptr, ang, g, kf);
    float dot = 0.f;
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
#pragma unroll
      for (int e = 0; e < 8; ++e) dot += h2f(qf[c][e]) * h2f(kf[c][e]);
    dot += __shfl_xor(dot, 16);
    dot += __shfl_xor(dot, 32);
    if (g == 0) s_new[j] = dot * scale_log2;
    const int blk = table[pos / kBlockTokens], tin = pos % kBlockTokens;
    if (j == 0) {
      f16* kt = arena + kv_tile_off(geom, blk, kvh, 0);
#pragma unroll
      for (int c = 0; c < D / 32; ++c) *reinterpret_cast<f16x8*>(kt + k_tile_index(tin, 32 * c + 8 * g)) = kf[c];
    }
    f16* vt = arena + kv_tile_off(geom, blk, kvh, 1);
    const float* vrow = row + (nq + nkv + kvh) * D;
    for (int dim = lane; dim < D; dim += 64) {
      float v = vrow[dim];
      if (bv) v += h2f(bv[kvh * D + dim]);
      const f16 hv = f2h_sat(v);
      v_new[dim] = h2f(hv);
      vt[v_tile_index(D, tin, dim)] = hv;
    }
  }
  float m = -INFINITY, l = 0.f;
  f32x4 o[D / 16];
#pragma unroll
  for (int n = 0; n < D / 16; ++n) o[n] = f32x4{0.f, 0.f, 0.f, 0.f};

  while (b < b1) {
    const int bn = b + 4 * NB;
    if (bn < b1) load_group_ids<D>(nxt, arena, geom, ids, b0, bn, b1, kvh, lane);
    attend_group<D>(cur, qf, b, pos - 1, scale_log2, m, l, o, lane);
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
    const float Mu = M == -INFINITY ? 0.f : M;               // no cached token in this split
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float sc = __builtin_amdgcn_exp2f(sm[w][h] - Mu);  // idle wave: m = -inf -> 0
      L += sl[w][h] * sc;
      O += so[w][h][dd] * sc;
    }
    if (owner) {                                             // the appended token
      const float sN = s_new[h];
      const float M2 = fmaxf(M, sN);
      const float a = __builtin_amdgcn_exp2f(M - M2), e = __builtin_amdgcn_exp2f(sN - M2);
      L = L * a + e;
      O = O * a + e * v_new[dd];
      M = M2;
    }
    const int head = kvh * G + h;
    if (n_slots == 1) {
      out[((int64_t)i * nq + head) * D + dd] = f2h_sat(O / L);
    } else {
      const int64_t pi = ((int64_t)i * nq + head) * n_slots + split;
      part_o[pi * D + dd] = O;
      if (dd == 0) { part_ml[pi * 2] = M; part_ml[pi * 2 + 1] = L; }
    }
  }
}

// Combine the split partials of one (row, head): out = sum_s O_s 2^(M_s-M) / sum_s L_s 2^(M_s-M).
// Every load address depends only on the launch shape, so the row's position, the
// statistics (lane s fetches (M_s, L_s)) and the first eight partial rows all go out
// together; which slots really exist for this row is applied afterwards by selection.  The
// other slots hold stale values of earlier launches: selected away, never multiplied.
template <int D>
__global__ __launch_bounds__(D < 64 ? 64 : D) void attn_merge_kernel(const float* __restrict__ part_o,
                                                       const float* __restrict__ part_ml, RowMeta rm,
                                                       int nq, int chunk, int n_splits, int n_shared,
                                                       int sh_chunk, const int32_t* __restrict__ t_start,
                                                       f16* __restrict__ out) {
  constexpr int BATCH = 8;
  const int n_slots = n_splits + n_shared;                    // <= 32
  const int i = blockIdx.x / nq;
  const int64_t base = (int64_t)blockIdx.x * n_slots;
  const int lane = threadIdx.x & 63;
  const int dd = min((int)threadIdx.x, D - 1);
  const float* po = part_o + base * D + dd;
  const int pos_abs = rm.pos[i];
  const int ts = t_start ? t_start[i] : 0;
  float2 ml = {0.f, 0.f};
  if (lane < n_slots) ml = *reinterpret_cast<const float2*>(part_ml + (base + lane) * 2);
  float v[BATCH], vn[BATCH];
#pragma unroll
  for (int u = 0; u < BATCH; ++u) v[u] = u < n_slots ? po[(int64_t)u * D] : 0.f;

  // slots of this row: its own splits 0 .. ceil((pos + 1 - ts) / chunk) - 1, then the chunks of
  // the part it shares with its set (slot n_splits + u exists while u * chunk < ts)
  const int ns = min(n_splits, (pos_abs - ts + chunk) / chunk);
  const bool mine = lane < n_splits ? lane < ns : (lane < n_slots && (lane - n_splits) * sh_chunk < ts);
  const uint64_t have = __ballot(mine);                       // slots live in lanes 0 .. 31
  const float ms = mine ? ml.x : -INFINITY, ls = mine ? ml.y : 0.f;
  const float M = wave_max(ms);                               // whole waves only: blockDim >= 64
  const float sc = __builtin_amdgcn_exp2f(ms - M);           // other lanes: 2^-inf = 0
  const float L = wave_sum(ls * sc);
  float O = 0.f;
  for (int s0 = 0; s0 < n_slots; s0 += BATCH) {
    const bool more = (have >> (s0 + BATCH)) != 0 && s0 + BATCH < n_slots;
    if (more) {                                               // next batch in flight while this one is used
#pragma unroll
      for (int u = 0; u < BATCH; ++u) vn[u] = s0 + BATCH + u < n_slots ? po[(int64_t)(s0 + BATCH + u) * D] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const float w = __shfl(sc, (s0 + u) & 31);
      O += ((have >> (s0 + u)) & 1u) ? v[u] * w : 0.f;
    }
    if (!more) break;
#pragma unroll
    for (int u = 0; u < BATCH; ++u) v[u] = vn[u];
  }
  if (threadIdx.x < D) out[(int64_t)blockIdx.x * D + dd] = f2h_sat(O / L);
}

// ----------------------------------------------------------------- prefill
// One work-group per (tile of 16 or 32 query positions, kv head): its rows are
// those positions x the G query heads that share the kv head, cut into
// row-groups of 16 (positions of one head), RGW row-groups per wave.  KV blocks
// travel HBM -> LDS once per work-group (global_load_lds, a ring of PF_STAGES
// stages of two blocks each) and every wave multiplies all its row-groups
// against them, so each K/V byte fetched serves up to 32*G query rows.
// Both products use the 16x16x32 MFMA: for P.V the 32-deep contraction runs
// over the two blocks of a stage (slots 0-3: tokens 4g..4g+3 of the first
// block, slots 4-7: of the second), which is the order the S^T accumulators and
// the stored V tiles already have.
constexpr int PF_STAGES = 3;


// One online-softmax update of all RGW row-groups of a wave over the two blocks
// in `f`.  The three phases run over all row-groups at a time, so that their
// independent MFMA chains and reductions overlap and the value operands are
// assembled once.  The running maximum is a reference, not an exact maximum: it
// is raised (two cross-lane exchanges and a rescale of the accumulator) only
// when some score of the wave exceeds it by more than 2^kMaxSlack, so
// probabilities stay below 2^kMaxSlack in half precision and the common step
// has no cross-lane traffic at all.
constexpr float kMaxSlack = 8.0f;

template <int D, int RGW, bool MASK>
__device__ __forceinline__ void attend_pairs(const char* __restrict__ stage, const int (&k_off)[D / 32],
                                             const int (&v_off)[D / 32], const f16x8 (&qf)[RGW][D / 32],
                                             int b, const int (&rpos)[RGW], float scale_log2,
                                             float (&m)[RGW], float (&l)[RGW], f32x4 (&o)[RGW][D / 16],
                                             int lane) {
  constexpr int TILE_B = 16 * D * 2;
  const int g = lane >> 4;
  // K fragments now, V fragments only once the probabilities exist: the two sets never
  // occupy registers together
  f16x8 kf[2][D / 32];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int c = 0; c < D / 32; ++c)
      kf[u][c] = *reinterpret_cast<const f16x8*>(stage + (u * 2) * TILE_B + k_off[c]);
  f32x4 acc[RGW][2];
#pragma unroll
  for (int r = 0; r < RGW; ++r)
#pragma unroll
    for (int u = 0; u < 2; ++u) acc[r][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < D / 32; ++c)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < RGW; ++r) acc[r][u] = mfma_qk(kf[u][c], qf[r][c], acc[r][u]);

  // scores stay unscaled (s = q.k); the 1/sqrt(d) log2(e) factor rides in the exponent's fma.
  // MASK = false: every token of the pair is visible to every row of the wave.
  f16x8 p[RGW];
#pragma unroll
  for (int r = 0; r < RGW; ++r) {
    float s[2][4];
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int t = (b + u) * kBlockTokens + 4 * g + v;
        s[u][v] = (!MASK || t <= rpos[r]) ? acc[r][u][v] : -INFINITY;
        mx = fmaxf(mx, s[u][v]);
      }
    mx *= scale_log2;
    if (__any(mx > m[r] + kMaxSlack)) {                 // wave-uniform; m = -inf at the start
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m[r], mx);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m[r] - m_use);   // m = -inf -> 0
      m[r] = m_new;
      l[r] *= alpha;
      float ao[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) ao[v] = __shfl(alpha, 4 * g + v);
#pragma unroll
      for (int n = 0; n < D / 16; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) o[r][n][v] *= ao[v];
    }
    const float m_use = m[r] == -INFINITY ? 0.f : m[r];
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][v], scale_log2, -m_use));
        psum += e;
        p[r][u * 4 + v] = f2h(e);
      }
    l[r] += psum;
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int c = 0; c < D / 32; ++c) {
    const f16x8 v0 = *reinterpret_cast<const f16x8*>(stage + 1 * TILE_B + v_off[c]);
    const f16x8 v1 = *reinterpret_cast<const f16x8*>(stage + 3 * TILE_B + v_off[c]);
    const f16x8 ve = f16x8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    const f16x8 vo = f16x8{v0[4], v0[5], v0[6], v0[7], v1[4], v1[5], v1[6], v1[7]};
#pragma unroll
    for (int r = 0; r < RGW; ++r) o[r][2 * c] = mfma_qk(p[r], ve, o[r][2 * c]);
#pragma unroll
    for (int r = 0; r < RGW; ++r) o[r][2 * c + 1] = mfma_qk(p[r], vo, o[r][2 * c + 1]);
  }
}

template <int D, int RGW>
__global__ __launch_bounds__(256, (D == 128 && RGW == 3) ? 2 : 1) void attn_prefill_kernel(
    const f16* __restrict__ q, const AttnWork* __restrict__ work, SeqState st,
    const f16* __restrict__ arena, KvGeom geom, int nq, int tile_pos, float scale_log2,
    f16* __restrict__ out) {
  constexpr int TILE_B = 16 * D * 2;      // bytes of one K or V tile
  constexpr int STAGE_B = 4 * TILE_B;     // two blocks x (K, V)
  constexpr int NI = TILE_B / 1024;       // load instructions per tile = per wave per stage
  __shared__ __attribute__((aligned(16))) char lds[PF_STAGES * STAGE_B];

  const AttnWork wk = work[blockIdx.x];
  const int kvh = blockIdx.y;
  const int G = nq / geom.n_kv_heads;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, j = lane & 15;
  const int n_rg = (tile_pos / 16) * G;
  const int last_pos = wk.pos0 + wk.n_rows - 1;
  const int b_end = last_pos / kBlockTokens + 1;
  const int n_pairs = (b_end + 1) >> 1;
  const int32_t* table = st.table + (int64_t)wk.slot * st.max_blocks;

  // ---- this wave's row-groups ----
  f16x8 qf[RGW][D / 32];
  float m[RGW], l[RGW];
  f32x4 o[RGW][D / 16];
  int rpos[RGW], gmax[RGW];
#pragma unroll
  for (int r = 0; r < RGW; ++r) {
    const int rg = wave * RGW + r;
    const int pos_blk = rg / G, head = kvh * G + rg % G;
    const int row_in = pos_blk * 16 + j;
    const bool active = rg < n_rg && pos_blk * 16 < wk.n_rows;
    const bool ok = active && row_in < wk.n_rows;
    gmax[r] = active ? wk.pos0 + min(wk.n_rows, pos_blk * 16 + 16) - 1 : -1;
    rpos[r] = ok ? wk.pos0 + row_in : gmax[r];
    const f16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
    // MFMA c contracts dims [32c, 32c+32), lane group g its slice [32c + 8g, +8): the order of the K tiles
    const f16* qp = q + ((int64_t)(wk.row0 + (ok ? row_in : 0)) * nq + (active ? head : 0)) * D + g * 8;
#pragma unroll
    for (int c = 0; c < D / 32; ++c) qf[r][c] = ok ? ld8(qp + c * 32) : zero8;
    m[r] = -INFINITY;
    l[r] = 0.f;
#pragma unroll
    for (int n = 0; n < D / 16; ++n) o[r][n] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // pairs of blocks that lie wholly below the first query position of this wave need no mask
  // (row-group r = 0 holds the wave's earliest positions; a wave without rows masks everything)
  const int p_free = gmax[0] >= 0 ? (wk.pos0 + ((wave * RGW) / G) * 16 + 1) / (2 * kBlockTokens) : 0;

  // ---- this wave's share of the loads: one tile of the stage (block u, K or V) ----
  const int u_ld = wave >> 1, isv_ld = wave & 1;
  // tiles are stored in operand order, chunk c of all lanes in a 1 KiB run: the copy into LDS
  // is verbatim and lane-linear, and so are the fragment reads (no bank conflicts, no swizzle)
  int src_off[NI];
#pragma unroll
  for (int t = 0; t < NI; ++t) src_off[t] = (t * 64 + lane) * 8;
  int id_chunk = -1, ids = 0;
  auto issue = [&](int pair, int stage) {
    const int b = min(2 * pair + u_ld, b_end - 1);     // past the end: re-read the last block (masked anyway)
    if ((b >> 6) != id_chunk) {                        // wave-uniform
      id_chunk = b >> 6;
      const int bb = id_chunk * 64 + lane;
      ids = bb < b_end ? table[bb] : 0;
    }
    const int blk = __shfl(ids, b & 63);
    const f16* tile = arena + kv_tile_off(geom, blk, kvh, isv_ld);
    char* dst = lds + stage * STAGE_B + (u_ld * 2 + isv_ld) * TILE_B;
#pragma unroll
    for (int t = 0; t < NI; ++t) dma16(tile + src_off[t], dst + t * 1024);
  };

  // ---- fragment addresses inside a stage ----
  int k_off[D / 32], v_off[D / 32];
#pragma unroll
  for (int c = 0; c < D / 32; ++c) k_off[c] = v_off[c] = c * 1024 + lane * 16;

#pragma unroll
  for (int s = 0; s < PF_STAGES - 1; ++s) issue(min(s, n_pairs - 1), s);
  auto step = [&](int p, auto masked) {
    wait_vmcnt((PF_STAGES - 2) * NI);
    __builtin_amdgcn_s_barrier();
    issue(min(p + PF_STAGES - 1, n_pairs - 1), (p + PF_STAGES - 1) % PF_STAGES);
    attend_pairs<D, RGW, decltype(masked)::value>(lds + (p % PF_STAGES) * STAGE_B, k_off, v_off, qf, 2 * p,
                                                  rpos, scale_log2, m, l, o, lane);
  };
  // all waves of the work-group run the same number of steps (the barrier is shared); each
  // wave's mask-free prefix is its own
  const int p_split = min(p_free, n_pairs);
  for (int p = 0; p < p_split; ++p) step(p, std::false_type{});
  for (int p = p_split; p < n_pairs; ++p) step(p, std::true_type{});
  wait_vmcnt(0);

#pragma unroll
  for (int r = 0; r < RGW; ++r) {
    const int rg = wave * RGW + r;
    const int pos_blk = rg / G, head = kvh * G + rg % G;
    float lr = l[r];
    lr += __shfl_xor(lr, 16);
    lr += __shfl_xor(lr, 32);
    float lo[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) lo[v] = __shfl(lr, 4 * g + v);
    if (gmax[r] < 0) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row_in = pos_blk * 16 + 4 * g + v;
      if (row_in < wk.n_rows) {
        f16* op = out + ((int64_t)(wk.row0 + row_in) * nq + head) * D;
        const float inv = 1.0f / lo[v];
#pragma unroll
        for (int n = 0; n < D / 16; ++n) op[16 * n + j] = f2h_sat(o[r][n][v] * inv);
      }
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

static bool groups_ok(const DecodeGroups& grp, int M, int n_splits, const int32_t* step_table) {
  if (grp.n_sets == 0 && grp.n_shared == 0 && !grp.t_start) return true;
  return grp.n_sets > 0 && grp.n_sets <= M && grp.n_shared > 0 && n_splits + grp.n_shared <= 32 &&
         grp.sh_chunk > 0 && grp.sh_chunk % (NB * kBlockTokens) == 0 && grp.sh_chunk <= 128 * kBlockTokens &&
         grp.t_start && grp.set_rows && grp.set_start && step_table;
}

hipError_t launch_attn_decode(hipStream_t s, const float* qkv, int M, RowMeta rm, SeqState st,
                              const f16* bq, const f16* bk, const f16* bv, const float* cos_tab,
                              const float* sin_tab, f16* arena_layer, KvGeom geom, int n_q_heads,
                              int chunk, int n_splits, float* part_o, float* part_ml, f16* out,
                              const int32_t* step_table, int step_stride, DecodeGroups grp) {
  if (step_table && step_stride <= 0) return hipErrorInvalidValue;
  if (M <= 0 || !geom_ok(geom, n_q_heads) || chunk <= 0 || chunk % (4 * NB * kBlockTokens) ||
      chunk > 128 * kBlockTokens || n_splits <= 0 || !groups_ok(grp, M, n_splits, step_table) ||
      (n_splits + grp.n_shared > 1 && (!part_o || !part_ml)) ||
      !qkv || !cos_tab || !sin_tab || (bq && (!bk || !bv)) ||
      (((uintptr_t)qkv | (uintptr_t)bq | (uintptr_t)bk | (uintptr_t)bv | (uintptr_t)arena_layer) & 15))
    return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)geom.head_dim);
  // Work-groups go to the eight XCDs round-robin in launch order (x fastest).  With an even
  // gridDim.x a split index would always land on the same few XCDs, and the low splits, which
  // every row has, would crowd them; an odd gridDim.x rotates the assignment row by row.
  dim3 grid((n_splits + grp.n_shared) | 1, geom.n_kv_heads, M);
#define AREAL_DEC(DD)                                                                              \
  attn_decode_kernel<DD><<<grid, 256, 0, s>>>(qkv, rm, st, bq, bk, bv, cos_tab, sin_tab,           \
                                               arena_layer, geom, n_q_heads, chunk, n_splits,      \
                                               scale_log2, part_o, part_ml, out, step_table,       \
                                               step_stride, grp);
  switch (geom.head_dim) {
    case 32: AREAL_DEC(32) break;
    case 64: AREAL_DEC(64) break;
    default: AREAL_DEC(128) break;
  }
#undef AREAL_DEC
  return hipGetLastError();
}

hipError_t launch_attn_merge(hipStream_t s, int M, RowMeta rm, int head_dim, int n_q_heads, int chunk,
                             int n_splits, const float* part_o, const float* part_ml, f16* out,
                             DecodeGroups grp) {
  const int n_slots = n_splits + grp.n_shared;
  if (M <= 0 || n_splits < 1 || n_slots < 2 || n_slots > 32 || chunk <= 0 || !part_o || !part_ml || !out ||
      (grp.n_shared > 0 && (!grp.t_start || grp.sh_chunk <= 0)) || (head_dim != 32 && head_dim != 64 && head_dim != 128))
    return hipErrorInvalidValue;
#define AREAL_MRG(DD)                                                                              \
  attn_merge_kernel<DD><<<M * n_q_heads, DD < 64 ? 64 : DD, 0, s>>>(part_o, part_ml, rm, n_q_heads, \
                                                                    chunk, n_splits, grp.n_shared,  \
                                                                    grp.sh_chunk, grp.t_start, out);
  switch (head_dim) {
    case 32: AREAL_MRG(32) break;
    case 64: AREAL_MRG(64) break;
    default: AREAL_MRG(128) break;
  }
#undef AREAL_MRG
  return hipGetLastError();
}

int attn_prefill_tile_rows(int n_q_heads, int n_kv_heads) {
  // tuning knob for sweeps: AREAL_PREFILL_TILE_ROWS=16|32 (read once)
  static const int forced = [] {
    const char* e = getenv("AREAL_PREFILL_TILE_ROWS");
    const int v = e ? atoi(e) : 0;
    return (v == 16 || v == 32) ? v : 0;
  }();
  // at most 3 row-groups per wave keep two work-groups resident per CU at head_dim 128
  // (7B shape, 7 query heads per KV head: 532 TFLOP/s with 16 positions against 377 with 32)
  const int G = n_q_heads / n_kv_heads;
  if (forced && (forced == 16 || G <= 8)) return forced;
  return G <= 6 ? 32 : 16;
}

hipError_t launch_attn_prefill(hipStream_t s, const f16* q, const AttnWork* work, int n_work,
                               SeqState st, const f16* arena_layer, KvGeom geom, int n_q_heads,
                               f16* out) {
  if (n_work <= 0 || !geom_ok(geom, n_q_heads)) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)geom.head_dim);
  const int G = n_q_heads / geom.n_kv_heads;
  const int tile = attn_prefill_tile_rows(n_q_heads, geom.n_kv_heads);
  const int rgw = ((tile / 16) * G + 3) / 4;           // row-groups per wave: 1 .. 4
  dim3 grid(n_work, geom.n_kv_heads);
#define AREAL_PF(DD, RR)                                                                          \
  attn_prefill_kernel<DD, RR><<<grid, 256, 0, s>>>(q, work, st, arena_layer, geom, n_q_heads, tile, \
                                                   scale_log2, out)
#define AREAL_PF_D(DD)                                                                            \
  switch (rgw) {                                                                                  \
    case 1: AREAL_PF(DD, 1); break;                                                               \
    case 2: AREAL_PF(DD, 2); break;                                                               \
    case 3: AREAL_PF(DD, 3); break;                                                               \
    default: AREAL_PF(DD, 4); break;                                                              \
  }
  switch (geom.head_dim) {
    case 32: AREAL_PF_D(32) break;
    case 64: AREAL_PF_D(64) break;
    default: AREAL_PF_D(128) break;
  }
#undef AREAL_PF_D
#undef AREAL_PF
  return hipGetLastError();
}

}  // namespace areal
