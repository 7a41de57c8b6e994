// Small HBM-bound kernels of the decoder block: token embedding, RMSNorm,
// rotary embedding + paged K/V store, parameter conversion to half precision.
#include "kernels.hpp"

namespace areal {

// h[r,:] = E[token(r),:] as float32.  In a decode step (tokens_in != null) the
// kernel also records the appended token in the history and installs the KV
// block the host reserved for a sequence that crossed a block boundary.
__global__ __launch_bounds__(256) void embed_kernel(const f16* __restrict__ E, int H, int V,
                                                    RowMeta rm, const int32_t* __restrict__ tokens_in,
                                                    const int32_t* __restrict__ new_block, SeqState st,
                                                    float* __restrict__ h) {
  const int r = blockIdx.x;
  const int slot = rm.slot[r], pos = rm.pos[r];
  int tok;
  int32_t* hp = st.hist + (int64_t)slot * st.max_seq_len + pos;
  if (tokens_in) {
    tok = tokens_in[r];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
    if (threadIdx.x == 0) *hp = tok;
  } else {
    tok = *hp;
  }
  if (new_block && threadIdx.x == 0) {
    int nb = new_block[r];
    if (nb >= 0) st.table[(int64_t)slot * st.max_blocks + pos / kBlockTokens] = nb;
  }
  const f16* src = E + (int64_t)tok * H;
  float* dst = h + (int64_t)r * H;
  for (int c = threadIdx.x * 8; c < H; c += 256 * 8) {
    f16x8 v = ld8(src + c);
    f32x4 a = {h2f(v[0]), h2f(v[1]), h2f(v[2]), h2f(v[3])};
    f32x4 b = {h2f(v[4]), h2f(v[5]), h2f(v[6]), h2f(v[7])};
    *reinterpret_cast<f32x4*>(dst + c) = a;
    *reinterpret_cast<f32x4*>(dst + c + 4) = b;
  }
}

hipError_t launch_embed(hipStream_t s, const f16* embed, int hidden, int vocab, int M, RowMeta rm,
                        const int32_t* tokens_in, const int32_t* new_block, SeqState st, float* h) {
  if (M <= 0 || hidden % 8 || vocab <= 0) return hipErrorInvalidValue;
  embed_kernel<<<M, 256, 0, s>>>(embed, hidden, vocab, rm, tokens_in, new_block, st, h);
  return hipGetLastError();
}

// y = x / sqrt(mean(x^2) + eps) * gain: one single-wave work-group per row (so
// that a decode batch spreads over all compute units), the row held in
// registers between the reduction and the scaling.  src_rows (optional)
// gathers: output row r is computed from input row src_rows[r].
template <int NV>   // float4 vectors per lane: hidden <= NV * 256
__global__ __launch_bounds__(64) void rmsnorm_kernel(const float* __restrict__ x,
                                                     const f16* __restrict__ gain, f16* __restrict__ y,
                                                     int H, float eps, const int32_t* __restrict__ src_rows,
                                                     float* __restrict__ zero_out, int zero_cols) {
  const int lane = threadIdx.x, row = blockIdx.x;
  const int src = src_rows ? src_rows[row] : row;
  const float* xp = x + (int64_t)src * H;
  f32x4 v[NV];
  f16x4 gn[NV];                       // the gains travel with the row: no second round trip after the sum
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 4;
    v[i] = c < H ? *reinterpret_cast<const f32x4*>(xp + c) : f32x4{0.f, 0.f, 0.f, 0.f};
    gn[i] = c < H ? *reinterpret_cast<const f16x4*>(gain + c) : f16x4{0, 0, 0, 0};
  }
#pragma unroll
  for (int i = 0; i < NV; ++i)
    ss += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
  if (zero_out) {
    float* zp = zero_out + (int64_t)row * zero_cols;
    const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
    for (int c = lane * 4; c < zero_cols; c += 256) *reinterpret_cast<f32x4*>(zp + c) = z4;
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
  f16* yp = y + (int64_t)row * H;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < H) {
      f16x4 o;
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = f2h_sat(v[i][k] * r * h2f(gn[i][k]));
      *reinterpret_cast<f16x4*>(yp + c) = o;
    }
  }
}

hipError_t launch_rmsnorm(hipStream_t s, const float* x, const f16* gain, f16* y, int M, int hidden,
                          float eps, const int32_t* src_rows, float* zero_out, int zero_cols) {
  if (M <= 0 || hidden % 4 || hidden > 32 * 256 || (zero_out && zero_cols % 4)) return hipErrorInvalidValue;
  if (hidden <= 2 * 256)
    rmsnorm_kernel<2><<<M, 64, 0, s>>>(x, gain, y, hidden, eps, src_rows, zero_out, zero_cols);
  else if (hidden <= 8 * 256)
    rmsnorm_kernel<8><<<M, 64, 0, s>>>(x, gain, y, hidden, eps, src_rows, zero_out, zero_cols);
  else if (hidden <= 16 * 256)
    rmsnorm_kernel<16><<<M, 64, 0, s>>>(x, gain, y, hidden, eps, src_rows, zero_out, zero_cols);
  else
    rmsnorm_kernel<32><<<M, 64, 0, s>>>(x, gain, y, hidden, eps, src_rows, zero_out, zero_cols);
  return hipGetLastError();
}

// Adds the optional QKV bias, rotates q and k heads (rotate-half pairing: dims
// j and j + d/2 turn by pos * theta^(-2j/d), angles from a host-built table),
// writes q as f16 [M, nq, d] and stores k, v into the sequence's KV block.
__global__ __launch_bounds__(256) void rope_kvwrite_kernel(
    const float* __restrict__ qkv, RowMeta rm, SeqState st, const f16* __restrict__ bq,
    const f16* __restrict__ bk, const f16* __restrict__ bv, const float* __restrict__ cos_tab,
    const float* __restrict__ sin_tab, f16* __restrict__ q_out, f16* __restrict__ arena_layer,
    KvGeom geom, int nq) {
  const int r = blockIdx.x;
  const int d = geom.head_dim, half = d >> 1, nkv = geom.n_kv_heads;
  const int slot = rm.slot[r], pos = rm.pos[r];
  const int blk = st.table[(int64_t)slot * st.max_blocks + pos / kBlockTokens];
  const int tin = pos % kBlockTokens;
  const int ld = (nq + 2 * nkv) * d;
  const float* row = qkv + (int64_t)r * ld;
  const float* ct = cos_tab + (int64_t)pos * half;
  const float* sn = sin_tab + (int64_t)pos * half;
  const int n_rot = (nq + nkv) * half;
  for (int idx = threadIdx.x; idx < n_rot; idx += 256) {
    const int head = idx / half, j = idx - head * half;
    float x1 = row[head * d + j], x2 = row[head * d + j + half];
    if (bq) {
      const f16* b = head < nq ? bq + head * d : bk + (head - nq) * d;
      x1 += h2f(b[j]);
      x2 += h2f(b[j + half]);
    }
    const float c = ct[j], sv = sn[j];
    const float y1 = x1 * c - x2 * sv, y2 = x2 * c + x1 * sv;
    if (head < nq) {
      f16* qo = q_out + ((int64_t)r * nq + head) * d;
      qo[j] = f2h_sat(y1);
      qo[j + half] = f2h_sat(y2);
    } else {
      f16* kt = arena_layer + kv_tile_off(geom, blk, head - nq, 0);
      kt[k_tile_index(tin, j)] = f2h_sat(y1);
      kt[k_tile_index(tin, j + half)] = f2h_sat(y2);
    }
  }
  const float* vrow = row + (nq + nkv) * d;
  for (int idx = threadIdx.x; idx < nkv * d; idx += 256) {
    const int kvh = idx / d, dim = idx - kvh * d;
    float v = vrow[idx];
    if (bv) v += h2f(bv[idx]);
    f16* vt = arena_layer + kv_tile_off(geom, blk, kvh, 1);
    vt[v_tile_index(d, tin, dim)] = f2h_sat(v);
  }
}

hipError_t launch_rope_kvwrite(hipStream_t s, const float* qkv, int M, RowMeta rm, SeqState st,
                               const f16* bq, const f16* bk, const f16* bv, const float* cos_tab,
                               const float* sin_tab, f16* q_out, f16* arena_layer, KvGeom geom,
                               int n_q_heads) {
  if (M <= 0 || geom.head_dim % 16 || (bq && (!bk || !bv))) return hipErrorInvalidValue;
  rope_kvwrite_kernel<<<M, 256, 0, s>>>(qkv, rm, st, bq, bk, bv, cos_tab, sin_tab, q_out, arena_layer,
                                        geom, n_q_heads);
  return hipGetLastError();
}

// A sampled token joins its sequence without a forward pass (the weights change before
// the pass that would have taken it as input): history entry and, at a block start, the
// block the host reserved.
__global__ __launch_bounds__(256) void append_kernel(int n, int V, RowMeta rm,
                                                     const int32_t* __restrict__ tokens_in,
                                                     const int32_t* __restrict__ new_block, SeqState st) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= n) return;
  const int slot = rm.slot[r], pos = rm.pos[r];
  int tok = tokens_in[r];
  tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
  st.hist[(int64_t)slot * st.max_seq_len + pos] = tok;
  const int nb = new_block[r];
  if (nb >= 0) st.table[(int64_t)slot * st.max_blocks + pos / kBlockTokens] = nb;
}
hipError_t launch_append(hipStream_t s, int n, int vocab, RowMeta rm, const int32_t* tokens_in,
                         const int32_t* new_block, SeqState st) {
  if (n <= 0 || vocab <= 0 || !tokens_in || !new_block) return hipErrorInvalidValue;
  append_kernel<<<(n + 255) / 256, 256, 0, s>>>(n, vocab, rm, tokens_in, new_block, st);
  return hipGetLastError();
}

// Prompt-prefix sharing: block-table entries of sequences that start out holding
// another sequence's blocks ({slot, index, block} triples), and the copy of the
// shared part of the token history ({dst slot, src slot, n tokens} triples).
__global__ __launch_bounds__(256) void table_patch_kernel(const int32_t* __restrict__ patch, int n,
                                                          SeqState st) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) st.table[(int64_t)patch[3 * i] * st.max_blocks + patch[3 * i + 1]] = patch[3 * i + 2];
}
__global__ __launch_bounds__(256) void hist_copy_kernel(const int32_t* __restrict__ job, SeqState st) {
  const int dst = job[3 * blockIdx.x], src = job[3 * blockIdx.x + 1], n = job[3 * blockIdx.x + 2];
  const int32_t* s = st.hist + (int64_t)src * st.max_seq_len;
  int32_t* d = st.hist + (int64_t)dst * st.max_seq_len;
  for (int t = threadIdx.x; t < n; t += 256) d[t] = s[t];
}
hipError_t launch_table_patch(hipStream_t s, const int32_t* patch, int n, SeqState st) {
  if (n <= 0 || !patch) return hipErrorInvalidValue;
  table_patch_kernel<<<(n + 255) / 256, 256, 0, s>>>(patch, n, st);
  return hipGetLastError();
}
hipError_t launch_hist_copy(hipStream_t s, const int32_t* jobs, int n, SeqState st) {
  if (n <= 0 || !jobs) return hipErrorInvalidValue;
  hist_copy_kernel<<<n, 256, 0, s>>>(jobs, st);
  return hipGetLastError();
}

// Per-pass metadata travels from the pinned host ring to its device mirror in a
// kernel of the library's own (16-byte words; src is device-mapped host memory).
__global__ __launch_bounds__(256) void stage_copy_kernel(const u32x4* __restrict__ src,
                                                         u32x4* __restrict__ dst, int n16) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

hipError_t launch_stage_copy(hipStream_t s, const void* src_host_mapped, void* dst, size_t bytes) {
  if (!src_host_mapped || !dst || bytes == 0 || bytes % 16 || ((uintptr_t)src_host_mapped & 15) ||
      ((uintptr_t)dst & 15) || bytes > (size_t)1 << 30)
    return hipErrorInvalidValue;
  const int n16 = (int)(bytes / 16);
  stage_copy_kernel<<<(n16 + 255) / 256, 256, 0, s>>>(reinterpret_cast<const u32x4*>(src_host_mapped),
                                                      reinterpret_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

// Calibration: a read of `n16` 16-byte words that does nothing else (one work-group per 64 KiB,
// eight loads in flight per lane), the yardstick for the kernels that stream K/V or weights.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16,
                                                          uint32_t never, u32x4* __restrict__ sink) {
  constexpr int PER_WG = 4096;                        // 16-byte words per work-group
  const int64_t w0 = (int64_t)blockIdx.x * PER_WG;
  u32x4 acc = {0, 0, 0, 0};
  for (int q = 0; q < PER_WG; q += 256 * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int64_t i = w0 + q + u * 256 + threadIdx.x;
      v[u] = i < n16 ? src[i] : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  // `never` is a value the xor of the data does not take (the caller's choice): keeps the loads alive
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == never && never != 0) *sink = acc;
}

hipError_t launch_stream_read(hipStream_t s, const void* src, size_t bytes, uint32_t never, void* sink16) {
  if (!src || !sink16 || bytes == 0 || bytes % 16 || ((uintptr_t)src & 15) || ((uintptr_t)sink16 & 15) ||
      bytes > (size_t)1 << 36)
    return hipErrorInvalidValue;
  const int64_t n16 = (int64_t)(bytes / 16);
  stream_read_kernel<<<(unsigned)((n16 + 4095) / 4096), 256, 0, s>>>(reinterpret_cast<const u32x4*>(src), n16, never,
                                                                       reinterpret_cast<u32x4*>(sink16));
  return hipGetLastError();
}

// Parameter sets arrive as float32 or bf16 and are held as halves for the
// matrix cores (round to nearest even; bf16 values with |w| >= 2^-14 convert
// exactly).  Magnitudes beyond the half range saturate to +-65504.
template <typename SRC>
__global__ __launch_bounds__(256) void to_f16_kernel(const SRC* __restrict__ src, f16* __restrict__ dst,
                                                     int64_t n) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    float v = (float)src[i];
    v = fminf(fmaxf(v, -65504.0f), 65504.0f);
    dst[i] = f2h(v);
  }
}

hipError_t launch_to_f16(hipStream_t s, const void* src, int src_is_bf16, f16* dst, int64_t n) {
  if (n <= 0 || !src || !dst) return hipErrorInvalidValue;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (src_is_bf16)
    to_f16_kernel<bf16_in><<<(int)blocks, 256, 0, s>>>(reinterpret_cast<const bf16_in*>(src), dst, n);
  else
    to_f16_kernel<float><<<(int)blocks, 256, 0, s>>>(reinterpret_cast<const float*>(src), dst, n);
  return hipGetLastError();
}

}  // namespace areal
