// Host runtime behind include/areal.h: context, sequence table, per-pass
// metadata staging, kernel sequencing of one decoder forward pass, and the
// five boundary calls.  All device work goes to the caller's stream.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/areal.h"
#include "../../include/areal_host.h"
#include "../../include/areal_ops.h"
#include "kernels.hpp"
#include <unordered_map>
#include <unordered_set>

#include "kv_alloc.hpp"
#include "gate.hpp"

using namespace areal;

namespace {

constexpr int kMaxSplits = 32;
constexpr int kRingSegs = 8;

thread_local std::string g_create_error;

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

struct Layout {                     // byte offsets into the workspace
  uint64_t h, xn, qkv, q, attn, act, xlast, part_o, part_ml, hist, table, cos_t, sin_t, ring, samp, wconv,
      total;
  uint64_t ring_bytes, wconv_elems;
  int max_blocks;
};

bool cfg_valid(const areal_model_cfg* c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (!c) return bad("cfg is NULL");
  if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->ffn <= 0 ||
      c->vocab <= 0)
    return bad("non-positive model dimension");
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 32, 64 or 128");
  if (c->n_q_heads % c->n_kv_heads || c->n_q_heads / c->n_kv_heads > 16)
    return bad("n_q_heads must be a multiple of n_kv_heads with at most 16 query heads per KV head");
  if (c->hidden % 8 || c->ffn % 8) return bad("hidden and ffn must be multiples of 8");
  if (c->hidden > 8192) return bad("hidden above 8192");
  if ((int64_t)c->vocab > 262144) return bad("vocab above 262144");
  if (c->max_seqs <= 0 || c->max_seq_len <= 0 || c->max_batch_tokens < c->max_seqs)
    return bad("need max_seqs > 0, max_seq_len > 0, max_batch_tokens >= max_seqs");
  if (c->max_seq_len > kMaxSplits * 2048) return bad("max_seq_len above 65536");
  if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return bad("bad rope_theta / rms_eps");
  return true;
}

uint64_t total_params(const areal_model_cfg& c) {
  const uint64_t H = c.hidden, F = c.ffn, qd = (uint64_t)c.n_q_heads * c.head_dim,
                 kd = (uint64_t)c.n_kv_heads * c.head_dim, V = c.vocab;
  const uint64_t per_layer = qd * H + 2 * kd * H + H * qd + 2 * F * H + H * F + 2 * H + qd + 2 * kd;
  return 2 * V * H + H + (uint64_t)c.n_layers * per_layer + 64 * (uint64_t)(c.n_layers * 12 + 3);
}

Layout make_layout(const areal_model_cfg& c) {
  Layout L{};
  const uint64_t M = c.max_batch_tokens, H = c.hidden, d = c.head_dim;
  const uint64_t qd = (uint64_t)c.n_q_heads * d, kd = (uint64_t)c.n_kv_heads * d;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes, 256); return o; };
  L.h = take(M * H * 4);
  L.xn = take(M * H * 2);
  L.qkv = take(M * (qd + 2 * kd) * 4);
  L.q = take(M * qd * 2);
  L.attn = take(M * qd * 2);
  L.act = take(M * (uint64_t)c.ffn * 2);
  L.xlast = take((uint64_t)c.max_seqs * H * 2);
  L.part_o = take((uint64_t)c.max_seqs * c.n_q_heads * kMaxSplits * d * 4);
  L.part_ml = take((uint64_t)c.max_seqs * c.n_q_heads * kMaxSplits * 2 * 4);
  L.max_blocks = (c.max_seq_len + AREAL_KV_BLOCK_TOKENS - 1) / AREAL_KV_BLOCK_TOKENS;
  L.hist = take((uint64_t)c.max_seqs * c.max_seq_len * 4);
  L.table = take((uint64_t)c.max_seqs * L.max_blocks * 4);
  L.cos_t = take((uint64_t)c.max_seq_len * (d / 2) * 4);
  L.sin_t = take((uint64_t)c.max_seq_len * (d / 2) * 4);
  // per pass: slot, pos, token, new_block per row + work items + last rows
  // (+ in a decode step the block ids of every row's sequence, laid out by row)
  const uint64_t per_pass = M * 16 + (M / 16 + 2 * (uint64_t)c.max_seqs + 64) * 16 + (uint64_t)c.max_seqs * 16 +
                            (uint64_t)c.max_seqs * (L.max_blocks + 4) * 4 +
                            // decode step: t_start per row, tile rows and start per set, block ids per set
                            (uint64_t)c.max_seqs * (4 + (kGroupTiles * 16 * 4 + 4 + (L.max_blocks + 4) * 4) / 2) + 256;
  L.ring_bytes = align_up(std::max<uint64_t>(per_pass * 2, 1u << 20), 4096) * kRingSegs;
  L.ring = take(L.ring_bytes);
  L.samp = take(sampler_scratch_bytes());
  L.wconv_elems = c.convert_weights ? total_params(c) : 0;
  L.wconv = take(L.wconv_elems * 2);
  L.total = off;
  return L;
}

struct SeqInfo {
  bool live = false;
  int32_t len = 0;
  int32_t kv_len = 0;                   // positions whose K/V is in the cache (< len after areal_append_tokens)
  int32_t n_shared = 0;                 // leading KV blocks held together with other sequences
  int64_t pending_version = 0;          // version whose logits the next token is sampled from
  std::vector<int64_t> versions;        // per position; -1 = prompt
};

struct WeightSet {
  const f16 *embed = nullptr, *lm_head = nullptr, *final_norm = nullptr;
  std::vector<const f16*> wq, wk, wv, wo, wgate, wup, wdown, norm_attn, norm_ffn, bq, bk, bv;
  bool has_bias = false;
};

}  // namespace

namespace areal {
void set_global_error(const std::string& msg) { g_create_error = msg; }
}  // namespace areal

struct areal_ctx {
  areal_model_cfg cfg;
  Layout lay;
  hipStream_t stream;
  char* ws;
  KvGeom geom;
  int64_t n_blocks;
  KvAllocator* alloc = nullptr;
  std::vector<SeqInfo> seqs;
  // prompts of the live sequences admitted by areal_prefill (host copies) and an index by
  // prompt hash: a later call finds the live sequences that already hold a prompt's blocks
  std::vector<std::vector<int32_t>> prompt_of;
  std::vector<uint64_t> prompt_hash_of;
  std::unordered_map<uint64_t, std::vector<int32_t>> prompt_index;
  WeightSet w;
  bool have_weights = false;
  int64_t version = 0;
  // metadata ring: pinned host mirror of a device ring, reused segment by segment
  char* ring_host = nullptr;
  char* ring_host_dev = nullptr;        // the same pinned memory as the device addresses it
  uint64_t seg_bytes = 0, seg_used = 0;
  int seg = 0;
  hipEvent_t seg_done[kRingSegs];
  bool seg_recorded[kRingSegs];
  std::string err;
  int split_target = 3072;              // decode attention: work-groups per launch aimed at
  int min_chunk = 256;
  // Decode attention can walk the leading blocks that rows share once per set of rows: 1 = whenever
  // rows share, 0 = never, -1 = when the shared part is most of what the launch reads (measured on
  // the MI355X: 7-9 % off the attention launch where 80 % of the context tokens read are shared, a
  // loss of 2-12 % where it is a quarter or less: the repeated reads of a block already meet in L2,
  // and the extra partial slots cost the merge more than the rows' own walks save)
  int group_decode = -1;
  int64_t set_rows_sum = 0, set_row_tokens_sum = 0, set_tokens_sum = 0;
  bool fused_scoring = true;            // scoring passes fold the log-sum-exp into the output projection
  // measurement hook
  int prof_class = -1, prof_layer = 0, prof_every = 1;
  int64_t prof_pass = 0;
  double prof_units = 0.0;
  std::vector<hipEvent_t> prof_events;      // start/stop pairs
  size_t prof_used = 0;

  template <class T> T* wsp(uint64_t off) const { return reinterpret_cast<T*>(ws + off); }
  SeqState seq_state() const {
    return SeqState{wsp<int32_t>(lay.hist), wsp<int32_t>(lay.table), cfg.max_seq_len, lay.max_blocks};
  }
};

namespace {

int fail(areal_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}
#define HIP_TRY(ctx, expr)                                                                        \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess)                                                                         \
      return fail(ctx, AREAL_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));           \
  } while (0)

// ---- metadata staging -------------------------------------------------------
// Reserve `bytes` in the ring (host pointer returned, device address in *dev).
// A pass stages everything it needs, then calls ring_flush once.
struct Staged { char* host; char* dev; };

int ring_begin(areal_ctx* c, uint64_t bytes_needed) {
  if (bytes_needed > c->seg_bytes) return fail(c, AREAL_E_NOMEM, "metadata for one pass exceeds a ring segment");
  if (c->seg_used + bytes_needed > c->seg_bytes) {
    HIP_TRY(c, hipEventRecord(c->seg_done[c->seg], c->stream));
    c->seg_recorded[c->seg] = true;
    c->seg = (c->seg + 1) % kRingSegs;
    c->seg_used = 0;
    if (c->seg_recorded[c->seg]) HIP_TRY(c, hipEventSynchronize(c->seg_done[c->seg]));
  }
  return AREAL_OK;
}
Staged ring_take(areal_ctx* c, uint64_t bytes) {
  const uint64_t off = (uint64_t)c->seg * c->seg_bytes + c->seg_used;
  c->seg_used += align_up(bytes, 64);
  return Staged{c->ring_host + off, c->ws + c->lay.ring + off};
}
int ring_flush(areal_ctx* c, uint64_t start_used) {
  const uint64_t off = (uint64_t)c->seg * c->seg_bytes + start_used;
  const uint64_t n = c->seg_used - start_used;
  if (n == 0) return AREAL_OK;
  HIP_TRY(c, launch_stage_copy(c->stream, c->ring_host_dev + off, c->ws + c->lay.ring + off, n));
  return AREAL_OK;
}

// ---- weights ----------------------------------------------------------------
bool weights_complete(const areal_ctx* c, const areal_weights* w) {
  if (!w || !w->embed || !w->lm_head || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
      !w->wgate || !w->wup || !w->wdown || !w->norm_attn || !w->norm_ffn)
    return false;
  const bool bias = w->bq || w->bk || w->bv;
  if (bias && !(w->bq && w->bk && w->bv)) return false;
  for (int l = 0; l < c->cfg.n_layers; ++l) {
    if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->wgate[l] || !w->wup[l] ||
        !w->wdown[l] || !w->norm_attn[l] || !w->norm_ffn[l])
      return false;
    if (bias && (!w->bq[l] || !w->bk[l] || !w->bv[l])) return false;
  }
  return true;
}

// Install `w` as the current parameter set (half: borrow in place; bf16 / f32:
// convert into the workspace copy, stream-ordered after all earlier passes).
int install_weights(areal_ctx* c, const areal_weights* w) {
  const areal_model_cfg& g = c->cfg;
  const int L = g.n_layers;
  const uint64_t H = g.hidden, F = g.ffn, qd = (uint64_t)g.n_q_heads * g.head_dim,
                 kd = (uint64_t)g.n_kv_heads * g.head_dim, V = g.vocab;
  WeightSet ws;
  ws.has_bias = w->bq != nullptr;
  uint64_t cursor = 0;
  hipError_t herr = hipSuccess;
  auto get = [&](const void* p, uint64_t n) -> const f16* {
    if (w->dtype == AREAL_DTYPE_F16) return reinterpret_cast<const f16*>(p);
    f16* dst = c->wsp<f16>(c->lay.wconv) + cursor;
    cursor += align_up(n, 64);
    if (herr == hipSuccess) herr = launch_to_f16(c->stream, p, w->dtype == AREAL_DTYPE_BF16, dst, (int64_t)n);
    return dst;
  };
  const bool tied = w->lm_head == w->embed;
  ws.embed = get(w->embed, V * H);
  ws.lm_head = tied ? ws.embed : get(w->lm_head, V * H);
  ws.final_norm = get(w->final_norm, H);
  for (int l = 0; l < L; ++l) {
    ws.wq.push_back(get(w->wq[l], qd * H));
    ws.wk.push_back(get(w->wk[l], kd * H));
    ws.wv.push_back(get(w->wv[l], kd * H));
    ws.wo.push_back(get(w->wo[l], H * qd));
    ws.wgate.push_back(get(w->wgate[l], F * H));
    ws.wup.push_back(get(w->wup[l], F * H));
    ws.wdown.push_back(get(w->wdown[l], H * F));
    ws.norm_attn.push_back(get(w->norm_attn[l], H));
    ws.norm_ffn.push_back(get(w->norm_ffn[l], H));
    if (ws.has_bias) {
      ws.bq.push_back(get(w->bq[l], qd));
      ws.bk.push_back(get(w->bk[l], kd));
      ws.bv.push_back(get(w->bv[l], kd));
    }
  }
  if (herr != hipSuccess) return fail(c, AREAL_E_HIP, std::string("weight conversion: ") + hipGetErrorString(herr));
  c->w = std::move(ws);
  c->have_weights = true;
  return AREAL_OK;
}

int check_weights_arg(areal_ctx* c, const areal_weights* w) {
  if (!weights_complete(c, w)) return fail(c, AREAL_E_INVAL, "incomplete weight set");
  if (w->dtype != AREAL_DTYPE_BF16 && w->dtype != AREAL_DTYPE_F32 && w->dtype != AREAL_DTYPE_F16)
    return fail(c, AREAL_E_INVAL, "unknown weight dtype");
  if (w->dtype != AREAL_DTYPE_F16 && !c->cfg.convert_weights)
    return fail(c, AREAL_E_INVAL, "bf16 / float32 weights need cfg.convert_weights = 1 at creation");
  return AREAL_OK;
}

// ---- measurement hook ---------------------------------------------------------
struct ProfScope {
  areal_ctx* c;
  bool on;
  ProfScope(areal_ctx* c_, int klass, int layer, bool pass_sampled, double units) : c(c_), on(false) {
    if (c->prof_class != klass || !pass_sampled || (layer >= 0 && layer != c->prof_layer)) return;
    if (c->prof_used + 2 > c->prof_events.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
      c->prof_events.push_back(a);
      c->prof_events.push_back(b);
    }
    on = hipEventRecord(c->prof_events[c->prof_used], c->stream) == hipSuccess;
    if (on) c->prof_units += units;
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(c->prof_events[c->prof_used + 1], c->stream);
    c->prof_used += 2;
  }
};

// ---- one forward pass -------------------------------------------------------
struct PassArgs {
  int M;                          // rows
  RowMeta rm;                     // device
  const int32_t* tokens_in;       // device or null (read history)
  const int32_t* new_block;       // device or null
  bool decode;
  int chunk, n_splits;            // decode attention partition
  const AttnWork* work;           // prefill attention work list (device)
  int n_work;
  const int32_t* last_rows;       // device: rows feeding the output projection (null: all rows)
  int n_out;                      // logits rows produced
  float* logits;                  // device [n_out, vocab]
  double attn_units;              // context tokens read (decode) / query-key pairs (prefill)
  const int32_t* step_table = nullptr;   // decode: block ids by launch row (device), row stride below
  int step_stride = 0;
  DecodeGroups groups;                   // decode: sets of rows that share leading blocks
  // scoring passes (teacher-forced log-probs of every row's next token)
  const int32_t* target = nullptr;   // device [M]: token each row predicts, -1 = none
  float inv_t = 1.f;
  float* scratch = nullptr;          // device float32 [scratch_rows, vocab]
  int scratch_rows = 0;
  float* logp = nullptr;             // device: entry of row 0 in the packed output
};

int run_pass(areal_ctx* c, const PassArgs& a) {
  const areal_model_cfg& g = c->cfg;
  const int H = g.hidden, F = g.ffn, nq = g.n_q_heads, nkv = g.n_kv_heads, d = g.head_dim;
  const int qd = nq * d, kd = nkv * d;
  hipStream_t s = c->stream;
  SeqState st = c->seq_state();
  float* h = c->wsp<float>(c->lay.h);
  f16* xn = c->wsp<f16>(c->lay.xn);
  float* qkv = c->wsp<float>(c->lay.qkv);
  f16* q = c->wsp<f16>(c->lay.q);
  f16* attn = c->wsp<f16>(c->lay.attn);
  f16* act = c->wsp<f16>(c->lay.act);
  f16* xlast = c->wsp<f16>(c->lay.xlast);
  const float* cos_t = c->wsp<float>(c->lay.cos_t);
  const float* sin_t = c->wsp<float>(c->lay.sin_t);
  f16* arena = reinterpret_cast<f16*>(g.kv_arena);
  const WeightSet& w = c->w;

  const bool sampled = c->prof_class >= 0 && (c->prof_pass++ % c->prof_every) == 0;
  const double rows = a.M;
  {
    ProfScope ps(c, AREAL_K_EMBED, -1, sampled, rows);
    HIP_TRY(c, launch_embed(s, w.embed, H, g.vocab, a.M, a.rm, a.tokens_in, a.new_block, st, h));
  }
  for (int l = 0; l < g.n_layers; ++l) {
    f16* arena_l = arena + (int64_t)l * c->geom.layer_stride;
    {
      ProfScope ps(c, AREAL_K_RMSNORM, l, sampled, rows);
      // the QKV product may split K and accumulate atomically: then its output is cleared here
      int qkv_cfg, qkv_splits;
      gemm_choose(a.M, qd + 2 * kd, H, GEMM_STORE_F32, &qkv_cfg, &qkv_splits);
      HIP_TRY(c, launch_rmsnorm(s, h, w.norm_attn[l], xn, a.M, H, g.rms_eps, nullptr,
                                qkv_splits > 1 ? qkv : nullptr, qd + 2 * kd));
    }
    {
      ProfScope ps(c, AREAL_K_GEMM_QKV, l, sampled, rows);
      GemmW wqkv{{w.wq[l], w.wk[l], w.wv[l]}, {qd, qd + kd, qd + 2 * kd}};
      HIP_TRY(c, launch_gemm_cfg(s, xn, wqkv, qkv, a.M, qd + 2 * kd, H, qd + 2 * kd, GEMM_STORE_F32, -1, -1));
    }
    const f16 *bq = w.has_bias ? w.bq[l] : nullptr, *bk = w.has_bias ? w.bk[l] : nullptr,
              *bv = w.has_bias ? w.bv[l] : nullptr;
    if (a.decode) {
      // bias, RoPE and the store of the appended K/V are part of the attention kernel
      {
        ProfScope ps(c, AREAL_K_ATTN_DECODE, l, sampled, a.attn_units);
        HIP_TRY(c, launch_attn_decode(s, qkv, a.M, a.rm, st, bq, bk, bv, cos_t, sin_t, arena_l, c->geom, nq,
                                      a.chunk, a.n_splits, c->wsp<float>(c->lay.part_o),
                                      c->wsp<float>(c->lay.part_ml), attn, a.step_table, a.step_stride,
                                      a.groups));
      }
      if (a.n_splits + a.groups.n_shared > 1) {
        ProfScope ps(c, AREAL_K_ATTN_MERGE, l, sampled, rows);
        HIP_TRY(c, launch_attn_merge(s, a.M, a.rm, d, nq, a.chunk, a.n_splits, c->wsp<float>(c->lay.part_o),
                                     c->wsp<float>(c->lay.part_ml), attn, a.groups));
      }
    } else {
      {
        ProfScope ps(c, AREAL_K_ROPE_KVWRITE, l, sampled, rows);
        HIP_TRY(c, launch_rope_kvwrite(s, qkv, a.M, a.rm, st, bq, bk, bv, cos_t, sin_t, q, arena_l, c->geom, nq));
      }
      ProfScope ps(c, AREAL_K_ATTN_PREFILL, l, sampled, a.attn_units);
      HIP_TRY(c, launch_attn_prefill(s, q, a.work, a.n_work, st, arena_l, c->geom, nq, attn));
    }
    {
      ProfScope ps(c, AREAL_K_GEMM_O, l, sampled, rows);
      GemmW wo{{w.wo[l], nullptr, nullptr}, {H, 0, 0}};
      HIP_TRY(c, launch_gemm_cfg(s, attn, wo, h, a.M, H, qd, H, GEMM_ADD_F32, -1, -1));
    }
    HIP_TRY(c, launch_rmsnorm(s, h, w.norm_ffn[l], xn, a.M, H, g.rms_eps, nullptr));
    {
      ProfScope ps(c, AREAL_K_GEMM_GATEUP, l, sampled, rows);
      GemmW wgu{{w.wgate[l], w.wup[l], nullptr}, {F, 0, 0}};
      HIP_TRY(c, launch_gemm_cfg(s, xn, wgu, act, a.M, F, H, F, GEMM_SWIGLU_F16, -1, -1));
    }
    {
      ProfScope ps(c, AREAL_K_GEMM_DOWN, l, sampled, rows);
      GemmW wd{{w.wdown[l], nullptr, nullptr}, {H, 0, 0}};
      HIP_TRY(c, launch_gemm_cfg(s, act, wd, h, a.M, H, F, H, GEMM_ADD_F32, -1, -1));
    }
  }
  if (a.target) {
    HIP_TRY(c, launch_rmsnorm(s, h, w.final_norm, xn, a.M, H, g.rms_eps, nullptr));
    GemmW wl{{w.lm_head, nullptr, nullptr}, {g.vocab, 0, 0}};
    if (c->fused_scoring && H % 64 == 0) {
      // Fused: the output projection keeps no logits at all, only a (max, sum of exponentials)
      // pair per row and column tile and the value at the row's target column, all inside the
      // caller's scratch; as many rows per launch as their pairs fit there.
      const int64_t floats = (int64_t)a.scratch_rows * g.vocab;
      auto cap = [&](int bn) { return floats / (2 * (int64_t)((g.vocab + bn - 1) / bn) + 1); };
      for (int r0 = 0; r0 < a.M;) {
        const int remaining = a.M - r0;
        int rows_now;
        if (remaining > 256 && cap(256) >= 512) rows_now = (int)std::min<int64_t>(remaining, cap(256));
        else rows_now = (int)std::min<int64_t>(std::min(remaining, 256), cap(128));
        const int n_tiles = gemm_lse_tiles(rows_now, g.vocab);
        float* tz = a.scratch + (int64_t)2 * n_tiles * rows_now;
        {
          ProfScope ps(c, AREAL_K_GEMM_LMHEAD, -1, sampled, (double)rows_now);
          HIP_TRY(c, launch_gemm_lse(s, xn + (int64_t)r0 * H, wl, rows_now, g.vocab, H, a.scratch, rows_now,
                                     GemmLse{a.target + r0, tz, a.inv_t}));
        }
        HIP_TRY(c, launch_lse_finish(s, a.scratch, rows_now, n_tiles, tz, a.target + r0, a.rm.pos + r0, rows_now,
                                     a.logp + r0));
        r0 += rows_now;
      }
    } else {
      // every row feeds the output projection, scratch_rows rows at a time: the
      // [M, vocab] logits never exist as a whole
      for (int r0 = 0; r0 < a.M; r0 += a.scratch_rows) {
        const int rows_now = std::min(a.scratch_rows, a.M - r0);
        {
          ProfScope ps(c, AREAL_K_GEMM_LMHEAD, -1, sampled, (double)rows_now);
          HIP_TRY(c, launch_gemm(s, xn + (int64_t)r0 * H, wl, a.scratch, rows_now, g.vocab, H, g.vocab,
                                 GEMM_STORE_F32));
        }
        HIP_TRY(c, launch_token_logprob(s, a.scratch, rows_now, g.vocab, a.inv_t, a.target + r0, a.rm.pos + r0,
                                        a.logp + r0));
      }
    }
  }
  if (a.n_out > 0) {
    HIP_TRY(c, launch_rmsnorm(s, h, w.final_norm, xlast, a.n_out, H, g.rms_eps, a.last_rows));
    ProfScope ps(c, AREAL_K_GEMM_LMHEAD, -1, sampled, (double)a.n_out);
    GemmW wl{{w.lm_head, nullptr, nullptr}, {g.vocab, 0, 0}};
    HIP_TRY(c, launch_gemm(s, xlast, wl, a.logits, a.n_out, g.vocab, H, g.vocab, GEMM_STORE_F32));
  }
  return AREAL_OK;
}

// Prefill-style passes over `spans` (prompt tokens given, or history re-read when
// tokens == null).  install_blocks: rows at block starts install their block id.
struct ScoreArgs {                // scoring: spans are consecutive sequences of one packed token array
  float inv_t;
  float* scratch;
  int scratch_rows;
  float* logp_out;                // device [total tokens], packed like `tokens`
};

int run_spans(areal_ctx* c, const std::vector<Span>& spans, const int32_t* tokens,
              const std::vector<int64_t>& tok_offset, bool install_blocks, float* logits_out,
              const ScoreArgs* score = nullptr) {
  const areal_model_cfg& g = c->cfg;
  auto passes = plan_passes(spans, g.max_batch_tokens);
  const int tile_rows = attn_prefill_tile_rows(g.n_q_heads, g.n_kv_heads);
  // span index lookup for token offsets: pieces come in span order
  size_t span_i = 0;
  int done_in_span = 0;
  for (auto& pass : passes) {
    int M = 0, n_work = 0, n_out = 0;
    for (auto& p : pass) {
      M += p.len;
      n_work += (p.len + tile_rows - 1) / tile_rows;
      if (p.out_index >= 0) ++n_out;
    }
    if (score) n_out = 0;                                 // no last-row logits
    const uint64_t bytes = align_up((uint64_t)M * 4, 64) * 5 + align_up((uint64_t)n_work * sizeof(AttnWork), 64) +
                           align_up((uint64_t)std::max(n_out, 1) * 4, 64);
    int rc = ring_begin(c, bytes);
    if (rc) return rc;
    const uint64_t start = c->seg_used;
    Staged s_slot = ring_take(c, (uint64_t)M * 4), s_pos = ring_take(c, (uint64_t)M * 4);
    Staged s_tok = ring_take(c, (uint64_t)M * 4), s_nb = ring_take(c, (uint64_t)M * 4);
    Staged s_work = ring_take(c, (uint64_t)n_work * sizeof(AttnWork));
    Staged s_last = ring_take(c, (uint64_t)std::max(n_out, 1) * 4);
    Staged s_tgt = ring_take(c, (uint64_t)M * 4);
    int32_t* htgt = (int32_t*)s_tgt.host;
    int64_t pass_base = -1;                               // packed index of the pass's row 0
    int32_t *hslot = (int32_t*)s_slot.host, *hpos = (int32_t*)s_pos.host, *htok = (int32_t*)s_tok.host,
            *hnb = (int32_t*)s_nb.host, *hlast = (int32_t*)s_last.host;
    AttnWork* hwork = (AttnWork*)s_work.host;
    int wi = 0, oi = 0, first_out = -1;
    double qk_pairs = 0.0;
    for (auto& p : pass) {
      qk_pairs += (double)p.len * p.pos0 + 0.5 * (double)p.len * (p.len + 1);
      const auto& blocks = c->alloc->blocks(p.slot);
      for (int r = 0; r < p.len; ++r) {
        const int pos = p.pos0 + r;
        hslot[p.row0 + r] = p.slot;
        hpos[p.row0 + r] = pos;
        if (tokens) htok[p.row0 + r] = tokens[tok_offset[span_i] + done_in_span + r];
        if (score) {
          const int64_t gi = tok_offset[span_i] + done_in_span + r;
          if (pass_base < 0) pass_base = gi - (p.row0 + r);
          htgt[p.row0 + r] = pos + 1 < spans[span_i].len ? tokens[gi + 1] : -1;
        }
        hnb[p.row0 + r] = (install_blocks && pos % AREAL_KV_BLOCK_TOKENS == 0) ? blocks[pos / AREAL_KV_BLOCK_TOKENS] : -1;
      }
      for (int r = 0; r < p.len; r += tile_rows)
        hwork[wi++] = AttnWork{p.slot, p.row0 + r, p.pos0 + r, std::min(tile_rows, p.len - r)};
      done_in_span += p.len;
      if (p.out_index >= 0) {
        if (first_out < 0) first_out = p.out_index;
        if (!score) hlast[oi++] = p.row0 + p.len - 1;
        ++span_i;
        done_in_span = 0;
      }
    }
    rc = ring_flush(c, start);
    if (rc) return rc;
    PassArgs a{};
    a.M = M;
    a.rm = RowMeta{(const int32_t*)s_slot.dev, (const int32_t*)s_pos.dev};
    a.tokens_in = tokens ? (const int32_t*)s_tok.dev : nullptr;
    a.new_block = install_blocks ? (const int32_t*)s_nb.dev : nullptr;
    a.decode = false;
    a.work = (const AttnWork*)s_work.dev;
    a.n_work = n_work;
    a.last_rows = (const int32_t*)s_last.dev;
    a.n_out = n_out;
    a.logits = n_out > 0 ? logits_out + (int64_t)first_out * g.vocab : nullptr;
    a.attn_units = qk_pairs;
    if (score) {
      a.target = (const int32_t*)s_tgt.dev;
      a.inv_t = score->inv_t;
      a.scratch = score->scratch;
      a.scratch_rows = score->scratch_rows;
      a.logp = score->logp_out + pass_base;
    }
    rc = run_pass(c, a);
    if (rc) return rc;
  }
  return AREAL_OK;
}

// Send `n` int32 triples through the metadata ring (in as many segments as it takes) and run
// `launch` on each staged chunk.
template <class F>
int stage_triples(areal_ctx* c, const std::vector<int32_t>& tri, F launch) {
  const size_t n = tri.size() / 3;
  const size_t per_seg = (size_t)(c->seg_bytes / 64) * 64 / 12;
  for (size_t i = 0; i < n; i += per_seg) {
    const size_t k = std::min(per_seg, n - i);
    int rc = ring_begin(c, align_up(k * 12, 64));
    if (rc) return rc;
    const uint64_t start = c->seg_used;
    Staged st = ring_take(c, k * 12);
    memcpy(st.host, tri.data() + 3 * i, k * 12);
    rc = ring_flush(c, start);
    if (rc) return rc;
    HIP_TRY(c, launch((const int32_t*)st.dev, (int)k));
  }
  return AREAL_OK;
}

}  // namespace

// ============================================================== C boundary ===
extern "C" {

uint64_t areal_workspace_bytes(const areal_model_cfg* cfg) {
  if (!cfg_valid(cfg, nullptr)) return 0;
  return make_layout(*cfg).total;
}

uint64_t areal_kv_block_bytes(const areal_model_cfg* cfg) {
  if (!cfg_valid(cfg, nullptr)) return 0;
  return (uint64_t)cfg->n_layers * cfg->n_kv_heads * 2 * AREAL_KV_BLOCK_TOKENS * cfg->head_dim * 2;
}

const char* areal_last_error(const areal_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int areal_create(const areal_model_cfg* cfg, areal_ctx** out) {
  std::string why;
  if (!out) return fail(nullptr, AREAL_E_INVAL, "out is NULL");
  *out = nullptr;
  if (!cfg_valid(cfg, &why)) return fail(nullptr, AREAL_E_INVAL, why);
  Layout lay = make_layout(*cfg);
  if (!cfg->workspace || ((uintptr_t)cfg->workspace & 255) || cfg->workspace_bytes < lay.total)
    return fail(nullptr, AREAL_E_NOMEM, "workspace missing, misaligned or smaller than areal_workspace_bytes");
  const uint64_t blk = areal_kv_block_bytes(cfg);
  if (!cfg->kv_arena || ((uintptr_t)cfg->kv_arena & 255) || cfg->kv_arena_bytes < blk)
    return fail(nullptr, AREAL_E_NOMEM, "kv_arena missing, misaligned or smaller than one block");
  areal_ctx* c = new areal_ctx();
  c->cfg = *cfg;
  if (const char* e = getenv("AREAL_DECODE_SPLIT_TARGET")) {   // tuning knob for sweeps
    const int v = atoi(e);
    if (v >= 64 && v <= 65536) c->split_target = v;
  }
  if (const char* e = getenv("AREAL_DECODE_GROUPS")) c->group_decode = atoi(e) > 0 ? 1 : (atoi(e) == 0 ? 0 : -1);
  if (const char* e = getenv("AREAL_SCORE_FUSED")) c->fused_scoring = atoi(e) != 0;
  if (const char* e = getenv("AREAL_DECODE_MIN_CHUNK")) {
    const int v = atoi(e);
    if (v >= 128 && v <= 2048 && v % 128 == 0) c->min_chunk = v;
  }
  c->lay = lay;
  c->stream = reinterpret_cast<hipStream_t>(cfg->hip_stream);
  c->ws = reinterpret_cast<char*>(cfg->workspace);
  c->n_blocks = (int64_t)std::min<uint64_t>(cfg->kv_arena_bytes / blk, 0x7fffffff);
  c->geom.n_kv_heads = cfg->n_kv_heads;
  c->geom.head_dim = cfg->head_dim;
  c->geom.block_stride = cfg->n_kv_heads * 2 * AREAL_KV_BLOCK_TOKENS * cfg->head_dim;
  c->geom.layer_stride = c->n_blocks * (int64_t)c->geom.block_stride;
  c->alloc = new KvAllocator(c->n_blocks, cfg->max_seqs, lay.max_blocks, AREAL_KV_BLOCK_TOKENS);
  c->seqs.resize(cfg->max_seqs);
  c->prompt_of.resize(cfg->max_seqs);
  c->prompt_hash_of.assign(cfg->max_seqs, 0);
  c->seg_bytes = lay.ring_bytes / kRingSegs;
  for (int i = 0; i < kRingSegs; ++i) { c->seg_done[i] = nullptr; c->seg_recorded[i] = false; }
  auto die = [&](hipError_t e, const char* what) {
    std::string m = std::string(what) + ": " + hipGetErrorString(e);
    areal_destroy(c);
    return fail(nullptr, AREAL_E_HIP, m);
  };
  hipError_t e = hipHostMalloc((void**)&c->ring_host, lay.ring_bytes, hipHostMallocMapped);
  if (e != hipSuccess) { c->ring_host = nullptr; return die(e, "hipHostMalloc(ring)"); }
  e = hipHostGetDevicePointer((void**)&c->ring_host_dev, c->ring_host, 0);
  if (e != hipSuccess) return die(e, "hipHostGetDevicePointer(ring)");
  for (int i = 0; i < kRingSegs; ++i) {
    e = hipEventCreateWithFlags(&c->seg_done[i], hipEventDisableTiming);
    if (e != hipSuccess) { c->seg_done[i] = nullptr; return die(e, "hipEventCreate"); }
  }
  // Masked positions of a partly filled block still pass through the value product
  // with weight 0: the pool must never hold NaN or Inf bit patterns.
  e = hipMemsetAsync(cfg->kv_arena, 0, (size_t)c->n_blocks * blk, c->stream);
  if (e != hipSuccess) return die(e, "hipMemsetAsync(kv_arena)");
  // rotary tables: angle = pos * theta^(-2j/d), evaluated in double
  {
    const int half = cfg->head_dim / 2;
    std::vector<float> ct((size_t)cfg->max_seq_len * half), sn(ct.size());
    std::vector<double> freq(half);
    for (int j = 0; j < half; ++j) freq[j] = pow((double)cfg->rope_theta, -2.0 * j / cfg->head_dim);
    for (int p = 0; p < cfg->max_seq_len; ++p)
      for (int j = 0; j < half; ++j) {
        const double a = (double)p * freq[j];
        ct[(size_t)p * half + j] = (float)cos(a);
        sn[(size_t)p * half + j] = (float)sin(a);
      }
    e = hipMemcpyAsync(c->ws + lay.cos_t, ct.data(), ct.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(c->ws + lay.sin_t, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return die(e, "rotary table upload");
  }
  *out = c;
  return AREAL_OK;
}

int areal_destroy(areal_ctx* c) {
  if (!c) return AREAL_E_INVAL;
  (void)hipStreamSynchronize(c->stream);
  for (int i = 0; i < kRingSegs; ++i)
    if (c->seg_done[i]) (void)hipEventDestroy(c->seg_done[i]);
  if (c->ring_host) (void)hipHostFree(c->ring_host);
  for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
  delete c->alloc;
  delete c;
  return AREAL_OK;
}

int areal_load_weights(areal_ctx* c, const areal_weights* w, uint64_t version) {
  if (!c) return AREAL_E_INVAL;
  int rc = check_weights_arg(c, w);
  if (rc) return rc;
  for (auto& s : c->seqs)
    if (s.live) return fail(c, AREAL_E_STATE, "sequences are live: use areal_update_weights_interrupt");
  if (version > (uint64_t)INT64_MAX) return fail(c, AREAL_E_INVAL, "version too large");
  rc = install_weights(c, w);
  if (rc) return rc;
  c->version = (int64_t)version;
  return AREAL_OK;
}

int areal_prefill(areal_ctx* c, int32_t n, const int32_t* seq_ids, const int32_t* tokens,
                  const int32_t* cu, float* logits_out) {
  if (!c) return AREAL_E_INVAL;
  if (!c->have_weights) return fail(c, AREAL_E_STATE, "no weights loaded");
  if (n == 0) return AREAL_OK;                       // nothing to admit
  if (n < 0 || !seq_ids || !tokens || !cu || !logits_out) return fail(c, AREAL_E_INVAL, "NULL argument or negative count");
  const areal_model_cfg& g = c->cfg;
  if (n > g.max_seqs) return fail(c, AREAL_E_INVAL, "more sequences than max_seqs");
  if (cu[0] != 0) return fail(c, AREAL_E_INVAL, "cu_seqlens[0] must be 0");
  std::vector<char> seen(g.max_seqs, 0);
  // Prompt-prefix sharing (16 answers are sampled per prompt): a sequence whose prompt equals
  // that of an earlier sequence of this call, or of a sequence still live from an earlier call
  // (the streaming regime admits the samples of a prompt one by one), holds that sequence's full
  // prompt blocks too and computes only what follows them.  One block fewer is shared when
  // the prompt ends on a block boundary, so that every sequence has a last row of its own to
  // produce logits from.  Every live sequence's K/V was computed under the current parameters
  // (a weight update recomputes all of them), so any live holder of the prompt will do.
  std::vector<int> leader(n, -1), live_leader(n, -1), n_sh(n, 0);
  std::vector<uint64_t> hashes(n, 0);
  {
    std::unordered_map<uint64_t, std::vector<int>> by_hash;
    for (int i = 0; i < n; ++i) {
      const int64_t len = (int64_t)cu[i + 1] - cu[i];
      if (len < 1) continue;                       // reported below
      uint64_t h = 1469598103934665603ull ^ (uint64_t)len;
      for (int64_t t = cu[i]; t < cu[i + 1]; ++t) h = (h ^ (uint32_t)tokens[t]) * 1099511628211ull;
      hashes[i] = h;
      auto& bucket = by_hash[h];
      for (int j : bucket)
        if (cu[j + 1] - cu[j] == len && !memcmp(tokens + cu[j], tokens + cu[i], (size_t)len * 4)) {
          leader[i] = j;
          break;
        }
      if (leader[i] < 0) {
        bucket.push_back(i);
        auto it = c->prompt_index.find(h);
        if (it != c->prompt_index.end())
          for (int32_t id : it->second) {
            const auto& p = c->prompt_of[id];
            if ((int64_t)p.size() == len && !memcmp(p.data(), tokens + cu[i], (size_t)len * 4)) {
              live_leader[i] = id;
              break;
            }
          }
      }
      if (leader[i] >= 0 || live_leader[i] >= 0) n_sh[i] = (int)((len - 1) / AREAL_KV_BLOCK_TOKENS);
    }
  }
  int64_t need_blocks = 0;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i];
    if (id < 0 || id >= g.max_seqs || seen[id]) return fail(c, AREAL_E_INVAL, "sequence id out of range or repeated");
    if (c->seqs[id].live) return fail(c, AREAL_E_INVAL, "sequence id already live");
    seen[id] = 1;
    const int64_t len = (int64_t)cu[i + 1] - cu[i];
    if (len < 1) return fail(c, AREAL_E_INVAL, "every prompt needs at least one token");
    if (len > g.max_seq_len) return fail(c, AREAL_E_NOMEM, "prompt longer than max_seq_len");
    need_blocks += c->alloc->blocks_for(len) - n_sh[i];
  }
  for (int64_t t = 0; t < cu[n]; ++t)
    if (tokens[t] < 0 || tokens[t] >= g.vocab) return fail(c, AREAL_E_INVAL, "token id outside the vocabulary");
  if (need_blocks > c->alloc->n_free()) return fail(c, AREAL_E_NOMEM, "KV arena exhausted");
  std::vector<Span> spans;
  std::vector<int64_t> tok_off;
  std::vector<int32_t> patches, hist_jobs;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i], len = cu[i + 1] - cu[i];
    const int shared_len = n_sh[i] * AREAL_KV_BLOCK_TOKENS;
    if (n_sh[i] > 0) {
      // the holder the blocks and the history are taken from: a sequence live before this call
      // where there is one (its history is already on the device; the first sample of this call
      // with the same prompt takes its own shared part from there in the same launches)
      const int lead_id = leader[i] < 0 ? live_leader[i]
                          : (live_leader[leader[i]] >= 0 ? live_leader[leader[i]] : seq_ids[leader[i]]);
      c->alloc->share_prefix(id, lead_id, n_sh[i]);
      c->seqs[lead_id].n_shared = std::max(c->seqs[lead_id].n_shared, n_sh[i]);
      const auto& lb = c->alloc->blocks(lead_id);
      for (int b = 0; b < n_sh[i]; ++b) { patches.push_back(id); patches.push_back(b); patches.push_back(lb[b]); }
      hist_jobs.push_back(id); hist_jobs.push_back(lead_id); hist_jobs.push_back(shared_len);
    }
    c->alloc->reserve(id, len);
    SeqInfo& s = c->seqs[id];
    s.live = true;
    s.len = len;
    s.kv_len = len;
    s.n_shared = std::max(s.n_shared, n_sh[i]);
    s.pending_version = c->version;
    s.versions.assign(len, -1);
    spans.push_back(Span{id, shared_len, len - shared_len, i});
    tok_off.push_back(cu[i] + shared_len);
    c->prompt_of[id].assign(tokens + cu[i], tokens + cu[i + 1]);
    c->prompt_hash_of[id] = hashes[i];
    c->prompt_index[hashes[i]].push_back(id);
  }
  SeqState st = c->seq_state();
  if (!patches.empty()) {
    int rc = stage_triples(c, patches, [&](const int32_t* d, int k) { return launch_table_patch(c->stream, d, k, st); });
    if (rc) return rc;
  }
  int rc = run_spans(c, spans, tokens, tok_off, true, logits_out);
  if (rc) return rc;
  if (!hist_jobs.empty())       // the shared part of the token history, once the leaders' rows have run
    rc = stage_triples(c, hist_jobs, [&](const int32_t* d, int k) { return launch_hist_copy(c->stream, d, k, st); });
  return rc;
}


int areal_decode_step(areal_ctx* c, int32_t n, const int32_t* seq_ids, const int32_t* tokens_in,
                      float* logits_out) {
  if (!c) return AREAL_E_INVAL;
  if (!c->have_weights) return fail(c, AREAL_E_STATE, "no weights loaded");
  if (n == 0) return AREAL_OK;                       // every sequence has finished
  if (n < 0 || !seq_ids || !tokens_in || !logits_out) return fail(c, AREAL_E_INVAL, "NULL argument or negative count");
  const areal_model_cfg& g = c->cfg;
  if (n > g.max_seqs) return fail(c, AREAL_E_INVAL, "more rows than max_seqs");
  std::vector<char> seen(g.max_seqs, 0);
  int64_t need_blocks = 0;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i];
    if (id < 0 || id >= g.max_seqs || seen[id]) return fail(c, AREAL_E_INVAL, "sequence id out of range or repeated");
    if (!c->seqs[id].live) return fail(c, AREAL_E_STATE, "decode on a sequence that was not prefilled");
    if (c->seqs[id].kv_len != c->seqs[id].len)
      return fail(c, AREAL_E_STATE, "sequence holds appended tokens without K/V: areal_update_weights_interrupt comes first");
    seen[id] = 1;
    if (c->seqs[id].len + 1 > g.max_seq_len) return fail(c, AREAL_E_NOMEM, "sequence would exceed max_seq_len");
    need_blocks += c->alloc->extra_needed(id, c->seqs[id].len + 1);
  }
  if (need_blocks > c->alloc->n_free()) return fail(c, AREAL_E_NOMEM, "KV arena exhausted");
  // Rows whose sequences hold the same leading blocks (the samples of a prompt): rows are
  // bucketed by their first block id, and the blocks all rows of a bucket have in common are
  // walked once per set of up to kGroupTiles * floor(16 / G) rows instead of once per row.
  const int P = 16 / (g.n_q_heads / g.n_kv_heads);
  std::vector<int> t_start(n, 0);
  struct RowSet { int start_blocks; std::vector<int> rows; };
  std::vector<RowSet> sets;
  int max_shared_blocks = 0;
  if (c->group_decode != 0 && n >= 2) {
    std::unordered_map<int32_t, std::vector<int>> by_first;
    std::vector<int32_t> order;
    for (int i = 0; i < n; ++i) {
      const auto& blocks = c->alloc->blocks(seq_ids[i]);
      if (blocks.empty()) continue;
      auto& v = by_first[blocks[0]];
      if (v.empty()) order.push_back(blocks[0]);
      v.push_back(i);
    }
    for (int32_t first : order) {
      const std::vector<int>& rows = by_first[first];
      if (rows.size() < 2) continue;
      const auto& lead = c->alloc->blocks(seq_ids[rows[0]]);
      // shared blocks are full and precede the position every row appends at
      int common = c->seqs[seq_ids[rows[0]]].len / AREAL_KV_BLOCK_TOKENS;
      for (size_t k = 1; k < rows.size() && common > 0; ++k) {
        const auto& b = c->alloc->blocks(seq_ids[rows[k]]);
        common = std::min(common, c->seqs[seq_ids[rows[k]]].len / AREAL_KV_BLOCK_TOKENS);
        int same = 0;
        while (same < common && b[same] == lead[same]) ++same;
        common = same;
      }
      if (common < 1) continue;
      for (size_t k = 0; k < rows.size(); k += (size_t)kGroupTiles * P) {
        RowSet rs{common, {}};
        for (size_t q = k; q < std::min(rows.size(), k + (size_t)kGroupTiles * P); ++q) rs.rows.push_back(rows[q]);
        sets.push_back(std::move(rs));
      }
      for (int r : rows) t_start[r] = common * AREAL_KV_BLOCK_TOKENS;
      max_shared_blocks = std::max(max_shared_blocks, common);
    }
  }
  // split the KV walk so that the grid holds a few work-groups per compute unit
  // (targets of 768 .. 6144 work-groups and minimum splits of 128 .. 512 tokens measured within
  // 5 % of each other on the rollout's context mixes; environment knobs AREAL_DECODE_SPLIT_TARGET
  // and AREAL_DECODE_MIN_CHUNK, read at areal_create, repeat that sweep)
  int64_t sum_ctx = 0;
  int max_ctx = 0, max_own = 0;
  for (int i = 0; i < n; ++i) {
    const int ctx = c->seqs[seq_ids[i]].len + 1;
    sum_ctx += ctx;
    max_ctx = std::max(max_ctx, ctx);
    max_own = std::max(max_own, ctx - t_start[i]);
  }
  if (c->group_decode < 0 && !sets.empty()) {
    int64_t shared_sum = 0;
    for (int i = 0; i < n; ++i) shared_sum += t_start[i];
    if (shared_sum * 10 < sum_ctx * 7) {
      sets.clear();
      std::fill(t_start.begin(), t_start.end(), 0);
      max_shared_blocks = 0;
      max_own = max_ctx;
    }
  }
  int64_t chunk = (sum_ctx * g.n_kv_heads / c->split_target + 127) / 128 * 128;
  chunk = std::min<int64_t>(std::max<int64_t>(chunk, c->min_chunk), 2048);   // a split spans at most 128 blocks
  int n_splits = (int)((max_own + chunk - 1) / chunk);
  // the shared part goes in short pieces (a work-group of a set has each wave walk all blocks of
  // its piece, so a piece is two block pairs where eight partial slots suffice, longer for longer
  // prompts)
  const int max_shared = max_shared_blocks * AREAL_KV_BLOCK_TOKENS;
  int sh_chunk = std::max(64, (max_shared + 8 * 64 - 1) / (8 * 64) * 64);
  int n_shared = max_shared ? (max_shared + sh_chunk - 1) / sh_chunk : 0;
  if (sh_chunk > 2048 || n_splits + n_shared > kMaxSplits) {   // very deep contexts: every row walks all its blocks itself
    sets.clear();
    std::fill(t_start.begin(), t_start.end(), 0);
    max_shared_blocks = 0;
    n_shared = 0;
    n_splits = (int)((max_ctx + chunk - 1) / chunk);
    if (n_splits > kMaxSplits) {
      chunk = ((max_ctx + kMaxSplits - 1) / kMaxSplits + 127) / 128 * 128;
      n_splits = (int)((max_ctx + chunk - 1) / chunk);
    }
  }
  // per-step block table: row i lists the blocks of seq_ids[i] from block t_start[i] / 16 on (the
  // attention kernel then finds its block ids from the launch row alone, without going through
  // the sequence's slot); row n + k lists the leading blocks of set k
  const int n_sets = (int)sets.size();
  int longest_blocks = max_shared_blocks;
  for (int i = 0; i < n; ++i)
    longest_blocks = std::max(longest_blocks, c->alloc->blocks_for(c->seqs[seq_ids[i]].len + 1) -
                                                  t_start[i] / AREAL_KV_BLOCK_TOKENS);
  const int tab_stride = (longest_blocks + 3) / 4 * 4;
  const uint64_t set_rows_bytes = (uint64_t)n_sets * kGroupTiles * 16 * 4;
  int rc = ring_begin(c, align_up((uint64_t)n * 4, 64) * 4 + align_up((uint64_t)(n + n_sets) * tab_stride * 4, 64) +
                             align_up(set_rows_bytes, 64) + align_up((uint64_t)n_sets * 4, 64));
  if (rc) return rc;
  const uint64_t start = c->seg_used;
  Staged s_slot = ring_take(c, (uint64_t)n * 4), s_pos = ring_take(c, (uint64_t)n * 4),
         s_nb = ring_take(c, (uint64_t)n * 4), s_ts = ring_take(c, (uint64_t)n * 4),
         s_tab = ring_take(c, (uint64_t)(n + n_sets) * tab_stride * 4);
  Staged s_rows{nullptr, nullptr}, s_start{nullptr, nullptr};
  if (n_sets) {
    s_rows = ring_take(c, set_rows_bytes);
    s_start = ring_take(c, (uint64_t)n_sets * 4);
  }
  int32_t *hslot = (int32_t*)s_slot.host, *hpos = (int32_t*)s_pos.host, *hnb = (int32_t*)s_nb.host,
          *hts = (int32_t*)s_ts.host, *htab = (int32_t*)s_tab.host;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i];
    SeqInfo& s = c->seqs[id];
    const int pos = s.len;
    const size_t had = c->alloc->blocks(id).size();
    c->alloc->reserve(id, pos + 1);
    const auto& blocks = c->alloc->blocks(id);
    const int skip = t_start[i] / AREAL_KV_BLOCK_TOKENS;
    hslot[i] = id;
    hpos[i] = pos;
    hts[i] = t_start[i];
    hnb[i] = blocks.size() > had ? blocks.back() : -1;
    int32_t* trow = htab + (size_t)i * tab_stride;
    memcpy(trow, blocks.data() + skip, (blocks.size() - skip) * 4);
    for (int b = (int)blocks.size() - skip; b < tab_stride; ++b) trow[b] = 0;
    s.versions.push_back(s.pending_version);
    s.len = pos + 1;
    s.kv_len = pos + 1;
    s.pending_version = c->version;
  }
  for (int k = 0; k < n_sets; ++k) {
    const RowSet& rs = sets[k];
    int32_t* trow = htab + (size_t)(n + k) * tab_stride;
    const auto& lead = c->alloc->blocks(seq_ids[rs.rows[0]]);
    memcpy(trow, lead.data(), (size_t)rs.start_blocks * 4);
    for (int b = rs.start_blocks; b < tab_stride; ++b) trow[b] = 0;
    int32_t* hrows = (int32_t*)s_rows.host + (size_t)k * kGroupTiles * 16;
    for (int q = 0; q < kGroupTiles * 16; ++q) hrows[q] = -1;
    for (size_t q = 0; q < rs.rows.size(); ++q) hrows[(q / P) * 16 + q % P] = rs.rows[q];
    ((int32_t*)s_start.host)[k] = rs.start_blocks * AREAL_KV_BLOCK_TOKENS;
  }
  rc = ring_flush(c, start);
  if (rc) return rc;
  PassArgs a{};
  a.M = n;
  a.rm = RowMeta{(const int32_t*)s_slot.dev, (const int32_t*)s_pos.dev};
  a.tokens_in = tokens_in;
  a.new_block = (const int32_t*)s_nb.dev;
  a.decode = true;
  a.chunk = (int)chunk;
  a.n_splits = n_splits;
  a.last_rows = nullptr;
  a.n_out = n;
  a.logits = logits_out;
  a.attn_units = (double)sum_ctx;
  a.step_table = (const int32_t*)s_tab.dev;
  a.step_stride = tab_stride;
  for (const RowSet& rs : sets) {
    c->set_rows_sum += (int64_t)rs.rows.size();
    c->set_row_tokens_sum += (int64_t)rs.rows.size() * rs.start_blocks * AREAL_KV_BLOCK_TOKENS;
    c->set_tokens_sum += (int64_t)rs.start_blocks * AREAL_KV_BLOCK_TOKENS;
  }
  if (n_sets) {
    a.groups.t_start = (const int32_t*)s_ts.dev;
    a.groups.set_rows = (const int32_t*)s_rows.dev;
    a.groups.set_start = (const int32_t*)s_start.dev;
    a.groups.n_sets = n_sets;
    a.groups.sh_chunk = sh_chunk;
    a.groups.n_shared = n_shared;
  }
  return run_pass(c, a);
}

int areal_append_tokens(areal_ctx* c, int32_t n, const int32_t* seq_ids, const int32_t* tokens_in) {
  if (!c) return AREAL_E_INVAL;
  if (n == 0) return AREAL_OK;
  if (n < 0 || !seq_ids || !tokens_in) return fail(c, AREAL_E_INVAL, "NULL argument or negative count");
  const areal_model_cfg& g = c->cfg;
  if (n > g.max_seqs) return fail(c, AREAL_E_INVAL, "more rows than max_seqs");
  std::vector<char> seen(g.max_seqs, 0);
  int64_t need_blocks = 0;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i];
    if (id < 0 || id >= g.max_seqs || seen[id]) return fail(c, AREAL_E_INVAL, "sequence id out of range or repeated");
    if (!c->seqs[id].live) return fail(c, AREAL_E_STATE, "append to a sequence that was not prefilled");
    seen[id] = 1;
    if (c->seqs[id].len + 1 > g.max_seq_len) return fail(c, AREAL_E_NOMEM, "sequence would exceed max_seq_len");
    need_blocks += c->alloc->extra_needed(id, c->seqs[id].len + 1);
  }
  if (need_blocks > c->alloc->n_free()) return fail(c, AREAL_E_NOMEM, "KV arena exhausted");
  int rc = ring_begin(c, align_up((uint64_t)n * 4, 64) * 3);
  if (rc) return rc;
  const uint64_t start = c->seg_used;
  Staged s_slot = ring_take(c, (uint64_t)n * 4), s_pos = ring_take(c, (uint64_t)n * 4),
         s_nb = ring_take(c, (uint64_t)n * 4);
  int32_t *hslot = (int32_t*)s_slot.host, *hpos = (int32_t*)s_pos.host, *hnb = (int32_t*)s_nb.host;
  for (int i = 0; i < n; ++i) {
    const int id = seq_ids[i];
    SeqInfo& s = c->seqs[id];
    const int pos = s.len;
    const size_t had = c->alloc->blocks(id).size();
    c->alloc->reserve(id, pos + 1);
    hslot[i] = id;
    hpos[i] = pos;
    hnb[i] = c->alloc->blocks(id).size() > had ? c->alloc->blocks(id).back() : -1;
    s.versions.push_back(s.pending_version);      // the version whose logits the token was drawn from
    s.len = pos + 1;                              // kv_len stays: no K/V for this position yet
  }
  rc = ring_flush(c, start);
  if (rc) return rc;
  HIP_TRY(c, launch_append(c->stream, n, g.vocab, RowMeta{(const int32_t*)s_slot.dev, (const int32_t*)s_pos.dev},
                           tokens_in, (const int32_t*)s_nb.dev, c->seq_state()));
  return AREAL_OK;
}

int areal_sample_logprob(areal_ctx* c, int32_t n, const float* logits, const int32_t* seq_ids,
                         const int32_t* positions, float temperature, float top_p, uint64_t seed,
                         const int32_t* forced, int32_t* tokens_out, float* logp_behav, float* logp_full) {
  if (!c) return AREAL_E_INVAL;
  if (n == 0) return AREAL_OK;
  if (n < 0 || !logits || !tokens_out || !logp_behav) return fail(c, AREAL_E_INVAL, "NULL argument or negative count");
  if (!(temperature > 0.f) || !(top_p > 0.f)) return fail(c, AREAL_E_INVAL, "temperature and top_p must be > 0");
  if (!forced && (!seq_ids || !positions)) return fail(c, AREAL_E_INVAL, "seq_ids and positions are required to draw");
  const int32_t *d_ids = nullptr, *d_pos = nullptr;
  if (!forced) {
    int rc = ring_begin(c, align_up((uint64_t)n * 4, 64) * 2);
    if (rc) return rc;
    const uint64_t start = c->seg_used;
    Staged a = ring_take(c, (uint64_t)n * 4), b = ring_take(c, (uint64_t)n * 4);
    memcpy(a.host, seq_ids, (size_t)n * 4);
    memcpy(b.host, positions, (size_t)n * 4);
    rc = ring_flush(c, start);
    if (rc) return rc;
    d_ids = (const int32_t*)a.dev;
    d_pos = (const int32_t*)b.dev;
  }
  const float inv_t = 1.0f / temperature;
  const bool sampled = c->prof_class == AREAL_K_SAMPLER && (c->prof_pass++ % c->prof_every) == 0;
  ProfScope ps(c, AREAL_K_SAMPLER, -1, sampled, (double)n);
  HIP_TRY(c, launch_sampler(c->stream, n, c->cfg.vocab, logits, d_ids, d_pos, inv_t, top_p, seed, forced,
                            tokens_out, logp_behav, logp_full, c->ws + c->lay.samp));
  return AREAL_OK;
}

int areal_update_weights_interrupt(areal_ctx* c, const areal_weights* new_w, uint64_t new_version,
                                   int32_t* n_live_out, int32_t* live_ids_out, float* logits_out,
                                   int64_t* retok_out) {
  if (!c) return AREAL_E_INVAL;
  if (!c->have_weights) return fail(c, AREAL_E_STATE, "no weights loaded");
  int rc = check_weights_arg(c, new_w);
  if (rc) return rc;
  if (!n_live_out || !live_ids_out) return fail(c, AREAL_E_INVAL, "NULL output argument");
  if (new_version > (uint64_t)INT64_MAX || (int64_t)new_version <= c->version)
    return fail(c, AREAL_E_STATE, "new_version must be greater than the current version");
  std::vector<Span> spans;
  int64_t total = 0;
  int nl = 0;
  // a shared prompt prefix is recomputed once, by the first live sequence that holds it
  std::unordered_set<int32_t> claimed;
  for (int id = 0; id < c->cfg.max_seqs; ++id)
    if (c->seqs[id].live) {
      const SeqInfo& q = c->seqs[id];
      int pos0 = 0;
      if (q.n_shared > 0 && !claimed.insert(c->alloc->blocks(id)[0]).second)
        pos0 = q.n_shared * AREAL_KV_BLOCK_TOKENS;
      spans.push_back(Span{id, pos0, q.len - pos0, nl});
      total += q.len - pos0;
      ++nl;
    }
  if (nl > 0 && !logits_out) return fail(c, AREAL_E_INVAL, "logits_out is NULL with live sequences");
  rc = install_weights(c, new_w);       // stream-ordered after every earlier pass
  if (rc) return rc;
  c->version = (int64_t)new_version;
  *n_live_out = nl;
  for (int i = 0; i < nl; ++i) {
    live_ids_out[i] = spans[i].slot;
    c->seqs[spans[i].slot].pending_version = c->version;
    c->seqs[spans[i].slot].kv_len = c->seqs[spans[i].slot].len;
  }
  if (retok_out) *retok_out = total;
  if (nl == 0) return AREAL_OK;
  // old K/V is never read again: every position is rewritten under the new
  // weights, in position order, before any later position attends to it
  return run_spans(c, spans, nullptr, {}, false, logits_out);
}

int areal_recompute_logprob(areal_ctx* c, int32_t n, const int32_t* tokens, const int32_t* cu,
                            float temperature, float* scratch, int32_t scratch_rows, float* logp_out) {
  if (!c) return AREAL_E_INVAL;
  if (!c->have_weights) return fail(c, AREAL_E_STATE, "no weights loaded");
  if (n == 0) return AREAL_OK;
  if (n < 0 || !tokens || !cu || !scratch || !logp_out || scratch_rows < 1)
    return fail(c, AREAL_E_INVAL, "NULL argument, negative count or no scratch rows");
  if (!(temperature > 0.f)) return fail(c, AREAL_E_INVAL, "temperature must be > 0");
  const areal_model_cfg& g = c->cfg;
  if (cu[0] != 0) return fail(c, AREAL_E_INVAL, "cu_seqlens[0] must be 0");
  std::vector<int> free_slots;
  for (int id = 0; id < g.max_seqs; ++id)
    if (!c->seqs[id].live) free_slots.push_back(id);
  if (free_slots.empty()) return fail(c, AREAL_E_NOMEM, "no free sequence slot to score with");
  for (int i = 0; i < n; ++i) {
    const int64_t len = (int64_t)cu[i + 1] - cu[i];
    if (len < 1) return fail(c, AREAL_E_INVAL, "every sequence needs at least one token");
    if (len > g.max_seq_len) return fail(c, AREAL_E_NOMEM, "sequence longer than max_seq_len");
    if (c->alloc->blocks_for(len) > c->alloc->n_free()) return fail(c, AREAL_E_NOMEM, "KV arena too small to score this sequence");
  }
  for (int64_t t = 0; t < cu[n]; ++t)
    if (tokens[t] < 0 || tokens[t] >= g.vocab) return fail(c, AREAL_E_INVAL, "token id outside the vocabulary");
  ScoreArgs sa{1.0f / temperature, scratch, scratch_rows, logp_out};
  // groups of consecutive sequences that fit the free slots and blocks; their
  // K/V lives in borrowed blocks that go back to the pool once the passes are
  // queued (later passes that reuse them are ordered after on the stream)
  int i = 0;
  while (i < n) {
    std::vector<Span> spans;
    std::vector<int64_t> tok_off;
    int64_t blocks = 0;
    while (i < n && spans.size() < free_slots.size()) {
      const int len = cu[i + 1] - cu[i];
      const int64_t nb = c->alloc->blocks_for(len);
      if (blocks + nb > c->alloc->n_free()) break;
      blocks += nb;
      spans.push_back(Span{free_slots[spans.size()], 0, len, (int)spans.size()});
      tok_off.push_back(cu[i]);
      ++i;
    }
    for (auto& sp : spans) c->alloc->reserve(sp.slot, sp.len);
    const int rc = run_spans(c, spans, tokens, tok_off, true, nullptr, &sa);
    for (auto& sp : spans) c->alloc->release(sp.slot);
    if (rc) return rc;
  }
  return AREAL_OK;
}

int areal_ppo_objective(areal_ctx* c, int64_t n, const float* logp_theta, const float* logp_prox,
                        const float* logp_behav, const float* adv, const uint8_t* mask, float eps,
                        float* obj_out, double* sums_out) {
  if (!c) return AREAL_E_INVAL;
  if (n == 0) return AREAL_OK;
  if (n < 0 || n > INT32_MAX || !logp_theta || !logp_prox || !logp_behav || !adv || !sums_out ||
      !(eps >= 0.f))
    return fail(c, AREAL_E_INVAL, "NULL argument, bad count or negative clip range");
  HIP_TRY(c, launch_ppo_objective(c->stream, (int)n, logp_theta, logp_prox, logp_behav, adv, mask, eps, obj_out,
                                  sums_out));
  return AREAL_OK;
}

int areal_free_seq(areal_ctx* c, int32_t id) {
  if (!c) return AREAL_E_INVAL;
  if (id < 0 || id >= c->cfg.max_seqs || !c->seqs[id].live) return fail(c, AREAL_E_INVAL, "sequence not live");
  c->alloc->release(id);
  c->seqs[id] = SeqInfo();
  if (!c->prompt_of[id].empty()) {
    auto it = c->prompt_index.find(c->prompt_hash_of[id]);
    if (it != c->prompt_index.end()) {
      auto& v = it->second;
      v.erase(std::remove(v.begin(), v.end(), id), v.end());
      if (v.empty()) c->prompt_index.erase(it);
    }
    std::vector<int32_t>().swap(c->prompt_of[id]);
  }
  return AREAL_OK;
}

int areal_seq_len(areal_ctx* c, int32_t id, int32_t* len_out) {
  if (!c || !len_out) return AREAL_E_INVAL;
  if (id < 0 || id >= c->cfg.max_seqs) return fail(c, AREAL_E_INVAL, "sequence id out of range");
  *len_out = c->seqs[id].live ? c->seqs[id].len : -1;
  return AREAL_OK;
}

int areal_get_tokens(areal_ctx* c, int32_t id, int32_t* out) {
  if (!c || !out) return AREAL_E_INVAL;
  if (id < 0 || id >= c->cfg.max_seqs || !c->seqs[id].live) return fail(c, AREAL_E_INVAL, "sequence not live");
  HIP_TRY(c, hipMemcpyAsync(out, c->wsp<int32_t>(c->lay.hist) + (int64_t)id * c->cfg.max_seq_len,
                            (size_t)c->seqs[id].len * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return AREAL_OK;
}

int areal_get_versions(areal_ctx* c, int32_t id, int64_t* out) {
  if (!c || !out) return AREAL_E_INVAL;
  if (id < 0 || id >= c->cfg.max_seqs || !c->seqs[id].live) return fail(c, AREAL_E_INVAL, "sequence not live");
  memcpy(out, c->seqs[id].versions.data(), c->seqs[id].versions.size() * sizeof(int64_t));
  return AREAL_OK;
}

int areal_kv_blocks(areal_ctx* c, int64_t* total, int64_t* free_) {
  if (!c) return AREAL_E_INVAL;
  if (total) *total = c->alloc->n_blocks();
  if (free_) *free_ = c->alloc->n_free();
  return AREAL_OK;
}

int areal_decode_set_counters(areal_ctx* c, int64_t* rows, int64_t* row_tokens, int64_t* set_tokens) {
  if (!c) return AREAL_E_INVAL;
  if (rows) *rows = c->set_rows_sum;
  if (row_tokens) *row_tokens = c->set_row_tokens_sum;
  if (set_tokens) *set_tokens = c->set_tokens_sum;
  return AREAL_OK;
}

int areal_adopt_seq(areal_ctx* c, int32_t id, int32_t len, int32_t fill_token) {
  return areal_adopt_seq_shared(c, id, len, fill_token, -1, 0);
}

int areal_adopt_seq_shared(areal_ctx* c, int32_t id, int32_t len, int32_t fill_token, int32_t src_id,
                           int32_t n_shared_blocks) {
  if (!c) return AREAL_E_INVAL;
  const areal_model_cfg& g = c->cfg;
  if (id < 0 || id >= g.max_seqs || c->seqs[id].live) return fail(c, AREAL_E_INVAL, "sequence id out of range or live");
  if (len < 1 || len > g.max_seq_len) return fail(c, AREAL_E_INVAL, "bad length");
  if (fill_token < 0 || fill_token >= g.vocab) return fail(c, AREAL_E_INVAL, "token id outside the vocabulary");
  const uint64_t nb = c->alloc->blocks_for(len);
  if (n_shared_blocks > 0) {
    if (src_id < 0 || src_id >= g.max_seqs || src_id == id || !c->seqs[src_id].live ||
        (uint64_t)n_shared_blocks >= nb || (size_t)n_shared_blocks > c->alloc->blocks(src_id).size())
      return fail(c, AREAL_E_INVAL, "shared blocks: source not live, or more blocks than it holds or than fit below the last");
    if ((int64_t)nb - n_shared_blocks > c->alloc->n_free()) return fail(c, AREAL_E_NOMEM, "KV arena exhausted");
  } else if (c->alloc->extra_needed(id, len) > c->alloc->n_free()) {
    return fail(c, AREAL_E_NOMEM, "KV arena exhausted");
  }
  int rc = ring_begin(c, align_up(nb * 4, 64));
  if (rc) return rc;
  if (n_shared_blocks > 0) {
    c->alloc->share_prefix(id, src_id, n_shared_blocks);
    c->seqs[src_id].n_shared = std::max(c->seqs[src_id].n_shared, n_shared_blocks);
  }
  c->alloc->reserve(id, len);
  Staged t = ring_take(c, nb * 4);
  memcpy(t.host, c->alloc->blocks(id).data(), nb * 4);
  // table rows start on 16-byte boundaries only if max_blocks % 4 == 0: go through the device ring
  HIP_TRY(c, launch_stage_copy(c->stream, c->ring_host_dev + (t.host - c->ring_host), t.dev, align_up(nb * 4, 16)));
  HIP_TRY(c, hipMemcpyAsync(c->wsp<int32_t>(c->lay.table) + (int64_t)id * c->lay.max_blocks, t.dev, nb * 4,
                            hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipMemsetD32Async((hipDeviceptr_t)(c->wsp<int32_t>(c->lay.hist) + (int64_t)id * g.max_seq_len),
                               fill_token, (size_t)len, c->stream));
  SeqInfo& s = c->seqs[id];
  s.live = true;
  s.len = len;
  s.kv_len = len;
  s.n_shared = std::max(0, n_shared_blocks);
  s.pending_version = c->version;
  s.versions.assign(len, -1);
  return AREAL_OK;
}

int areal_profile_begin(areal_ctx* c, int32_t klass, int32_t layer, int32_t every) {
  if (!c) return AREAL_E_INVAL;
  if (klass < 0 || klass >= AREAL_K_COUNT || layer < 0 || layer >= c->cfg.n_layers || every < 1)
    return fail(c, AREAL_E_INVAL, "bad profile selection");
  c->prof_class = klass;
  c->prof_layer = layer;
  c->prof_every = every;
  c->prof_pass = 0;
  c->prof_units = 0.0;
  c->prof_used = 0;
  return AREAL_OK;
}

int areal_profile_end(areal_ctx* c, int64_t* n_out, double* ms_out, double* units_out) {
  if (!c) return AREAL_E_INVAL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  double ms = 0.0;
  for (size_t i = 0; i + 1 < c->prof_used; i += 2) {
    float t = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&t, c->prof_events[i], c->prof_events[i + 1]));
    ms += t;
  }
  if (n_out) *n_out = (int64_t)(c->prof_used / 2);
  if (ms_out) *ms_out = ms;
  if (units_out) *units_out = c->prof_units;
  c->prof_class = -1;
  c->prof_used = 0;
  return AREAL_OK;
}

// ---- single-kernel entry points (include/areal_ops.h) -------------------------
int areal_op_gemm(void* stream, const void* A, const void* W0, const void* W1, void* C, int32_t M,
                  int32_t N, int32_t K, int32_t mode, int32_t cfg, int32_t splits) {
  if (mode < 0 || mode > 2 || !A || !W0 || !C || (mode == 2 && !W1)) return AREAL_E_INVAL;
  GemmW w{{(const f16*)W0, mode == 2 ? (const f16*)W1 : nullptr, nullptr}, {N, 0, 0}};
  hipError_t e = launch_gemm_cfg((hipStream_t)stream, (const f16*)A, w, C, M, N, K, N, (GemmMode)mode, cfg, splits);
  if (e == hipErrorInvalidValue) return AREAL_E_INVAL;
  return e == hipSuccess ? AREAL_OK : AREAL_E_HIP;
}
int areal_op_gemm_num_configs(void) { return gemm_num_configs(); }
int areal_op_gemm_choose(int32_t M, int32_t N, int32_t K, int32_t mode, int32_t* cfg_out, int32_t* splits_out) {
  if (M <= 0 || N <= 0 || K <= 0 || mode < 0 || mode > 2 || !cfg_out || !splits_out) return AREAL_E_INVAL;
  int c, sp;
  gemm_choose(M, N, K, (GemmMode)mode, &c, &sp);
  *cfg_out = c;
  *splits_out = sp;
  return AREAL_OK;
}

int areal_op_stream_read(void* hip_stream, const void* src, uint64_t bytes, void* sink16) {
  if (!src || !sink16 || bytes == 0 || bytes % 16) {
    set_global_error("areal_op_stream_read: NULL pointer, or a size that is not a positive multiple of 16");
    return AREAL_E_INVAL;
  }
  const hipError_t e = launch_stream_read(reinterpret_cast<hipStream_t>(hip_stream), src, (size_t)bytes,
                                          0x5bd1e995u, sink16);
  if (e != hipSuccess) {
    set_global_error(std::string("areal_op_stream_read: ") + hipGetErrorString(e));
    return e == hipErrorInvalidValue ? AREAL_E_INVAL : AREAL_E_HIP;
  }
  return AREAL_OK;
}

}  // extern "C"
