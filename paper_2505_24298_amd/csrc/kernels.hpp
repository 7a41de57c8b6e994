// Host-callable launchers of the gfx950 kernels (internal C++ interface; the
// public boundary is include/areal.h).  Every launcher validates the shapes
// its kernel assumes and returns hipErrorInvalidValue instead of launching
// when they do not hold.
#pragma once
#include <string>

#include "common.hpp"

namespace areal {

// ---- elementwise.hip --------------------------------------------------------
struct RowMeta {               // device arrays, one entry per row of the pass
  const int32_t* slot;         // sequence slot of the row
  const int32_t* pos;          // absolute position of the row's token
};
struct SeqState {              // device-resident per-sequence state
  int32_t* hist;               // [max_seqs][max_seq_len] token history
  int32_t* table;              // [max_seqs][max_blocks] KV block ids
  int max_seq_len, max_blocks;
};

hipError_t launch_embed(hipStream_t s, const f16* embed, int hidden, int vocab, int M, RowMeta rm,
                        const int32_t* tokens_in, const int32_t* new_block, SeqState st, float* h);
// zero_out (optional): float32 [M, zero_cols] cleared row by row alongside (the
// buffer a following split-K product accumulates into).
hipError_t launch_rmsnorm(hipStream_t s, const float* x, const f16* gain, f16* y, int M, int hidden,
                          float eps, const int32_t* src_rows, float* zero_out = nullptr,
                          int zero_cols = 0);
hipError_t launch_rope_kvwrite(hipStream_t s, const float* qkv, int M, RowMeta rm, SeqState st,
                               const f16* bq, const f16* bk, const f16* bv, const float* cos_tab,
                               const float* sin_tab, f16* q_out, f16* arena_layer, KvGeom geom,
                               int n_q_heads);
// rows (rm.slot[r], rm.pos[r]): history[slot][pos] = tokens_in[r]; new_block[r] >= 0 is installed
// as block pos/16 of the slot
hipError_t launch_append(hipStream_t s, int n, int vocab, RowMeta rm, const int32_t* tokens_in,
                         const int32_t* new_block, SeqState st);
// {slot, block index, block id} triples -> block table; {dst slot, src slot, n tokens} -> history
hipError_t launch_table_patch(hipStream_t s, const int32_t* patch, int n, SeqState st);
hipError_t launch_hist_copy(hipStream_t s, const int32_t* jobs, int n, SeqState st);
hipError_t launch_stage_copy(hipStream_t s, const void* src_host_mapped, void* dst, size_t bytes);
// reads `bytes` (multiple of 16) and discards them; *sink16 (16 bytes) is written only if the xor of all
// words read equals `never` (pass any value: a write there is harmless)
hipError_t launch_stream_read(hipStream_t s, const void* src, size_t bytes, uint32_t never, void* sink16);
hipError_t launch_to_f16(hipStream_t s, const void* src, int src_is_bf16, f16* dst, int64_t n);

// ---- gemm.hip ---------------------------------------------------------------
// C[M,N] (+)= A[M,K] * W[N,K]^T, half-precision inputs, float32 accumulation on MFMA.
// W may be up to three row-segments (e.g. wq | wk | wv), each [rows, K].
struct GemmW {
  const f16* ptr[3];
  int end[3];                  // cumulative row counts; end[last used] == N
};
enum GemmMode {
  GEMM_STORE_F32 = 0,          // C float32 = acc
  GEMM_ADD_F32 = 1,            // C float32 += acc            (residual update)
  GEMM_SWIGLU_F16 = 2,        // two W of [N,K] (gate, up): C half = silu(A gate^T) * (A up^T)
};
// The output projection of a scoring pass without its [M, N] result: per row and column tile the
// pair (max, sum of exponentials relative to it) of z = (A W^T) * inv_t, and z at the row's target
// column.  part: float2 [n_tiles][ld_rows] (n_tiles = gemm_lse_tiles(M, N)); target: [M], -1 = none;
// target_z: [M], written for rows whose target is in [0, N).  Requires K % 64 == 0.
struct GemmLse {
  const int32_t* target;
  float* target_z;
  float inv_t;
};
int gemm_lse_tiles(int M, int N);
hipError_t launch_gemm_lse(hipStream_t s, const f16* A, GemmW W, int M, int N, int K, void* part, int ld_rows,
                           GemmLse lse);
hipError_t launch_gemm(hipStream_t s, const f16* A, GemmW W, void* C, int M, int N, int K, int ldc,
                       GemmMode mode);
// Same with an explicit tile configuration (0 .. gemm_num_configs()-1) and K
// split; -1 = take the tuned choice.  A split > 1 accumulates with float32
// atomics: for GEMM_STORE_F32 the caller must have zeroed C.
hipError_t launch_gemm_cfg(hipStream_t s, const f16* A, GemmW W, void* C, int M, int N, int K, int ldc,
                           GemmMode mode, int cfg, int splits);
void gemm_choose(int M, int N, int K, GemmMode mode, int* cfg, int* splits);
int gemm_num_configs();

// ---- attention.hip ----------------------------------------------------------
struct AttnWork {              // prefill work item: a tile of consecutive query rows of one sequence
  int32_t slot, row0, pos0, n_rows;   // n_rows <= attn_prefill_tile_rows()
};
int attn_prefill_tile_rows(int n_q_heads, int n_kv_heads);   // 16 or 32
// Rows of a decode launch whose sequences hold the same leading KV blocks (the samples of one
// prompt): those blocks are walked once per set of rows instead of once per row.  A set is up
// to kGroupTiles MFMA tiles of 16 rows = floor(16 / G) sequences x G query heads each; the
// work-groups of the sets are part of the same launch.  All arrays are device memory.
constexpr int kGroupTiles = 4;
struct DecodeGroups {
  const int32_t* t_start = nullptr;   // [M] leading tokens of row i that its set covers (multiple of 16; 0: none)
  const int32_t* set_rows = nullptr;  // [n_sets][kGroupTiles][16] launch rows of tile t (first floor(16/G) entries
                                      // used, -1 = empty; entry 0 of tile 0 is valid: its blocks are the ones walked)
  const int32_t* set_start = nullptr; // [n_sets] the t_start of the set's rows
  int n_sets = 0;                     // <= M
  int sh_chunk = 0;                   // tokens of the shared part per work-group (multiple of 32, at most 2048)
  int n_shared = 0;                   // partial slots per row for the shared part: ceil(max t_start / sh_chunk)
};
// decode: one query row per sequence (row i <-> rm.slot[i], rm.pos[i]), taken from the float32
// QKV rows [M, (nq + 2 nkv) d] of the pass: bias, RoPE and rounding of q and of the appended
// token's k happen inside, and the appended k, v are stored into the sequence's block
// (table entry pos/16 must be installed).  Context = positions 0 .. pos.  Row i's own
// work-groups cover positions t_start[i] .. pos in splits of `chunk` tokens (multiple of 128,
// at most 2048), n_splits >= ceil((pos + 1 - t_start[i]) / chunk) for every row; positions
// below t_start[i] are covered by the row's set.  With more than one partial slot per row
// (n_splits + grp.n_shared > 1, at most 32) the partials go to `part_o` / `part_ml` and
// launch_attn_merge (same chunk, n_splits, grp) combines them into `out`.  `step_table`
// (optional, device int32 [M, step_stride]): the block ids of row i's sequence, entries
// 0 .. pos/16 at least, laid out by launch row; replaces the lookup through st.table.
hipError_t launch_attn_decode(hipStream_t s, const float* qkv, int M, RowMeta rm, SeqState st,
                              const f16* bq, const f16* bk, const f16* bv, const float* cos_tab,
                              const float* sin_tab, f16* arena_layer, KvGeom geom, int n_q_heads,
                              int chunk, int n_splits, float* part_o, float* part_ml, f16* out,
                              const int32_t* step_table = nullptr, int step_stride = 0,
                              DecodeGroups grp = DecodeGroups{});
hipError_t launch_attn_merge(hipStream_t s, int M, RowMeta rm, int head_dim, int n_q_heads, int chunk,
                             int n_splits, const float* part_o, const float* part_ml, f16* out,
                             DecodeGroups grp = DecodeGroups{});
hipError_t launch_attn_prefill(hipStream_t s, const f16* q, const AttnWork* work, int n_work,
                               SeqState st, const f16* arena_layer, KvGeom geom, int n_q_heads,
                               f16* out);

// ---- sampler.hip ------------------------------------------------------------
// `scratch` (optional, device, 16-byte aligned, sampler_scratch_bytes()): lets the launch spread a
// row over several work-groups when few rows are sampled with top-p = 1; its contents are
// overwritten.  Without it every row is one work-group.
hipError_t launch_sampler(hipStream_t s, int n, int vocab, const float* logits, const int32_t* seq_ids,
                          const int32_t* positions, float inv_temperature, float top_p, uint64_t seed,
                          const int32_t* forced, int32_t* tokens_out, float* logp_behav, float* logp_full,
                          void* scratch = nullptr);
size_t sampler_scratch_bytes();
// text areal_last_error(NULL) returns (calls that have no context)
void set_global_error(const std::string& msg);

// ---- scoring.hip ------------------------------------------------------------
// Row r with target[r] >= 0: out[r + 1] = log softmax(logits[r] * inv_t)[target[r]];
// rows with pos[r] == 0 also set out[r] = 0.  (Rows are consecutive tokens of
// packed sequences: row r predicts the token stored at r + 1.)
// out[r + 1] = target_z[r] - log sum exp over the row, from the per-tile pairs of launch_gemm_lse
// (rows with target[r] < 0 are skipped; out[r] = 0 where pos[r] == 0)
hipError_t launch_lse_finish(hipStream_t s, const void* part, int ld_rows, int n_tiles, const float* target_z,
                             const int32_t* target, const int32_t* pos, int n, float* out);
hipError_t launch_token_logprob(hipStream_t s, const float* logits, int n, int vocab, float inv_t,
                                const int32_t* target, const int32_t* pos, float* out);

// Decoupled PPO objective (forward): sums[0..2] += {sum of per-token objective, tokens whose
// clipped term is active, tokens counted}; obj_out (optional) per token; mask (optional) bytes.
hipError_t launch_ppo_objective(hipStream_t s, int n, const float* logp_theta, const float* logp_prox,
                                const float* logp_behav, const float* adv, const uint8_t* mask, float eps,
                                float* obj_out, double* sums);

}  // namespace areal
