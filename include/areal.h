/*
 * areal.h -- C boundary of the MI355X rollout-generation library.
 *
 * The library implements the rollout worker of the AReaL paper (Section 4.1):
 * batched autoregressive generation of a decoder-only policy over many
 * variable-length sequences (`generate`), and the in-flight weight update
 * that interrupts it (`update_weights`).  Every sampled token comes with the
 * log-probability the sampling policy gave it, log pi_behav(a_t | s_t), which
 * the decoupled PPO objective (Section 5.2, Eq. 4-5) divides by, and with the
 * version of the policy that produced it (Proposition 1: the behaviour
 * policy of an interrupted trajectory is defined position by position).
 *
 *   generate        = areal_prefill, then repeat { areal_sample_logprob,
 *                     areal_decode_step } until the caller ends the sequence
 *                     with areal_free_seq
 *   update_weights  = areal_update_weights_interrupt
 *
 * Conventions
 *  - Plain C ABI, no exceptions, no abort.  Every call returns AREAL_OK (0)
 *    or a negative error code; areal_last_error() gives the text.  A call
 *    that fails leaves the context as it was before the call; the exception
 *    is AREAL_E_HIP (the runtime itself failed): the context is then only
 *    good for areal_destroy.
 *  - "device" pointers are HIP device memory owned by the caller (in the
 *    tests and benchmark: PyTorch allocations); "host" pointers are ordinary
 *    process memory, read or written before the call returns.
 *  - All device work is enqueued on the caller's stream (areal_model_cfg.
 *    hip_stream) in call order.  Calls return without waiting for the GPU;
 *    outputs in device memory are valid once the stream reaches that point.
 *  - One context serves one GPU and is not thread safe.
 *  - Launch-shape tuning knobs are read from the environment when a context
 *    is created (AREAL_DECODE_SPLIT_TARGET, AREAL_DECODE_MIN_CHUNK) or on
 *    first use (AREAL_GEMM_MAX_SPLITS, AREAL_PREFILL_TILE_ROWS); unset, the
 *    measured optima apply.  They change timings, never results beyond
 *    float32 summation order.
 *  - Matrices are row-major, out-features major: y = x W^T with W [out, in].
 *  - The model is the Qwen2 family: pre-norm blocks, RMSNorm, rotary position
 *    embedding in rotate-half pairing, grouped-query causal attention,
 *    SwiGLU feed-forward, untied (or aliased) output projection.
 */
#ifndef AREAL_H
#define AREAL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AREAL_OK        0
#define AREAL_E_INVAL  (-1)  /* bad argument: NULL, shape, unknown or duplicate sequence id      */
#define AREAL_E_NOMEM  (-2)  /* KV arena, workspace or a per-sequence limit exhausted            */
#define AREAL_E_STATE  (-3)  /* call out of order: no weights, decode before prefill, version
                                not increasing                                                   */
#define AREAL_E_HIP    (-4)  /* the HIP runtime reported an error                                */

#define AREAL_DTYPE_F32   0
#define AREAL_DTYPE_BF16  1
#define AREAL_DTYPE_F16   2

#define AREAL_KV_BLOCK_TOKENS 16

typedef struct areal_ctx areal_ctx;   /* opaque; owned by the library */

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float   rope_theta;          /* rotary base (1e6 for the Qwen2 shapes)                 */
  float   rms_eps;             /* added to the mean square inside the root (1e-6)         */
  int32_t max_seqs;            /* sequence ids are 0 .. max_seqs-1                        */
  int32_t max_seq_len;         /* prompt + generated tokens per sequence                  */
  int32_t max_batch_tokens;    /* rows of one forward pass; longer prefills are chunked   */
  int32_t convert_weights;     /* 1: parameter sets may be given as bf16 or float32; the
                                  library converts them to half precision (nearest even)
                                  into space reserved in the workspace.  0: only half-
                                  precision sets, read in place                           */
  void*    kv_arena;           /* device; paged K/V pool, any size >= one block; cleared
                                  by areal_create on hip_stream                           */
  uint64_t kv_arena_bytes;
  void*    workspace;          /* device; >= areal_workspace_bytes(cfg), 256-B aligned    */
  uint64_t workspace_bytes;
  void*    hip_stream;         /* hipStream_t owned by the caller; NULL = default stream  */
} areal_model_cfg;

/* One parameter set.  The matrix cores take half-precision (IEEE fp16)
 * operands with float32 accumulation: the paper's precision (Table 3:
 * parameters and KV cache fp16).  A set given as AREAL_DTYPE_F16 is read in
 * place: its device pointers must stay valid and unchanged until the next
 * areal_load_weights / areal_update_weights_interrupt has been called AND the
 * stream has passed it.  A set given as bf16 or float32 is converted during the
 * call that receives it (stream-ordered; bf16 values of magnitude >= 2^-14
 * convert exactly, smaller ones round to the nearest half subnormal, larger
 * than 65504 saturate) and is not read afterwards.
 * Per-layer arrays are host arrays of n_layers device pointers.
 * Range: the values that become matrix-core operands or K/V-cache entries
 * (normalised activations, q / k / v, attention output, SwiGLU output) are rounded
 * to half precision too; magnitudes above 65,504 saturate to +-65,504 (no infinities
 * are produced from finite values).  The residual stream, norm statistics,
 * accumulators, softmax statistics and logits are float32.
 * Reproducibility: projections whose K range is split over work-groups accumulate with
 * float32 atomic adds in no fixed order, so logits can differ from run to run in the last
 * bits (about 1e-7 relative); AREAL_GEMM_MAX_SPLITS=1 in the environment removes the splits,
 * and with them the run-to-run differences, at a cost in decode speed.  The sampler is a
 * pure function of the logits it is given. */
typedef struct {
  int32_t dtype;                                    /* AREAL_DTYPE_F16, _BF16 or _F32        */
  const void *embed;                                /* [vocab, hidden]                       */
  const void *lm_head;                              /* [vocab, hidden]; may equal embed      */
  const void *final_norm;                           /* [hidden]                              */
  const void *const *wq, *const *wk, *const *wv;    /* [nq*d, hidden], [nkv*d, hidden] x2    */
  const void *const *wo;                            /* [hidden, nq*d]                        */
  const void *const *wgate, *const *wup;            /* [ffn, hidden]                         */
  const void *const *wdown;                         /* [hidden, ffn]                         */
  const void *const *norm_attn, *const *norm_ffn;   /* [hidden]                              */
  const void *const *bq, *const *bk, *const *bv;    /* [nq*d], [nkv*d] x2; NULL = no bias    */
} areal_weights;

/* Bytes of workspace a context with this configuration needs (0 if the
 * configuration is invalid).  Bytes of one 16-token KV block over all layers. */
uint64_t areal_workspace_bytes(const areal_model_cfg* cfg);
uint64_t areal_kv_block_bytes(const areal_model_cfg* cfg);

int areal_create(const areal_model_cfg* cfg, areal_ctx** out);
int areal_destroy(areal_ctx* ctx);          /* waits for the stream, frees host state only */
const char* areal_last_error(const areal_ctx* ctx);   /* ctx may be NULL: last create error */

/* Section 4.1 "loads parameters of new versions": register the parameter set
 * every later forward pass uses.  Allowed only while no sequence is live (with
 * live sequences use areal_update_weights_interrupt).  `version` tags the
 * tokens sampled from logits computed under this set. */
int areal_load_weights(areal_ctx* ctx, const areal_weights* w, uint64_t version);

/* Section 4.1 `generate`, first half; Section 3.1 state s_1 = q.  Starts n_seqs
 * new sequences: reserves KV blocks, runs the decoder over the packed prompt
 * tokens with causal attention (in chunks of max_batch_tokens rows), stores K
 * and V in the paged cache, and writes the logits for each sequence's first
 * generated token.
 *   seq_ids    host [n_seqs]   unused ids in 0 .. max_seqs-1, all distinct
 *   tokens     host [cu_seqlens[n_seqs]]  packed prompts, each length >= 1
 *   cu_seqlens host [n_seqs+1] prefix sums of the prompt lengths, [0] = 0
 *   logits_out device float32 [n_seqs, vocab]
 * Sequences whose prompts are identical (the paper samples 16 answers per
 * prompt, Table 3) share the KV blocks of the prompt, whether they arrive in
 * one call or one by one while an earlier one is still live (the streaming
 * regime of Section 4.1): the first of them computes the prompt, each of the
 * others holds the same full blocks (all but the block with the prompt's last
 * token) and computes only the positions after them.  Nothing else changes for the caller: every sequence has its own
 * id, logits row, history and later blocks, and a shared block returns to the
 * pool when its last holder terminates.  areal_update_weights_interrupt
 * recomputes a shared part once.
 * n_seqs == 0 is a no-op (AREAL_OK, no pointer is read).  On any error no
 * sequence is admitted and no block is reserved. */
int areal_prefill(areal_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids,
                  const int32_t* tokens, const int32_t* cu_seqlens, float* logits_out);

/* Section 3.1 transition s_{t+1} = concat(s_t, a_t); Section 4.1 `generate`,
 * the decoding loop.  Appends tokens_in[i] to sequence seq_ids[i] and runs one
 * forward pass at one row per sequence against each sequence's own cached K/V.
 *   seq_ids   host [n_seqs]    live, distinct
 *   tokens_in device int32 [n_seqs]  (typically tokens_out of the sampler)
 *   logits_out device float32 [n_seqs, vocab]  logits for the NEXT token
 * The appended token is tagged with the version whose logits it was sampled
 * from (the version loaded when those logits were computed).
 * n_seqs == 0 is a no-op.  AREAL_E_NOMEM (KV pool exhausted, or a sequence at
 * max_seq_len) leaves every sequence as it was: free some and call again. */
int areal_decode_step(areal_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids,
                      const int32_t* tokens_in, float* logits_out);

/* Section 5.2: pi_behav is the policy used for sampling; Table 3 defaults
 * temperature 1, top-p 1, top-k off.  For each row of float32 logits:
 *   z = logits * (1/T); fixed-point masses c_i = floor(sexp(z_i - max z) * 2^32);
 *   nucleus = shortest prefix, ranked by (c desc, id asc), whose mass reaches
 *   ceil(top_p * sum c); r = floor(R * S_nuc / 2^64) with R the first two words
 *   of Philox4x32-10(counter=(position, seq_id, 0, 0), key=seed); the token is
 *   the first kept id, ascending, whose running mass exceeds r.
 *   logp_behav = log(c_tok / S_nuc); logp_full = log_softmax(z)[tok].
 * The token id is a pure function of (logits row, T, top_p, seed, seq_id,
 * position).  Logits must be finite.
 *   logits    device float32 [n, vocab]
 *   seq_ids, positions  host [n]  (position = index the sampled token will have)
 *   forced_tokens  device int32 [n] or NULL.  Given: no draw; tokens_out =
 *                  forced_tokens and the log-probs are those of the forced
 *                  tokens (-inf behaviour log-prob outside the nucleus).
 *   tokens_out device int32 [n]; logp_behav_out device float32 [n];
 *   logp_full_out device float32 [n] or NULL.
 * T <= 0, top_p <= 0 or NaN -> AREAL_E_INVAL; n == 0 is a no-op. */
int areal_sample_logprob(areal_ctx* ctx, int32_t n, const float* logits,
                         const int32_t* seq_ids, const int32_t* positions,
                         float temperature, float top_p, uint64_t philox_seed,
                         const int32_t* forced_tokens,
                         int32_t* tokens_out, float* logp_behav_out, float* logp_full_out);

/* areal_sample_logprob for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  No context: the scratch buffer that lets a row be spread over several
 * work-groups is a static device array inside the library (about 1 MiB per GPU, held until
 * the process ends).  The call allocates nothing and takes DEVICE arrays throughout:
 *   hip_stream  hipStream_t (NULL = default stream) on the current device
 *   logits      device float32 [n, vocab]
 *   seq_ids, positions  device int32 [n] (unused, may be NULL, with forced_tokens)
 *   forced_tokens, tokens_out, logp_behav_out, logp_full_out  as areal_sample_logprob
 * Same results as areal_sample_logprob (token ids bit for bit).  At most
 * AREAL_SAMPLE_STATIC_MAX_ROWS rows of at most AREAL_SAMPLE_STATIC_MAX_VOCAB logits per
 * call; more returns AREAL_E_NOMEM and does nothing (split the batch).  Every call on a
 * GPU uses that GPU's one array: calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream are ordered.  Errors: text via areal_last_error(NULL). */
#define AREAL_SAMPLE_STATIC_MAX_ROWS  128
#define AREAL_SAMPLE_STATIC_MAX_VOCAB 262144
int areal_sample_logprob_static(void* hip_stream, int32_t n, int32_t vocab, const float* logits,
                                const int32_t* seq_ids, const int32_t* positions,
                                float temperature, float top_p, uint64_t philox_seed,
                                const int32_t* forced_tokens, int32_t* tokens_out,
                                float* logp_behav_out, float* logp_full_out);

/* Section 4.1 `update_weights`: interrupt all generations in flight, switch to
 * the new parameters, discard the K/V computed with the old ones and recompute
 * them: every live sequence's whole prefix (prompt + tokens generated so far)
 * is prefilled again under new_w.  Tokens already emitted, and their version
 * tags, are untouched (Proposition 1).  new_version > the current version.
 *   n_live_out        host int32          number of live sequences
 *   live_seq_ids_out  host int32 [max_seqs]  their ids, ascending
 *   logits_out        device float32 [n_live, vocab] in that order; may be
 *                     NULL only if no sequence is live
 *   reprefilled_tokens_out  host int64 or NULL: positions recomputed (shared
 *                     prompt blocks count once) */
int areal_update_weights_interrupt(areal_ctx* ctx, const areal_weights* new_w,
                                   uint64_t new_version, int32_t* n_live_out,
                                   int32_t* live_seq_ids_out, float* logits_out,
                                   int64_t* reprefilled_tokens_out);

/* Proposition 1 (the behaviour policy of an interrupted trajectory is defined
 * position by position): a weight update usually lands between
 * areal_sample_logprob and the areal_decode_step that would consume the sampled
 * tokens.  Those tokens were drawn from the old version's logits and must carry
 * the old version's tag.  areal_append_tokens appends tokens_in[i] to sequence
 * seq_ids[i] with that tag and NO forward pass (history and block table only);
 * the areal_update_weights_interrupt that follows recomputes every prefix, the
 * appended position included, under the new parameters and returns the logits
 * for the token after it.  Until that call the sequence has a position without
 * K/V: areal_decode_step on it fails with AREAL_E_STATE.  (Without this call
 * the order sample -> update -> decode would tag the token with the new
 * version: append, or decode, before updating.)
 *   seq_ids host [n] live, distinct; tokens_in device int32 [n].
 * Errors as areal_decode_step; n == 0 is a no-op. */
int areal_append_tokens(areal_ctx* ctx, int32_t n_seqs, const int32_t* seq_ids,
                        const int32_t* tokens_in);

/* Section 5.2, Eq. 5 (decoupled PPO objective): the proximal policy's token
 * log-probabilities are recomputed over complete trajectories, with whatever
 * parameters are loaded now, when a training batch has arrived.  For each
 * packed sequence x_0 .. x_{L-1}:
 *   logp_out[cu[i] + t] = log softmax(logits(x_0..x_{t-1}) / T)[x_t],  t >= 1,
 *   logp_out[cu[i]]     = 0.
 * One causal forward over all tokens (the prefill kernels, chunks of
 * max_batch_tokens rows).  No logits are stored: the output projection leaves a
 * (max, sum of exponentials) pair per row and column tile in the scratch and a
 * second kernel folds them (when the hidden size is not a multiple of 64 the
 * logits of scratch_rows rows at a time are written there and reduced instead).
 * Live sequences are untouched: the pass borrows unused sequence slots and free
 * KV blocks and returns them before it returns (AREAL_E_NOMEM, nothing
 * queued, if there is no free slot or one sequence alone does not fit the free
 * blocks).
 *   tokens      host [cu_seqlens[n_seqs]]   packed sequences, each length >= 1
 *   cu_seqlens  host [n_seqs+1]
 *   logits_scratch  device float32 [scratch_rows, vocab], scratch_rows >= 1
 *   logp_out    device float32 [cu_seqlens[n_seqs]] */
int areal_recompute_logprob(areal_ctx* ctx, int32_t n_seqs, const int32_t* tokens,
                            const int32_t* cu_seqlens, float temperature,
                            float* logits_scratch, int32_t scratch_rows, float* logp_out);

/* Section 5.2, Eq. 5 (decoupled PPO objective), forward value over n tokens:
 *   u_t = exp(logp_theta - logp_prox),  w_t = exp(logp_prox - logp_behav),
 *   obj_t = w_t * min(u_t A_t, clip(u_t, 1 - eps, 1 + eps) A_t)      (0 where mask is 0)
 * logp_behav is what areal_sample_logprob emitted, logp_prox what
 * areal_recompute_logprob returns for the proximal parameters, logp_theta the
 * same for the current ones.  All arrays device, float32 [n]; mask device
 * uint8 [n] or NULL; obj_out device float32 [n] or NULL.
 *   sums_out  device float64 [3], ACCUMULATED into (the caller clears it):
 *             sum of obj_t, tokens whose clipped term is the smaller one,
 *             tokens counted. */
int areal_ppo_objective(areal_ctx* ctx, int64_t n, const float* logp_theta, const float* logp_prox,
                        const float* logp_behav, const float* adv, const uint8_t* mask, float eps,
                        float* obj_out, double* sums_out);

/* Termination (Section 4.1 "until the next interruption or termination"): the
 * caller decides when a sequence ends; its KV blocks return to the pool. */
int areal_free_seq(areal_ctx* ctx, int32_t seq_id);

/* Host-side state queries.  areal_get_tokens waits for the stream. */
int areal_seq_len(areal_ctx* ctx, int32_t seq_id, int32_t* len_out);   /* -1 if not live */
int areal_get_tokens(areal_ctx* ctx, int32_t seq_id, int32_t* tokens_out /* host [len] */);
/* Policy version per position: -1 for prompt tokens, else the version that
 * produced the token (Proposition 1). */
int areal_get_versions(areal_ctx* ctx, int32_t seq_id, int64_t* versions_out /* host [len] */);
int areal_kv_blocks(areal_ctx* ctx, int64_t* total_out, int64_t* free_out);
/* Decode attention can walk KV blocks that several rows of a step hold together (the samples
 * of one prompt, Table 3: 16 answers per prompt) once per set of rows and not once per row.
 * It does so in the steps where at least 70 % of the context tokens read are shared in this
 * way; AREAL_DECODE_GROUPS=1 / 0 in the environment at areal_create makes it always / never.
 * The result is the same up to float32 summation order.
 * Sums over the decode steps since areal_create (any pointer may be NULL):
 *   rows_out        rows that were part of a set,
 *   row_tokens_out  context tokens of those rows that their set walked for them,
 *   set_tokens_out  context tokens the sets walked (each set once). */
int areal_decode_set_counters(areal_ctx* ctx, int64_t* rows_out, int64_t* row_tokens_out,
                              int64_t* set_tokens_out);

/* Benchmark helper: make `seq_id` a live sequence of `len` tokens whose K/V are
 * taken to be whatever the arena blocks assigned to it already hold and whose
 * token history is `fill_token`.  No forward pass runs.  Lets a decode step be
 * timed at a chosen context depth without generating up to it. */
int areal_adopt_seq(areal_ctx* ctx, int32_t seq_id, int32_t len, int32_t fill_token);
/* The same with the first n_shared_blocks KV blocks held together with the live sequence
 * src_id (as the samples of one prompt share the prompt's blocks after areal_prefill):
 * n_shared_blocks must be below the block count of `len` and at most what src_id holds. */
int areal_adopt_seq_shared(areal_ctx* ctx, int32_t seq_id, int32_t len, int32_t fill_token,
                           int32_t src_id, int32_t n_shared_blocks);

/* Measurement hook (Section 3.2 motivates the roofline: decoding is memory-IO
 * bound).  Between areal_profile_begin and areal_profile_end the library
 * brackets one kernel launch of class `kernel_class` (layer `layer` of every
 * `every`-th forward pass; the sampler and the output projection have no
 * layer) with HIP events on the stream.  areal_profile_end waits for the
 * stream and reports how many launches were bracketed, their summed duration,
 * and their summed work units: context tokens read (attention decode),
 * query-key pairs (attention prefill), rows (everything else). */
#define AREAL_K_EMBED 0
#define AREAL_K_RMSNORM 1
#define AREAL_K_GEMM_QKV 2
#define AREAL_K_ROPE_KVWRITE 3
#define AREAL_K_ATTN_DECODE 4
#define AREAL_K_ATTN_PREFILL 5
#define AREAL_K_GEMM_O 6
#define AREAL_K_GEMM_GATEUP 7
#define AREAL_K_GEMM_DOWN 8
#define AREAL_K_GEMM_LMHEAD 9
#define AREAL_K_SAMPLER 10
#define AREAL_K_ATTN_MERGE 11
#define AREAL_K_COUNT 12
int areal_profile_begin(areal_ctx* ctx, int32_t kernel_class, int32_t layer, int32_t every);
int areal_profile_end(areal_ctx* ctx, int64_t* n_samples_out, double* total_ms_out,
                      double* total_units_out);

#ifdef __cplusplus
}
#endif
#endif /* AREAL_H */
