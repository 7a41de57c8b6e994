/*
 * areal_host.h -- host-only entry points of the library: the paged KV block
 * allocator, the pass planner and the staleness gate of the rollout
 * controller, exposed so that they can be exercised without a GPU.  They are the same objects the generation calls of areal.h
 * use internally (KV cache management is named by the paper, Section 2 "LLM
 * Training and Inference", as a requirement of generation; the token budget
 * per pass follows the padding-free packing of Section 6).
 * None of these functions touches the GPU.
 */
#ifndef AREAL_HOST_H
#define AREAL_HOST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct areal_kvalloc areal_kvalloc;

/* A pool of n_blocks blocks of 16 tokens for sequences 0 .. max_seqs-1.
 * Returns NULL on invalid arguments.  The caller destroys it. */
areal_kvalloc* areal_kvalloc_create(int64_t n_blocks, int32_t max_seqs, int32_t max_blocks_per_seq);
void areal_kvalloc_destroy(areal_kvalloc* a);
/* Grow sequence `seq` so that it can hold n_tokens.  0 on success; AREAL_E_NOMEM
 * (and no change) if the pool or the per-sequence limit is too small. */
int areal_kvalloc_reserve(areal_kvalloc* a, int32_t seq, int64_t n_tokens);
/* Drop `seq`'s hold on all its blocks; a block returns to the pool when its
 * last holder lets go. */
void areal_kvalloc_release(areal_kvalloc* a, int32_t seq);
/* Prompt-prefix sharing (the paper samples 16 answers per prompt, Table 3):
 * `dst`, which must hold no blocks, starts out holding the first n_blocks blocks
 * of `src` as well.  0 on success, AREAL_E_INVAL otherwise (no change). */
int areal_kvalloc_share(areal_kvalloc* a, int32_t dst, int32_t src, int32_t n_blocks);
int64_t areal_kvalloc_free_blocks(const areal_kvalloc* a);
/* Copy up to `cap` block ids of `seq` into out (host); returns the block count. */
int32_t areal_kvalloc_table(const areal_kvalloc* a, int32_t seq, int32_t* out, int32_t cap);
/* Deterministically permute the free list (block placement must not matter). */
void areal_kvalloc_shuffle(areal_kvalloc* a, uint64_t seed);

/* Cut n_spans sequences of the given lengths (each starting at position 0)
 * into forward passes of at most max_rows rows, in order.  Writes up to `cap`
 * records of 6 int32 {pass, span, pos0, len, row0, out_index} to out (host)
 * and returns the number of records; out_index is the span index on the piece
 * that ends a span, else -1. */
int32_t areal_plan_passes(int32_t n_spans, const int32_t* lens, int32_t max_rows, int32_t* out,
                          int32_t cap);

/* Section 5.1 (staleness-aware training): the rollout controller submits the
 * N-th generation request only if floor((N-1)/B) <= i + eta, with B the
 * training batch size, i the current policy version and eta the maximum
 * staleness of a training batch (eta = 0: synchronous).  The gate counts the
 * requests it has admitted (N_r) and holds the version it was last told.
 * create: NULL unless batch_size >= 1 and eta >= 0.  submit: tries n more
 * requests, returns how many it admitted (0 .. n).  set_version: versions only
 * grow; AREAL_E_STATE otherwise. */
typedef struct areal_gate areal_gate;
areal_gate* areal_gate_create(int64_t batch_size, int64_t eta);
void areal_gate_destroy(areal_gate* g);
int64_t areal_gate_submit(areal_gate* g, int64_t n);
int64_t areal_gate_budget(const areal_gate* g);      /* requests admissible right now */
int areal_gate_set_version(areal_gate* g, int64_t version);
int64_t areal_gate_submitted(const areal_gate* g);   /* N_r */

/* Appendix, Algorithm 1 (dynamic batching): partition n sequences of the given
 * lengths into micro-batches of total length <= capacity, at least k_min of
 * them, balanced in sequence count: longest first, a sequence opens a new
 * micro-batch while fewer than k_min exist or none has room, else joins the
 * micro-batch with room that holds the fewest sequences (earliest on a tie).
 * batch_of (host [n]) receives each sequence's micro-batch index; returns the
 * number of micro-batches, or AREAL_E_INVAL for n < 0, lengths < 1,
 * capacity < 1 or k_min < 1.  A sequence longer than capacity stands alone. */
int32_t areal_dynamic_batching(int32_t n, const int32_t* lens, int64_t capacity, int32_t k_min,
                               int32_t* batch_of);

#ifdef __cplusplus
}
#endif
#endif /* AREAL_HOST_H */
