/*
 * dk_engine.h - continuous-batching scheduler and block-granular prefix cache
 * on top of the decode-step library (decodekit.h).  Host-side C ABI: plain
 * pointers and sizes; the only device memory is a caller-owned arena.
 *
 * What it implements (the serving method of the paper, section "Text Model
 * Inference"):
 *   - Algorithm 1 (continuous batching scheduler): a waiting queue and a
 *     running batch of at most max_batch rows; a call to dk_engine_step first
 *     refills free rows from the queue, then runs one batched decode step
 *     that advances every running row by a token, then retires the rows that
 *     finished, so their places are free for the next call.
 *   - Algorithm 2 (text prefix cache lookup): a new prompt is matched against
 *     cached prompts, the KV state of the longest cached prefix is reused and
 *     the forward pass resumes at the returned start position.  Here the cache
 *     is block-granular: an entry is one full 16-token KV block, keyed by its
 *     tokens and by the entry of the block before it, so the chain of entries
 *     of a prompt names exactly its prefixes at block boundaries.  The lookup
 *     walks the chain forward instead of hashing every prefix from the longest
 *     down; both return the longest cached prefix (at block granularity).
 *     The reused blocks are shared through the block table (reference counts),
 *     not copied.
 *   - least-recently-used eviction bounds the cache (the paper's "Memory
 *     Management" paragraph): when the pool has no free block, the cached
 *     block that was used longest ago, is not the parent of another cached
 *     block and is not in use by a request is dropped.
 *
 * Readings where the paper is silent: a prompt that is cached completely still
 * has to produce its first token, so at most (|P|-1) / 16 blocks are reused and
 * at least the last prompt token is computed; blocks are cached when a prompt
 * has been prefilled (not when the request ends); only prompt blocks are cached.
 *
 * Threading: an engine and the objects it uses (model, pool) belong to one
 * thread at a time.  dk_engine_step synchronises the stream (it has to read the
 * new tokens to decide completion).
 */
#ifndef DK_ENGINE_H
#define DK_ENGINE_H

#include "decodekit.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- prefix index (host only; usable without the engine) ------------------- */

typedef struct dk_prefix_index dk_prefix_index;

/* An empty index for blocks of `block_size` tokens (16).  *out is owned by the
 * caller until dk_prefix_index_destroy, which also drops the index's references
 * on the blocks of `pool` it holds (pass the pool the blocks came from). */
dk_status dk_prefix_index_create(int32_t block_size, dk_prefix_index **out);
dk_status dk_prefix_index_destroy(dk_prefix_index *index, dk_kv_pool *pool);

/* Algorithm 2's lookup.  h_tokens[0..n_tokens) is a prompt; at most `max_blocks`
 * leading full blocks are looked up.  Writes the physical block ids of the
 * longest cached chain to h_out_blocks[0..*out_n) (not retained: the caller
 * retains what it uses) and marks those entries as just used.  The start
 * position of Algorithm 2 is *out_n * block_size. */
dk_status dk_prefix_index_match(dk_prefix_index *index, const int32_t *h_tokens, int32_t n_tokens,
                                int32_t max_blocks, int32_t *h_out_blocks, int32_t *out_n);

/* Algorithm 2's "store": registers the first n_blocks full blocks of a prompt,
 * whose KV lives in the physical blocks h_blocks[0..n_blocks) of `pool`.  A block
 * whose chain entry does not exist yet is adopted (the index takes one reference
 * on it with dk_kv_retain_block); where an entry exists already it is kept and
 * only marked as just used.  *out_adopted (may be NULL) = number adopted. */
dk_status dk_prefix_index_insert(dk_prefix_index *index, dk_kv_pool *pool, const int32_t *h_tokens,
                                 int32_t n_blocks, const int32_t *h_blocks, int32_t *out_adopted);

/* Drops the least recently used entry that has no cached successor and whose
 * block nobody but the index references, releasing the block to the pool.
 * DK_E_POOL_EXHAUSTED if no entry can be dropped.  *out_block (may be NULL) = the
 * block released. */
dk_status dk_prefix_index_evict_lru(dk_prefix_index *index, dk_kv_pool *pool, int32_t *out_block);

/* Number of cached blocks. */
dk_status dk_prefix_index_size(const dk_prefix_index *index, int32_t *out_entries);

/* ---- engine ---------------------------------------------------------------- */

typedef struct dk_engine dk_engine;

typedef struct dk_engine_config {
    int32_t max_batch;           /* M of Algorithm 1: 1..DK_MAX_BATCH                      */
    int32_t max_blocks_per_seq;  /* longest sequence (prompt + output) in 16-token blocks  */
    int32_t prefill_chunk;       /* prompt tokens per prefill call: 1..DK_MAX_BATCH        */
    int32_t prefix_cache;        /* 0: Algorithm 2 off (every prompt is computed in full)  */
} dk_engine_config;

typedef struct dk_engine_stats {
    int64_t iterations;          /* calls of dk_engine_step that did something             */
    int64_t decode_steps;        /* batched decode steps                                    */
    int64_t generated_tokens;    /* tokens appended to outputs                              */
    int64_t prefill_tokens;      /* prompt tokens computed                                  */
    int64_t reused_tokens;       /* prompt tokens taken from the prefix cache               */
    int64_t evictions;           /* cached blocks dropped                                   */
    int32_t cached_blocks;       /* blocks the prefix cache holds now                       */
    int32_t active, pending;     /* running rows and waiting requests now                   */
} dk_engine_stats;

/* Device bytes the engine needs in its arena (block tables, lengths, tokens and
 * the workspaces of dk_decode_step / dk_prefill_chunk, logits and sampler scratch). */
dk_status dk_engine_device_bytes(const dk_model *model, const dk_engine_config *cfg, size_t *out_bytes);

/* d_arena: caller-owned device memory of at least dk_engine_device_bytes, 256-byte
 * aligned, left to the engine until dk_engine_destroy.  model and pool stay owned
 * by the caller and must outlive the engine; the pool's blocks that are free at
 * this moment are the engine's to allocate. */
dk_status dk_engine_create(dk_model *model, dk_kv_pool *pool, const dk_engine_config *cfg, void *d_arena,
                           size_t arena_bytes, dk_engine **out);
/* Releases every block the engine holds (requests and cache). */
dk_status dk_engine_destroy(dk_engine *engine);

/* Queues a request (Q.push).  h_prompt[0..n_prompt): token ids, n_prompt >= 1;
 * generation stops after max_new_tokens >= 1 tokens or after the token eos_token
 * (-1: none) has been generated (it is part of the output).  The prompt plus the
 * output must fit max_blocks_per_seq blocks.  *out_id identifies the request. */
dk_status dk_engine_submit(dk_engine *engine, const int32_t *h_prompt, int32_t n_prompt,
                           int32_t max_new_tokens, int32_t eos_token, int64_t *out_id);

/* One iteration of Algorithm 1 on the given stream: admits pending requests while
 * there is room (prefix lookup, block allocation, chunked prefill of the part of
 * the prompt that is not cached, which also yields the request's first token),
 * one decode step for all active requests, removal of the completed ones.
 * A request for which no KV block can be found even after eviction ends with the
 * state DK_REQ_FAILED (only possible when the pool is too small for the batch).
 * *out_active (may be NULL) = running + waiting requests afterwards: 0 means nothing is left to do. */
dk_status dk_engine_step(dk_engine *engine, void *hip_stream, int32_t *out_active);

/* Sampling beyond greedy for every token generated from now on (dk_sampling and its exact
 * definition: decodekit.h, dk_sample_tokens).  params == NULL returns to greedy.  The random number of
 * a token is that of dk_sample_tokens with step = the number of sampler calls since this call (one per
 * admitted request for its first token, one per decode iteration) and row = the request's row in that
 * iteration: the same requests submitted in the same order give the same tokens. */
dk_status dk_engine_set_sampling(dk_engine *engine, const dk_sampling *params);

enum { DK_REQ_PENDING = 0, DK_REQ_ACTIVE = 1, DK_REQ_DONE = 2, DK_REQ_FAILED = 3 };

/* Copies the tokens generated so far (all of them, from the first) to
 * h_out_tokens[0..min(capacity, n)); *out_n = n, *out_state one of DK_REQ_*,
 * *out_reused (may be NULL) = prompt tokens the prefix cache supplied. */
dk_status dk_engine_poll(const dk_engine *engine, int64_t id, int32_t *h_out_tokens, int32_t capacity,
                         int32_t *out_n, int32_t *out_state, int32_t *out_reused);

/* Forgets a finished request (its output is no longer retrievable). */
dk_status dk_engine_forget(dk_engine *engine, int64_t id);

dk_status dk_engine_get_stats(const dk_engine *engine, dk_engine_stats *out);

#ifdef __cplusplus
}
#endif
#endif
