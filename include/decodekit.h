/*
 * decodekit - the continuous-batching decode step of a decoder-only
 * transformer on one MI355X (gfx950), behind a C ABI.
 *
 * One call of dk_decode_step is the body of the paper's continuous-batching
 * loop (Algorithm 1, "generate one token for all active requests"): every one
 * of the B active sequences advances by one token against its own KV cache.
 * The KV cache is a pool of fixed-size blocks addressed through per-sequence
 * block tables; sequences that resumed from the same cached prompt prefix (the
 * KV state and start position returned by the paper's text prefix cache
 * lookup, Algorithm 2) name the same physical blocks for that prefix.
 *
 * Conventions
 *   - Every function returns a dk_status (0 = DK_OK, negative = error).  After
 *     an error, dk_last_error() gives a text for the calling thread.  Nothing
 *     throws or aborts across this boundary.
 *   - "device pointer" = memory of the current HIP device, allocated and
 *     freed by the caller (e.g. a torch tensor).  The library never allocates
 *     or frees device memory; it keeps non-owning pointers.  Handles returned
 *     by dk_create_* are small host objects freed by dk_destroy_*.
 *   - Kernels are enqueued on the HIP stream passed as `hip_stream`
 *     (a hipStream_t cast to void*; NULL = the default stream).  No call
 *     synchronises the device; outputs are valid once the caller has
 *     synchronised that stream.
 *   - bf16 = upper 16 bits of an IEEE float32.  Matrices are row-major
 *     W[out][in] and act as y = W x.
 */
#ifndef DECODEKIT_H
#define DECODEKIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t dk_status;
enum {
    DK_OK = 0,
    DK_E_INVALID_ARG = -1,
    DK_E_POOL_EXHAUSTED = -2,
    DK_E_BAD_BLOCK = -3,
    DK_E_WORKSPACE_TOO_SMALL = -4,
    DK_E_UNSUPPORTED_SHAPE = -5,
    DK_E_HIP = -6
};

/* Limits of the library (dk_create_model / dk_decode_step reject beyond). */
#define DK_MAX_BATCH 64
#define DK_MAX_EXPERTS 256

/*
 * Shape of the decoder.  The paper delegates the model forward to its model
 * library; the shapes are those of the model families it benchmarks (Table 1).
 *   head_dim    64 or 128;  n_q_heads a multiple of n_kv_heads (group <= 8)
 *   hidden, ffn, expert_ffn, n_q_heads*head_dim: multiples of 8
 *   qk_norm     1: RMSNorm over head_dim of every q and k head before the
 *               rotary embedding (gains g_q, g_k shared by all heads)
 *   n_experts   0 = dense SwiGLU MLP of width ffn; >0 = mixture of n_experts
 *               SwiGLU experts of width expert_ffn, top_k chosen per token by
 *               a softmax router (ties to the lower index), the chosen
 *               probabilities renormalised to sum to one
 *   tie_lm_head informational (the caller passes the same pointer twice)
 */
typedef struct dk_model_config {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t qk_norm, n_experts, top_k, expert_ffn, tie_lm_head;
    double rms_eps, rope_theta;
} dk_model_config;

/* Device pointers to one layer's bf16 weights (caller-owned). */
typedef struct dk_layer_weights {
    const void *g_attn;   /* [hidden]            gain of the pre-attention norm */
    const void *w_qkv;    /* [(nq+2nkv)*d, hidden]  q rows, then k rows, then v */
    const void *g_q;      /* [head_dim] or NULL  (qk_norm)                      */
    const void *g_k;      /* [head_dim] or NULL                                 */
    const void *w_o;      /* [hidden, nq*d]                                     */
    const void *g_mlp;    /* [hidden]            gain of the pre-MLP norm       */
    const void *w_gate;   /* dense [ffn, hidden];  MoE [E, expert_ffn, hidden]  */
    const void *w_up;     /* same shape as w_gate                               */
    const void *w_down;   /* dense [hidden, ffn];  MoE [E, hidden, expert_ffn]  */
    const void *w_router; /* [E, hidden] or NULL                                */
} dk_layer_weights;

typedef struct dk_weight_ptrs {
    const void *embed;    /* device, bf16 [vocab, hidden]                       */
    const void *lm_head;  /* device, bf16 [vocab, hidden] (may equal embed)     */
    const void *g_final;  /* device, bf16 [hidden]                              */
    const dk_layer_weights *layers; /* HOST array of n_layers entries; copied   */
} dk_weight_ptrs;

typedef struct dk_kv_pool dk_kv_pool;
typedef struct dk_model dk_model;

/* Text of the last error on this thread; valid until the next call here. */
const char *dk_last_error(void);

/* Library version string and the GPU architecture its kernels were built for. */
const char *dk_version(void);

/* ---------------------------------------------------------------- KV pool --
 *
 * Layout (part of this ABI): a dense bf16 array
 *     pool[layer][block][kv][kv_head][slot][dim]      kv: 0 = K, 1 = V
 * i.e. element offset
 *     ((((layer*num_blocks + block)*2 + kv)*n_kv_heads + head)*block_size + slot)*head_dim + dim
 * so one (block, K|V, head) tile is a contiguous run of block_size*head_dim
 * elements.  Cached K is stored after q/k-norm and rotary embedding.  A
 * sequence's cache grows by one token per decode step (the paper's per-request
 * KV cache, background section on unified memory) and is never copied.
 */

/* Bytes of device memory a pool of num_blocks blocks needs.  Host only. */
dk_status dk_kv_pool_bytes(const dk_model_config *cfg, int32_t num_blocks, int32_t block_size,
                           size_t *out_bytes);

/* Wraps caller-owned device memory `dev_mem` (>= dk_kv_pool_bytes) as a pool.
 * All blocks start free.  block_size must be 16.  Host only (dev_mem is not
 * touched). */
dk_status dk_create_kv_pool(const dk_model_config *cfg, int32_t num_blocks, int32_t block_size,
                            void *dev_mem, size_t dev_bytes, dk_kv_pool **out);
dk_status dk_destroy_kv_pool(dk_kv_pool *pool);

/* Host-side block accounting.  alloc: takes a free block (lowest id first),
 * refcount 1, DK_E_POOL_EXHAUSTED if none.  alloc_id: takes that specific
 * block if free (lets a caller place blocks in its own order), DK_E_BAD_BLOCK
 * if out of range or in use.  retain: refcount+1 on a block in use - this is
 * how a second sequence shares a cached prefix block.  release: refcount-1,
 * the block returns to the free list at 0.  refcount: current count (0 =
 * free).  A block with refcount > 1 must not be an append target; the
 * caller gives each sequence a private block for its growing tail. */
dk_status dk_kv_alloc_block(dk_kv_pool *pool, int32_t *out_block_id);
dk_status dk_kv_alloc_block_id(dk_kv_pool *pool, int32_t block_id);
dk_status dk_kv_retain_block(dk_kv_pool *pool, int32_t block_id);
dk_status dk_kv_release_block(dk_kv_pool *pool, int32_t block_id);
dk_status dk_kv_refcount(const dk_kv_pool *pool, int32_t block_id, int32_t *out_refcount);
dk_status dk_kv_free_blocks(const dk_kv_pool *pool, int32_t *out_free);

/* Element offset of (layer, block, kv, head, slot, dim) in the pool.  Host only. */
dk_status dk_kv_offset(const dk_kv_pool *pool, int32_t layer, int32_t block, int32_t kv,
                       int32_t head, int32_t slot, int32_t dim, int64_t *out_offset);

/* Checks, on HOST copies of the tables, what a decode step over them needs:
 * every block id on positions 0..seq_lens[b] is in range and in use, and the
 * append target block of every sequence has refcount 1 and is not another
 * row's append target.  DK_E_BAD_BLOCK names the offender in dk_last_error. */
dk_status dk_kv_validate_tables(const dk_kv_pool *pool, const int32_t *h_block_tables,
                                int32_t max_blocks_per_seq, const int32_t *h_seq_lens, int32_t B);

/* Writes one token's K and V for every sequence into one layer of the pool,
 * at logical position seq_lens[b] through the block table (used to load
 * contexts and by tests; dk_decode_step appends by itself).
 *   d_block_tables  device int32 [B][max_blocks_per_seq]
 *   d_seq_lens      device int32 [B]
 *   d_k, d_v        device bf16 [B][n_kv_heads][head_dim], stored bit for bit */
dk_status dk_append_kv(dk_kv_pool *pool, int32_t layer, const int32_t *d_block_tables,
                       int32_t max_blocks_per_seq, const int32_t *d_seq_lens, int32_t B,
                       const void *d_k, const void *d_v, void *hip_stream);

/* ------------------------------------------------------------------ model -- */

/* Validates the shape and records the weight pointers (not dereferenced
 * here).  DK_E_UNSUPPORTED_SHAPE for shapes outside the limits above. */
dk_status dk_create_model(const dk_model_config *cfg, const dk_weight_ptrs *weights,
                          dk_model **out);

/*
 * The same model with 4-bit weights, the precision of the checkpoints the paper
 * benchmarks (evaluation setup: 4-bit quantised models): group-wise affine, a
 * group being 64 consecutive columns of a row with one bf16 scale and one bf16
 * bias, the weight being  scale * q + bias  for the code q in 0..15.
 * Dense and mixture-of-experts models (the expert stacks are 4-bit, the router
 * stays bf16); hidden, n_q_heads*head_dim and ffn (expert_ffn) multiples of 128,
 * and for expert layers hidden and expert_ffn of at least 512.
 *
 * Same structs as dk_create_model; g_* and embed stay bf16 as there, while
 * w_qkv, w_o, w_gate, w_up, w_down and lm_head each point to one packed matrix
 * [N rows][K columns] (caller-owned device memory, 16-byte aligned) of
 *     N*K/2 bytes of codes, then ceil(N/16) * K/128 * 128 bytes of scales and biases:
 *   codes   row after row; a row is K/128 steps of 16 little-endian 32-bit words
 *           indexed [lg 0..3][s 0..3]; word (lg, s) holds the 8 columns
 *           step*128 + s*32 + lg*8 + j, column j in bits 4j..4j+3 (j = 0..7);
 *   scales  per tile of 16 rows and per step 64 bf16 numbers indexed
 *   biases  [lg 0..3][h 0..1][i 0..3][scale, bias]: the scale and the bias of row
 *           16*tile + 4*lg + i for the columns step*128 + h*64 .. + 63 (rows past
 *           N: anything finite).
 * lm_head must not alias embed.  Steps of such a model run the single persistent
 * kernel where it applies (as for bf16 weights) and otherwise the matrix-core
 * kernels, at every batch size.
 */
dk_status dk_create_model_q4(const dk_model_config *cfg, const dk_weight_ptrs *weights,
                             dk_model **out);
dk_status dk_destroy_model(dk_model *model);

/* Bytes of device scratch a decode step needs for batches up to max_B whose
 * block tables are at most max_blocks_per_seq wide.  Host only. */
dk_status dk_workspace_bytes(const dk_model *model, int32_t max_B, int32_t max_blocks_per_seq,
                             size_t *out_bytes);

/* dk_decode_step flags */
#define DK_STEP_ADVANCE 1u /* after the step: d_tokens[b] = next token, d_seq_lens[b] += 1 */
#define DK_STEP_NO_FUSED 4u /* do not use the single persistent step kernel even where it
                               applies (batches of 1-2 rows of small dense models) */
/* HIP graphs: with DK_STEP_NO_FUSED a step enqueues kernels only and keeps no host state between
 * calls, so it may be captured into a graph and replayed (with DK_STEP_ADVANCE every replay moves
 * the sequences on); call it once eagerly on the device first.  The persistent kernel alternates
 * two buffer sets and counts steps on the host: it must not be captured. */
#define DK_STEP_PROFILE 2u /* time every kernel of the step with its own start/stop events;
                              the call then synchronises the stream before it returns and
                              adds the times to the totals dk_profile_read returns */

/* Kernel classes of a profiled step. */
enum {
    DK_K_EMBED = 0,      /* embedding rows, rotary angles                         */
    DK_K_GEMV,           /* weight-streaming GEMV (batches up to 4 rows)          */
    DK_K_GEMM,           /* weight-streaming skinny GEMM on the matrix cores      */
    DK_K_ATTENTION,      /* head norm + rotation + KV append + paged attention    */
    DK_K_MOE_ROUTER,
    DK_K_MOE_EXPERT,
    DK_K_MOE_COMBINE,
    DK_K_ARGMAX,
    DK_K_FUSED_STEP,     /* the whole step as one persistent kernel               */
    DK_K_COUNT
};

/*
 * One decode step for B sequences (Algorithm 1's per-iteration token
 * generation, batched; rows do not interact).
 *
 * For each row b, with T = d_seq_lens[b] tokens already cached: embeds
 * d_tokens[b]; per layer: RMSNorm, q/k/v projection, optional q/k head norm,
 * half-split rotary embedding at position T, stores k and v (rounded to bf16,
 * nearest even) at position T through the block table, grouped-query
 * attention over positions 0..T, output projection + residual, RMSNorm,
 * SwiGLU MLP or expert mixture + residual; final RMSNorm, lm_head, and the
 * greedy next token (lowest index among equal maxima).
 *
 *   d_block_tables  device int32 [B][max_blocks_per_seq]; entries up to index
 *                   T/block_size must be valid blocks of `pool`, the last of
 *                   them private to row b (see dk_kv_validate_tables)
 *   d_seq_lens      device int32 [B]; T < max_blocks_per_seq*block_size
 *   d_tokens        device int32 [B], each in [0, vocab)
 *   d_workspace     device scratch >= dk_workspace_bytes(model, B, max_blocks_per_seq),
 *                   256-byte aligned.  Between the steps of one model the caller
 *                   must leave it alone: the persistent step kernel (batches of
 *                   1-2 rows of small dense models) keeps hand-over buffers in it
 *                   that one step prepares for the next.  A workspace that was
 *                   overwritten, or is used with this model for the first time
 *                   after other use, must be announced with dk_workspace_reset.
 *   d_logits        device float32 [B][vocab], or NULL to skip storing logits
 *   d_next_tokens   device int32 [B]
 *   flags           0, DK_STEP_ADVANCE (then d_tokens / d_seq_lens are written;
 *                   otherwise the step leaves them untouched and the caller
 *                   advances them) and/or DK_STEP_PROFILE
 * The block tables are never modified.  Fast arithmetic: bf16 storage, float32
 * accumulation and float32 residual stream.
 */
dk_status dk_decode_step(dk_model *model, dk_kv_pool *pool, const int32_t *d_block_tables,
                         int32_t max_blocks_per_seq, int32_t *d_seq_lens, int32_t *d_tokens,
                         int32_t B, void *d_workspace, size_t workspace_bytes, float *d_logits,
                         int32_t *d_next_tokens, uint32_t flags, void *hip_stream);

/*
 * dk_decode_step for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * step with the workspace taken from a fixed device array inside the library
 * instead of a caller buffer.  The call allocates nothing, on the device or
 * through any allocating library routine.
 *
 * Same arguments, results and error behaviour as dk_decode_step without
 * d_workspace / workspace_bytes.  Limits and rules of its own:
 *   - the step's workspace must fit DK_STATIC_SCRATCH_BYTES.  Where only the
 *     persistent step kernel's hand-over buffers outgrow it (long tables of the
 *     3B- / 8B-class shapes at batch 1) the step runs one kernel per stage, as with
 *     DK_STEP_NO_FUSED; if that does not fit either, DK_E_WORKSPACE_TOO_SMALL and
 *     nothing is launched (every workload shape of this library at up to 64 rows fits);
 *   - DK_STEP_PROFILE is refused (it creates events): DK_E_INVALID_ARG;
 *   - every GPU the library runs on holds its own copy of the array until the
 *     process ends, and every call on a GPU uses that GPU's copy: calls that
 *     overlap on one GPU (two streams, two threads) race, so order them; a
 *     call keeps no results in the array beyond what the persistent step kernel
 *     prepares for the next step of the same model, and the library notices
 *     when another model used the array in between and starts over by itself.
 */
#define DK_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
dk_status dk_decode_step_static(dk_model *model, dk_kv_pool *pool, const int32_t *d_block_tables,
                                int32_t max_blocks_per_seq, int32_t *d_seq_lens, int32_t *d_tokens,
                                int32_t B, float *d_logits, int32_t *d_next_tokens, uint32_t flags,
                                void *hip_stream);

/*
 * Chunked prefill of one sequence: what n decode steps of that sequence fed
 * with the prompt tokens d_tokens[0..n) would do, in one pass.  This is the step
 * that turns the part of a prompt behind the cached prefix into KV state
 * (Algorithm 2 returns the cached KV state and the start position; Algorithm 1
 * then generates from the full state).
 *
 * With `start` tokens of the sequence already in the pool, row i of the chunk
 * is position start + i: its k and v are stored at that position (same
 * arithmetic and rounding as dk_decode_step), it attends to positions
 * 0..start+i, and d_next_tokens[i] / d_logits[i] are the greedy token / logits
 * after prompt token start + i (the last row's are the first generated token).
 *
 *   d_block_table   device int32 [max_blocks]: the sequence's table; entries up
 *                   to index (start+n-1)/block_size must be valid blocks, those
 *                   holding positions >= start private to the sequence
 *   start           >= 0; start + n <= max_blocks*block_size
 *   d_tokens        device int32 [n], 1 <= n <= DK_MAX_BATCH
 *   d_workspace     >= dk_workspace_bytes(model, n, max_blocks), 256-byte aligned;
 *                   may be the workspace of the decode steps (the next persistent
 *                   decode step re-initialises its part by itself)
 *   d_logits        device float32 [n][vocab] or NULL
 *   d_next_tokens   device int32 [n]; NULL together with d_logits skips the final
 *                   norm, lm_head and argmax (a chunk that is not the last of its prompt)
 * Longer prompts are fed chunk after chunk.  The weights are streamed once per
 * chunk, so the cost of a chunk is that of one decode step of n rows.
 */
dk_status dk_prefill_chunk(dk_model *model, dk_kv_pool *pool, const int32_t *d_block_table,
                           int32_t max_blocks, int32_t start, const int32_t *d_tokens, int32_t n,
                           void *d_workspace, size_t workspace_bytes, float *d_logits,
                           int32_t *d_next_tokens, void *hip_stream);

/*
 * Sampling beyond greedy (the paper does not describe its sampler; this is the
 * usual temperature / top-k / nucleus scheme, spelled out so that it can be
 * checked): for each row, with s_i = logit_i / temperature and
 * p_i = exp(s_i - max s):
 *   top_k  (0 < top_k < V): the candidates are all i with p_i >= the top_k-th
 *          largest p (equal values at the cut all stay); otherwise every i;
 *   top_p  (< 1): t* = the largest value such that the candidates with p_i >= t*
 *          hold at least top_p of the candidates' total; kept = those candidates;
 *   draw:  r = u * (total of the kept set); the result is the first kept index,
 *          in ascending order, whose running total exceeds r, where
 *          u = (x >> 8) / 2^24 and x is the first word of Philox4x32-10 with
 *          counter (step low, step high, row, 0) and key (seed low, seed high).
 * The same (seed, step, row, logits) always give the same token.
 *
 *   d_logits   device float32 [B][V] (e.g. the d_logits of dk_decode_step)
 *   d_scratch  device scratch of at least dk_sample_scratch_bytes(B, V), 256-byte aligned
 *   d_out      device int32 [B]
 * temperature > 0, top_k >= 0 (0: off), 0 < top_p <= 1 (1: off).
 */
typedef struct dk_sampling {
    float temperature;
    int32_t top_k;
    float top_p;
    uint64_t seed;
} dk_sampling;

dk_status dk_sample_scratch_bytes(int32_t B, int32_t V, size_t *out_bytes);
dk_status dk_sample_tokens(const float *d_logits, int32_t B, int32_t V, const dk_sampling *params,
                           uint64_t step, void *d_scratch, size_t scratch_bytes, int32_t *d_out,
                           void *hip_stream);

/* Totals of all profiled steps of `model` so far: out_ms[DK_K_COUNT] kernel
 * execution time in milliseconds per class, out_launches[DK_K_COUNT] launches
 * per class.  reset != 0 clears the totals.  Host only. */
dk_status dk_profile_read(dk_model *model, double *out_ms, int64_t *out_launches, int32_t reset);

/* Declares the workspace contents of `model` lost: the next decode step
 * re-initialises what it needs.  Host only. */
dk_status dk_workspace_reset(dk_model *model);

/* The persistent step kernel bounds every wait it does; if a wait ever ran out
 * (its blocks were not all resident, e.g. on a GPU shared with other work) the
 * step's results are invalid (every next token of that step is -1) and this
 * reports it: out[0] = serial number of the
 * last step that gave up (0 = none), out[1] = waits that ran out since the
 * workspace was first used.  Synchronises the stream.  DK_E_INVALID_ARG if the
 * workspace has not been used by a persistent step of `model`. */
dk_status dk_fused_status(const dk_model *model, const void *d_workspace, uint32_t *out,
                          void *hip_stream);

/* Test hook for that failure path: the number of polls after which a block of
 * the persistent kernel gives up a wait (0 restores the default, about 65 000,
 * i.e. tens of milliseconds).  With a limit of 1 practically every step gives
 * up at once; the kernel still runs to its end normally, writes the token -1
 * for every row (and does not advance tokens / lengths under DK_STEP_ADVANCE),
 * and dk_fused_status reports the step.  Host only. */
dk_status dk_debug_set_wait_limit(dk_model *model, int32_t polls);

/* Measurement aid for the persistent step kernel: from the next step on, every block records the device's
 * constant 100 MHz clock at the stage boundaries of layer `layer` into d_stamps[block][DK_STAGE_STAMPS]
 * (int64, device memory of at least blocks x DK_STAGE_STAMPS x 8 bytes with blocks = compute units of the
 * device; owned by the caller, must outlive the steps; entries a block does not reach keep their old value).
 * Boundaries: 0 layer begins, 1 q|k|v rows handed over, 2 q|k|v of the block's attention item arrived,
 * 3 chunk attention done, 4 merged attention output handed over (collecting blocks only), 5 attention output
 * arrived, 6 x_mid handed over, 7 x_mid arrived, 8 activations handed over, 9 activations arrived, 10 x_out
 * handed over, 11 next layer's input arrived; and of the step itself 12 kernel entry, 13 first layer begins,
 * 14 lm_head begins (last layer done), 15 the block's lm_head rows streamed.  Only the instance for batch 1 of the 0.6B-class shapes with
 * bf16 weights (head_dim 128, query groups of 2) has a stamping twin; other steps ignore the setting.
 * d_stamps NULL switches the stamps off (the default: the ordinary kernel, which has no trace of them).
 * Host only. */
#define DK_STAGE_STAMPS 16
dk_status dk_debug_set_stage_stamps(dk_model *model, int32_t layer, void *d_stamps, size_t stamps_bytes);

/* Experts chosen in the most recent decode step that used `d_workspace` with
 * the same B and max_blocks_per_seq (mixture-of-experts models only): copies
 * int32 [n_layers][B][top_k], each row in order of decreasing router
 * probability, to the HOST buffer h_out and synchronises the stream.  Used to
 * count the distinct experts a step streamed and to compare routing decisions. */
dk_status dk_step_routing(const dk_model *model, const void *d_workspace, int32_t B,
                          int32_t max_blocks_per_seq, int32_t *h_out, void *hip_stream);

/* Algorithmic HBM bytes of one decode step: every dense weight byte once,
 * every distinct live KV byte once (a shared block counts once), the B
 * embedding rows and the logits written.  Host only; takes HOST copies of the
 * tables.  `distinct_experts_per_layer` is a host array of n_layers counts for
 * MoE models (NULL for dense). */
dk_status dk_step_algorithmic_bytes(const dk_model *model, const dk_kv_pool *pool,
                                    const int32_t *h_block_tables, int32_t max_blocks_per_seq,
                                    const int32_t *h_seq_lens, int32_t B, int32_t with_logits,
                                    const int32_t *distinct_experts_per_layer,
                                    uint64_t *out_bytes);

/* Measurement aid: enqueues one kernel that reads `bytes` bytes (a multiple of 16) of device memory
 * once, 16 bytes per lane and eight loads in flight per lane, one block per compute unit, and does nothing
 * else (d_sink: device memory of at least 8 KB, practically never written).  Timed by the caller over a buffer larger than
 * the caches it gives the read-only bandwidth a streaming kernel can reach on this device, the practical
 * ceiling the decode kernels are compared with beside the published peak. */
dk_status dk_read_stream(const void *d_buf, size_t bytes, void *d_sink, void *hip_stream);

/* Introspection (host only, launches nothing): which kernel a batched weight-streaming GEMM of the decode
 * step takes for a matrix of N rows and K columns at B batch rows (5..64), on a device with
 * `compute_units` compute units (0: the current device's count, 256 if none answers).  The choice is the
 * candidate with the smallest estimated duration of a latency/occupancy model of the weight stream.
 * epilogue: 0 plain store (q | k | v, lm_head), 1 residual projection (attention output, down), 2 the
 * gate/up pair with SwiGLU (N = rows of each of the two matrices).  four_bit: 1 for 4-bit weights.
 * out_waves: 0 = the kernel whose waves split K (then out_slices = 1); otherwise the waves per block of
 * the kernel whose waves share the activation tile, with K cut into out_slices slices across blocks.
 * out_estimate_us: the model's estimate for the choice (0 where no estimate is made: 4-bit weights, K
 * not a multiple of 128).  DK_E_INVALID_ARG for NULL outputs, B outside 5..64 or non-positive sizes. */
dk_status dk_gemm_plan_query(int32_t epilogue, int32_t N, int32_t K, int32_t B, int32_t four_bit,
                             int32_t compute_units, int32_t *out_waves, int32_t *out_slices,
                             double *out_estimate_us);

#ifdef __cplusplus
}
#endif
#endif /* DECODEKIT_H */
