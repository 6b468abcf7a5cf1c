// Continuous-batching scheduler (the paper's Algorithm 1) and block-granular
// prefix cache (Algorithm 2 with least-recently-used eviction) - host code.
// It drives the device only through the public entry points of decodekit.h
// (dk_kv_* block accounting, dk_prefill_chunk, dk_decode_step) plus plain
// copies of block tables, lengths and tokens.
//
// Included at the end of decodekit.hip (shares its error reporting).
#pragma once
#include <array>
#include <deque>
#include <map>
#include <memory>

#include "../../include/dk_engine.h"

// ---------------------------------------------------------------------------
// Prefix index: one entry per cached full block.  An entry is identified by the
// entry of the block before it (-1 for the first block of a prompt) and by its
// own 16 tokens, so a chain of entries spells a prompt prefix exactly - no hash
// collisions to worry about, and "the longest cached prefix" is simply how far
// the chain can be walked.
// ---------------------------------------------------------------------------
struct dk_prefix_index {
    static constexpr int kBlock = 16;
    struct Entry {
        int parent = -1;
        int block = -1;
        int children = 0;
        uint64_t last_used = 0;
        std::array<int32_t, kBlock> toks{};
        bool live = false;
    };
    using Key = std::pair<int, std::array<int32_t, kBlock>>;
    std::vector<Entry> entries;
    std::vector<int> free_slots;
    std::map<Key, int> by_key;
    uint64_t tick = 0;

    static std::array<int32_t, kBlock> block_tokens(const int32_t *t)
    {
        std::array<int32_t, kBlock> a;
        std::copy(t, t + kBlock, a.begin());
        return a;
    }
    int find(int parent, const int32_t *t) const
    {
        auto it = by_key.find(Key(parent, block_tokens(t)));
        return it == by_key.end() ? -1 : it->second;
    }
    int add(int parent, const int32_t *t, int block)
    {
        int id;
        if (!free_slots.empty()) { id = free_slots.back(); free_slots.pop_back(); }
        else { id = (int)entries.size(); entries.emplace_back(); }
        Entry &e = entries[(size_t)id];
        e.parent = parent;
        e.block = block;
        e.children = 0;
        e.last_used = ++tick;
        e.toks = block_tokens(t);
        e.live = true;
        by_key[Key(parent, e.toks)] = id;
        if (parent >= 0) entries[(size_t)parent].children++;
        return id;
    }
    void remove(int id)
    {
        Entry &e = entries[(size_t)id];
        by_key.erase(Key(e.parent, e.toks));
        if (e.parent >= 0) entries[(size_t)e.parent].children--;
        e.live = false;
        free_slots.push_back(id);
    }
    int size() const { return (int)by_key.size(); }
};

dk_status dk_prefix_index_create(int32_t block_size, dk_prefix_index **out)
{
    if (!out) return fail(DK_E_INVALID_ARG, "NULL argument");
    if (block_size != dk_prefix_index::kBlock)
        return fail(DK_E_UNSUPPORTED_SHAPE, "block_size %d (16 supported)", block_size);
    *out = new dk_prefix_index();
    return DK_OK;
}

dk_status dk_prefix_index_destroy(dk_prefix_index *index, dk_kv_pool *pool)
{
    if (!index) return DK_OK;
    if (pool)
        for (const auto &e : index->entries)
            if (e.live) (void)dk_kv_release_block(pool, e.block);
    delete index;
    return DK_OK;
}

dk_status dk_prefix_index_match(dk_prefix_index *index, const int32_t *h_tokens, int32_t n_tokens,
                                int32_t max_blocks, int32_t *h_out_blocks, int32_t *out_n)
{
    if (!index || !h_tokens || !out_n || (max_blocks > 0 && !h_out_blocks))
        return fail(DK_E_INVALID_ARG, "NULL argument");
    if (n_tokens < 0) return fail(DK_E_INVALID_ARG, "n_tokens %d", n_tokens);
    const int limit = std::min(max_blocks, n_tokens / dk_prefix_index::kBlock);
    int parent = -1, n = 0;
    while (n < limit) {
        const int id = index->find(parent, h_tokens + (size_t)n * dk_prefix_index::kBlock);
        if (id < 0) break;
        index->entries[(size_t)id].last_used = ++index->tick;
        h_out_blocks[n++] = index->entries[(size_t)id].block;
        parent = id;
    }
    *out_n = n;
    return DK_OK;
}

dk_status dk_prefix_index_insert(dk_prefix_index *index, dk_kv_pool *pool, const int32_t *h_tokens,
                                 int32_t n_blocks, const int32_t *h_blocks, int32_t *out_adopted)
{
    if (!index || !pool || (n_blocks > 0 && (!h_tokens || !h_blocks)))
        return fail(DK_E_INVALID_ARG, "NULL argument");
    int parent = -1, adopted = 0;
    for (int i = 0; i < n_blocks; i++) {
        const int32_t *t = h_tokens + (size_t)i * dk_prefix_index::kBlock;
        int id = index->find(parent, t);
        if (id < 0) {
            const dk_status s = dk_kv_retain_block(pool, h_blocks[i]);   // the cache's own reference
            if (s != DK_OK) return s;
            id = index->add(parent, t, h_blocks[i]);
            adopted++;
        } else {
            index->entries[(size_t)id].last_used = ++index->tick;
        }
        parent = id;
    }
    if (out_adopted) *out_adopted = adopted;
    return DK_OK;
}

dk_status dk_prefix_index_evict_lru(dk_prefix_index *index, dk_kv_pool *pool, int32_t *out_block)
{
    if (!index || !pool) return fail(DK_E_INVALID_ARG, "NULL argument");
    int best = -1;
    for (int id = 0; id < (int)index->entries.size(); id++) {
        const auto &e = index->entries[(size_t)id];
        if (!e.live || e.children != 0) continue;
        int32_t rc = 0;
        if (dk_kv_refcount(pool, e.block, &rc) != DK_OK || rc != 1) continue;   // a request uses it
        if (best < 0 || e.last_used < index->entries[(size_t)best].last_used) best = id;
    }
    if (best < 0) return fail(DK_E_POOL_EXHAUSTED, "no cached block can be dropped");
    const int32_t block = index->entries[(size_t)best].block;
    index->remove(best);
    const dk_status s = dk_kv_release_block(pool, block);
    if (s != DK_OK) return s;
    if (out_block) *out_block = block;
    return DK_OK;
}

dk_status dk_prefix_index_size(const dk_prefix_index *index, int32_t *out_entries)
{
    if (!index || !out_entries) return fail(DK_E_INVALID_ARG, "NULL argument");
    *out_entries = index->size();
    return DK_OK;
}

// ---------------------------------------------------------------------------
// Engine
// ---------------------------------------------------------------------------
namespace {

struct EngineRequest {
    int64_t id = 0;
    std::vector<int32_t> prompt, out, blocks;
    int max_new = 0, eos = -1;
    int T = 0;            // tokens whose K/V are in the pool
    int last = 0;         // the token to feed next
    int reused = 0;       // prompt tokens supplied by the prefix cache
    int state = DK_REQ_PENDING;
};

}  // namespace

struct dk_engine {
    dk_model *model = nullptr;
    dk_kv_pool *pool = nullptr;
    dk_engine_config cfg{};
    dk_prefix_index *index = nullptr;
    std::map<int64_t, std::unique_ptr<EngineRequest>> all;
    std::deque<EngineRequest *> queue;        // Q
    std::vector<EngineRequest *> active;      // B, row i of the device tables is active[i]
    int64_t next_id = 1;
    dk_engine_stats stats{};
    // device arena
    int32_t *d_tables = nullptr, *d_seq = nullptr, *d_tok = nullptr, *d_next = nullptr, *d_chunk = nullptr;
    char *d_ws = nullptr;
    size_t ws_bytes = 0;
    bool no_fused = false;                    // the persistent step kernel gave up once: not used again
    // sampling beyond greedy (dk_engine_set_sampling): logits of a step, the sampler's scratch and output
    bool sampling = false;
    dk_sampling sampling_params{};
    uint64_t sample_step = 0;                 // counter of the sampler's random numbers: one per sampled batch
    float *d_logits = nullptr;
    char *d_sample_ws = nullptr;
    size_t sample_ws_bytes = 0;
    int32_t *d_sampled = nullptr;
    std::vector<int32_t> h_tables;            // host mirror [M][max_blocks]
    std::vector<char> row_dirty;
    // lengths and last tokens on the device are stale (the batch changed, or tokens were sampled on the side);
    // otherwise the decode step advances them itself and nothing is uploaded
    bool state_dirty = true;
};

namespace {

struct ArenaLayout { size_t tables, seq, tok, next, chunk, ws, ws_bytes, logits, sample_ws, sample_ws_bytes, sampled, total; };

dk_status engine_layout(const dk_model *model, const dk_engine_config *cfg, ArenaLayout *L)
{
    if (!model || !cfg) return fail(DK_E_INVALID_ARG, "NULL argument");
    if (cfg->max_batch < 1 || cfg->max_batch > DK_MAX_BATCH)
        return fail(DK_E_INVALID_ARG, "max_batch %d (1..%d)", cfg->max_batch, DK_MAX_BATCH);
    if (cfg->prefill_chunk < 1 || cfg->prefill_chunk > DK_MAX_BATCH)
        return fail(DK_E_INVALID_ARG, "prefill_chunk %d (1..%d)", cfg->prefill_chunk, DK_MAX_BATCH);
    if (cfg->max_blocks_per_seq < 1) return fail(DK_E_INVALID_ARG, "max_blocks_per_seq %d", cfg->max_blocks_per_seq);
    // a decode step may run with any batch 1..M and a prefill chunk with any size up to the configured one
    size_t ws = 0;
    {
        const dk_status s = dk_workspace_bytes(model, std::max(cfg->max_batch, cfg->prefill_chunk), cfg->max_blocks_per_seq, &ws);
        if (s != DK_OK) return s;
    }
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off = align_up(off + bytes, 256); return o; };
    L->tables = take((size_t)cfg->max_batch * cfg->max_blocks_per_seq * 4);
    L->seq = take((size_t)cfg->max_batch * 4);
    L->tok = take((size_t)cfg->max_batch * 4);
    L->next = take((size_t)DK_MAX_BATCH * 4);
    L->chunk = take((size_t)DK_MAX_BATCH * 4);
    L->ws = take(ws);
    L->ws_bytes = ws;
    // sampling: logits of every row of a step (or of a prefill chunk), scratch, tokens
    const int rows = std::max(cfg->max_batch, cfg->prefill_chunk);
    const dk_model_config &mc = model->cfg;
    size_t sws = 0;
    const dk_status ms = dk_sample_scratch_bytes(cfg->max_batch, mc.vocab, &sws);
    if (ms != DK_OK) return ms;
    L->logits = take((size_t)rows * mc.vocab * 4);
    L->sample_ws = take(sws);
    L->sample_ws_bytes = sws;
    L->sampled = take((size_t)DK_MAX_BATCH * 4);
    L->total = off;
    return DK_OK;
}

// a free block, dropping least recently used cached blocks while the pool is empty
dk_status engine_alloc_block(dk_engine *e, int32_t *out)
{
    for (;;) {
        int32_t nfree = 0;
        dk_status s = dk_kv_free_blocks(e->pool, &nfree);
        if (s != DK_OK) return s;
        if (nfree > 0) return dk_kv_alloc_block(e->pool, out);
        s = dk_prefix_index_evict_lru(e->index, e->pool, nullptr);
        if (s != DK_OK) return s;          // DK_E_POOL_EXHAUSTED: nothing left to drop
        e->stats.evictions++;
    }
}

void engine_release_blocks(dk_engine *e, EngineRequest *r)
{
    for (int32_t b : r->blocks) (void)dk_kv_release_block(e->pool, b);
    r->blocks.clear();
}

void engine_set_row(dk_engine *e, int row, const EngineRequest *r)
{
    int32_t *dst = e->h_tables.data() + (size_t)row * e->cfg.max_blocks_per_seq;
    std::fill(dst, dst + e->cfg.max_blocks_per_seq, -1);
    std::copy(r->blocks.begin(), r->blocks.end(), dst);
    e->row_dirty[(size_t)row] = 1;
    e->state_dirty = true;
}

dk_status engine_upload_rows(dk_engine *e, hipStream_t st)
{
    const size_t mb = (size_t)e->cfg.max_blocks_per_seq;
    for (size_t row = 0; row < e->row_dirty.size(); row++) {
        if (!e->row_dirty[row]) continue;
        DK_HIP(hipMemcpyAsync(e->d_tables + row * mb, e->h_tables.data() + row * mb, mb * 4,
                              hipMemcpyHostToDevice, st));
        e->row_dirty[row] = 0;
    }
    return DK_OK;
}

bool engine_finished(const EngineRequest *r)
{
    return (int)r->out.size() >= r->max_new || (r->eos >= 0 && !r->out.empty() && r->out.back() == r->eos);
}

// Moves one request from the waiting queue into the running batch: prefix lookup, blocks,
// prefill (Algorithm 1's admission, with Algorithm 2 inside).  DK_E_POOL_EXHAUSTED (with
// everything undone) means "not now".
dk_status engine_admit(dk_engine *e, EngineRequest *r, hipStream_t st)
{
    const int bs = dk_prefix_index::kBlock;
    const int P = (int)r->prompt.size();
    // Algorithm 2: the longest cached prefix, but at least the last prompt token is computed
    int matched = 0;
    std::vector<int32_t> hit((size_t)std::max(1, (P - 1) / bs));
    if (e->cfg.prefix_cache) {
        const dk_status s = dk_prefix_index_match(e->index, r->prompt.data(), P, (P - 1) / bs, hit.data(), &matched);
        if (s != DK_OK) return s;
    }
    for (int i = 0; i < matched; i++) {
        const dk_status s = dk_kv_retain_block(e->pool, hit[(size_t)i]);
        if (s != DK_OK) { engine_release_blocks(e, r); return s; }
        r->blocks.push_back(hit[(size_t)i]);
    }
    const int need = (P + bs - 1) / bs;
    while ((int)r->blocks.size() < need) {
        int32_t b = -1;
        const dk_status s = engine_alloc_block(e, &b);
        if (s != DK_OK) { engine_release_blocks(e, r); return s; }
        r->blocks.push_back(b);
    }
    const int start = matched * bs;
    r->reused = start;
    const int row = (int)e->active.size();
    engine_set_row(e, row, r);
    dk_status s = engine_upload_rows(e, st);
    if (s != DK_OK) { engine_release_blocks(e, r); return s; }
    const int32_t *d_table = e->d_tables + (size_t)row * e->cfg.max_blocks_per_seq;
    for (int o = start; o < P; o += e->cfg.prefill_chunk) {
        const int n = std::min(e->cfg.prefill_chunk, P - o);
        const bool last = o + n >= P;
        DK_HIP(hipMemcpyAsync(e->d_chunk, r->prompt.data() + o, (size_t)n * 4, hipMemcpyHostToDevice, st));
        s = dk_prefill_chunk(e->model, e->pool, d_table, e->cfg.max_blocks_per_seq, o, e->d_chunk, n, e->d_ws,
                             e->ws_bytes, (last && e->sampling) ? e->d_logits : nullptr, last ? e->d_next : nullptr, st);
        if (s != DK_OK) { engine_release_blocks(e, r); return s; }
        if (last) {
            int32_t first = 0;
            const int32_t *d_first = e->d_next + (n - 1);
            if (e->sampling) {
                // the prompt's last position decides the first token: one row through the sampler
                const dk_model_config &mc = e->model->cfg;
                s = dk_sample_tokens(e->d_logits + (size_t)(n - 1) * mc.vocab, 1, mc.vocab, &e->sampling_params,
                                     e->sample_step++, e->d_sample_ws, e->sample_ws_bytes, e->d_sampled, st);
                if (s != DK_OK) { engine_release_blocks(e, r); return s; }
                d_first = e->d_sampled;
            }
            DK_HIP(hipMemcpyAsync(&first, d_first, 4, hipMemcpyDeviceToHost, st));
            DK_HIP(hipStreamSynchronize(st));
            r->out.push_back(first);
            r->last = first;
        } else {
            DK_HIP(hipStreamSynchronize(st));   // the prompt chunk buffer is reused by the next chunk
        }
    }
    r->T = P;
    e->stats.prefill_tokens += P - start;
    e->stats.reused_tokens += start;
    e->stats.generated_tokens += 1;
    // Algorithm 2's store: the prompt's full blocks become reusable
    if (e->cfg.prefix_cache && P / bs > 0) {
        s = dk_prefix_index_insert(e->index, e->pool, r->prompt.data(), P / bs, r->blocks.data(), nullptr);
        if (s != DK_OK) return s;
    }
    r->state = DK_REQ_ACTIVE;
    e->active.push_back(r);
    return DK_OK;
}

// Takes a row out of the running batch: its blocks are released and the last row moves into the hole
void engine_retire(dk_engine *e, size_t row, int state)
{
    EngineRequest *r = e->active[row];
    engine_release_blocks(e, r);
    r->state = state;
    const size_t last = e->active.size() - 1;
    if (row != last) {
        e->active[row] = e->active[last];
        engine_set_row(e, (int)row, e->active[row]);
    }
    e->active.pop_back();
}

}  // namespace

dk_status dk_engine_device_bytes(const dk_model *model, const dk_engine_config *cfg, size_t *out_bytes)
{
    if (!out_bytes) return fail(DK_E_INVALID_ARG, "NULL argument");
    ArenaLayout L{};
    const dk_status s = engine_layout(model, cfg, &L);
    if (s != DK_OK) return s;
    *out_bytes = L.total;
    return DK_OK;
}

dk_status dk_engine_create(dk_model *model, dk_kv_pool *pool, const dk_engine_config *cfg, void *d_arena,
                           size_t arena_bytes, dk_engine **out)
{
    if (!model || !pool || !cfg || !d_arena || !out) return fail(DK_E_INVALID_ARG, "NULL argument");
    ArenaLayout L{};
    dk_status s = engine_layout(model, cfg, &L);
    if (s != DK_OK) return s;
    if ((uintptr_t)d_arena % 256) return fail(DK_E_INVALID_ARG, "arena must be 256-byte aligned");
    if (arena_bytes < L.total)
        return fail(DK_E_WORKSPACE_TOO_SMALL, "arena %zu bytes, %zu needed", arena_bytes, L.total);
    std::unique_ptr<dk_engine> e(new dk_engine());
    e->model = model;
    e->pool = pool;
    e->cfg = *cfg;
    if ((s = dk_prefix_index_create(dk_prefix_index::kBlock, &e->index)) != DK_OK) return s;
    char *base = static_cast<char *>(d_arena);
    e->d_tables = reinterpret_cast<int32_t *>(base + L.tables);
    e->d_seq = reinterpret_cast<int32_t *>(base + L.seq);
    e->d_tok = reinterpret_cast<int32_t *>(base + L.tok);
    e->d_next = reinterpret_cast<int32_t *>(base + L.next);
    e->d_chunk = reinterpret_cast<int32_t *>(base + L.chunk);
    e->d_ws = base + L.ws;
    e->d_logits = reinterpret_cast<float *>(base + L.logits);
    e->d_sample_ws = base + L.sample_ws;
    e->sample_ws_bytes = L.sample_ws_bytes;
    e->d_sampled = reinterpret_cast<int32_t *>(base + L.sampled);
    e->ws_bytes = L.ws_bytes;
    e->h_tables.assign((size_t)cfg->max_batch * cfg->max_blocks_per_seq, -1);
    e->row_dirty.assign((size_t)cfg->max_batch, 1);
    *out = e.release();
    return DK_OK;
}

dk_status dk_engine_destroy(dk_engine *engine)
{
    if (!engine) return DK_OK;
    for (auto &kv : engine->all) engine_release_blocks(engine, kv.second.get());
    (void)dk_prefix_index_destroy(engine->index, engine->pool);
    delete engine;
    return DK_OK;
}

dk_status dk_engine_submit(dk_engine *engine, const int32_t *h_prompt, int32_t n_prompt,
                           int32_t max_new_tokens, int32_t eos_token, int64_t *out_id)
{
    if (!engine || !h_prompt || !out_id) return fail(DK_E_INVALID_ARG, "NULL argument");
    if (n_prompt < 1 || max_new_tokens < 1)
        return fail(DK_E_INVALID_ARG, "prompt of %d tokens, %d new tokens", n_prompt, max_new_tokens);
    const int64_t room = (int64_t)engine->cfg.max_blocks_per_seq * dk_prefix_index::kBlock;
    // the last generated token is never fed back, so it needs no cache position
    if ((int64_t)n_prompt + max_new_tokens - 1 > room)
        return fail(DK_E_INVALID_ARG, "prompt %d + output %d exceed %lld cache positions", n_prompt,
                    max_new_tokens, (long long)room);
    std::unique_ptr<EngineRequest> r(new EngineRequest());
    r->id = engine->next_id++;
    r->prompt.assign(h_prompt, h_prompt + n_prompt);
    r->max_new = max_new_tokens;
    r->eos = eos_token;
    *out_id = r->id;
    engine->queue.push_back(r.get());
    engine->all[r->id] = std::move(r);
    return DK_OK;
}

dk_status dk_engine_step(dk_engine *engine, void *hip_stream, int32_t *out_active)
{
    if (!engine) return fail(DK_E_INVALID_ARG, "NULL argument");
    dk_engine *e = engine;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int bs = dk_prefix_index::kBlock;
    bool worked = false;

    // admission happens only here, between two decode steps: fill free rows from the waiting queue
    while ((int)e->active.size() < e->cfg.max_batch && !e->queue.empty()) {
        EngineRequest *r = e->queue.front();
        const dk_status s = engine_admit(e, r, st);
        if (s == DK_E_POOL_EXHAUSTED) {
            if (!e->active.empty()) break;     // retry when a request has left and freed blocks
            e->queue.pop_front();              // nobody will free anything: it can never run
            r->state = DK_REQ_FAILED;
            worked = true;
            continue;
        }
        if (s != DK_OK) return s;
        e->queue.pop_front();
        worked = true;
        if (engine_finished(r)) engine_retire(e, e->active.size() - 1, DK_REQ_DONE);
    }

    // one batched decode step advances every running row by a token
    if (!e->active.empty()) {
        // a sequence whose next position starts a block needs that block first
        for (size_t row = 0; row < e->active.size();) {
            EngineRequest *r = e->active[row];
            if (r->T % bs == 0 && (int)r->blocks.size() <= r->T / bs) {
                int32_t b = -1;
                const dk_status s = engine_alloc_block(e, &b);
                if (s == DK_E_POOL_EXHAUSTED) { engine_retire(e, row, DK_REQ_FAILED); continue; }
                if (s != DK_OK) return s;
                r->blocks.push_back(b);
                engine_set_row(e, (int)row, r);
            }
            row++;
        }
    }
    if (!e->active.empty()) {
        const int B = (int)e->active.size();
        std::vector<int32_t> seq((size_t)B), tok((size_t)B), nxt((size_t)B), smp((size_t)B);
        const dk_model_config &mc = e->model->cfg;
        for (int i = 0; i < B; i++) { seq[(size_t)i] = e->active[(size_t)i]->T; tok[(size_t)i] = e->active[(size_t)i]->last; }
        dk_status s = engine_upload_rows(e, st);
        if (s != DK_OK) return s;
        auto upload_state = [&]() -> dk_status {
            DK_HIP(hipMemcpyAsync(e->d_seq, seq.data(), (size_t)B * 4, hipMemcpyHostToDevice, st));
            DK_HIP(hipMemcpyAsync(e->d_tok, tok.data(), (size_t)B * 4, hipMemcpyHostToDevice, st));
            return DK_OK;
        };
        if (e->state_dirty) {
            s = upload_state();
            if (s != DK_OK) return s;
            e->state_dirty = false;
        }
        // the step feeds its own (greedy) tokens and lengths to the next one (an invalid step advances
        // nothing); with sampling the drawn tokens then replace the greedy ones on the device
        for (int attempt = 0; attempt < 2; attempt++) {
            s = dk_decode_step(e->model, e->pool, e->d_tables, e->cfg.max_blocks_per_seq, e->d_seq, e->d_tok, B,
                               e->d_ws, e->ws_bytes, e->sampling ? e->d_logits : nullptr, e->d_next,
                               DK_STEP_ADVANCE | (e->no_fused ? DK_STEP_NO_FUSED : 0u), st);
            if (s != DK_OK) return s;
            DK_HIP(hipMemcpyAsync(nxt.data(), e->d_next, (size_t)B * 4, hipMemcpyDeviceToHost, st));
            if (e->sampling) {
                // the greedy tokens above still tell whether the step was valid; the sampled ones are used
                s = dk_sample_tokens(e->d_logits, B, mc.vocab, &e->sampling_params, e->sample_step, e->d_sample_ws,
                                     e->sample_ws_bytes, e->d_sampled, st);
                if (s != DK_OK) return s;
                DK_HIP(hipMemcpyAsync(smp.data(), e->d_sampled, (size_t)B * 4, hipMemcpyDeviceToHost, st));
                DK_HIP(hipMemcpyAsync(e->d_tok, e->d_sampled, (size_t)B * 4, hipMemcpyDeviceToDevice, st));
            }
            DK_HIP(hipStreamSynchronize(st));
            bool valid = true;   // an invalid step marks every row with -1; check them all
            for (int i = 0; i < B; i++) valid = valid && nxt[(size_t)i] >= 0;
            if (valid) break;
            if (e->sampling) {   // tokens drawn from an invalid step's logits went to the device: restore
                s = upload_state();
                if (s != DK_OK) return s;
            }
            // the persistent kernel could not keep its blocks resident (its waits are bounded and it
            // says so with the token -1): the step left lengths and tokens alone, so it is simply
            // repeated, now and from here on as a chain of kernels
            if (attempt == 1) return fail(DK_E_HIP, "decode step reported an invalid result twice");
            e->no_fused = true;
            (void)dk_workspace_reset(e->model);
        }
        e->stats.decode_steps++;
        e->stats.generated_tokens += B;
        if (e->sampling) {
            e->sample_step++;
            nxt = smp;
        }
        for (int i = 0; i < B; i++) {
            EngineRequest *r = e->active[(size_t)i];
            r->out.push_back(nxt[(size_t)i]);
            r->last = nxt[(size_t)i];
            r->T++;
        }
        // rows that reached their length or their stop token retire now, so the next call can refill them
        for (size_t row = 0; row < e->active.size();) {
            if (engine_finished(e->active[row])) engine_retire(e, row, DK_REQ_DONE);
            else row++;
        }
        worked = true;
    }
    if (worked) e->stats.iterations++;
    if (out_active) *out_active = (int32_t)(e->active.size() + e->queue.size());
    return DK_OK;
}

dk_status dk_engine_set_sampling(dk_engine *engine, const dk_sampling *params)
{
    if (!engine) return fail(DK_E_INVALID_ARG, "NULL argument");
    if (!params) {
        engine->sampling = false;
        return DK_OK;
    }
    if (!(params->temperature > 0.f) || params->top_k < 0 || !(params->top_p > 0.f) || params->top_p > 1.f)
        return fail(DK_E_INVALID_ARG, "sampling parameters: temperature %g (> 0), top_k %d (>= 0), top_p %g (0 < p <= 1)",
                    (double)params->temperature, params->top_k, (double)params->top_p);
    engine->sampling = true;
    engine->sampling_params = *params;
    engine->sample_step = 0;
    return DK_OK;
}

dk_status dk_engine_poll(const dk_engine *engine, int64_t id, int32_t *h_out_tokens, int32_t capacity,
                         int32_t *out_n, int32_t *out_state, int32_t *out_reused)
{
    if (!engine || !out_n || !out_state || (capacity > 0 && !h_out_tokens))
        return fail(DK_E_INVALID_ARG, "NULL argument");
    auto it = engine->all.find(id);
    if (it == engine->all.end()) return fail(DK_E_INVALID_ARG, "unknown request %lld", (long long)id);
    const EngineRequest *r = it->second.get();
    const int n = (int)r->out.size();
    std::copy(r->out.begin(), r->out.begin() + std::min(n, std::max(capacity, 0)), h_out_tokens);
    *out_n = n;
    *out_state = r->state;
    if (out_reused) *out_reused = r->reused;
    return DK_OK;
}

dk_status dk_engine_forget(dk_engine *engine, int64_t id)
{
    if (!engine) return fail(DK_E_INVALID_ARG, "NULL argument");
    auto it = engine->all.find(id);
    if (it == engine->all.end()) return fail(DK_E_INVALID_ARG, "unknown request %lld", (long long)id);
    const int st = it->second->state;
    if (st != DK_REQ_DONE && st != DK_REQ_FAILED)
        return fail(DK_E_INVALID_ARG, "request %lld is still running", (long long)id);
    engine->all.erase(it);
    return DK_OK;
}

dk_status dk_engine_get_stats(const dk_engine *engine, dk_engine_stats *out)
{
    if (!engine || !out) return fail(DK_E_INVALID_ARG, "NULL argument");
    *out = engine->stats;
    out->cached_blocks = engine->index->size();
    out->active = (int32_t)engine->active.size();
    out->pending = (int32_t)engine->queue.size();
    return DK_OK;
}
