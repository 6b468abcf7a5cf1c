"""Host tests of the block-granular prefix cache (no GPU): the chain index
against a plain restatement of the paper's prefix-cache lookup (Algorithm 2:
try the whole prompt, then every shorter prefix from the longest down, return
the cached state and the start position), restricted to block boundaries, with
least-recently-used eviction checked against a brute-force model."""
import numpy as np
import pytest

import workloads as W
import paper_2601_19139_amd as dk

BS = 16


def make_pool(n_blocks):
    cfg = dk.DkModelConfig.from_shape(W.CONFIGS["tiny"])
    return dk.create_kv_pool(cfg, n_blocks, BS, 0x1000, dk.kv_pool_bytes(cfg, n_blocks, BS))


class ReferenceCache:
    """Algorithm 2 with exact keys instead of digests: a dict from a token prefix (a tuple
    whose length is a multiple of the block size) to the block holding its last 16 tokens."""

    def __init__(self):
        self.entries = {}

    def lookup(self, prompt, max_blocks):
        # longest first, as the algorithm's loop does
        for nb in range(min(max_blocks, len(prompt) // BS), 0, -1):
            key = tuple(prompt[:nb * BS])
            if key in self.entries:
                # a cached prefix implies its own prefixes are cached (chains are stored whole)
                return [self.entries[tuple(prompt[:(i + 1) * BS])] for i in range(nb)]
        return []

    def store(self, prompt, blocks):
        adopted = 0
        for i, b in enumerate(blocks):
            key = tuple(prompt[:(i + 1) * BS])
            if key not in self.entries:
                self.entries[key] = b
                adopted += 1
        return adopted


def test_lookup_matches_the_longest_prefix_search():
    rng = np.random.default_rng(5)
    pool = make_pool(400)
    idx = dk.prefix_index_create(BS)
    ref = ReferenceCache()
    stems = [rng.integers(0, 50, size=rng.integers(16, 90)) for _ in range(6)]
    for trial in range(60):
        stem = stems[rng.integers(len(stems))]
        cut = rng.integers(1, len(stem) + 1)
        prompt = np.concatenate([stem[:cut], rng.integers(0, 50, size=rng.integers(0, 40))]).astype(np.int32)
        max_blocks = (len(prompt) - 1) // BS           # the engine's rule: the last token is always computed
        got = dk.prefix_index_match(idx, prompt, max_blocks)
        want = ref.lookup(list(prompt), max_blocks)
        assert list(got) == want, (trial, got, want)
        # "compute" the rest and store the prompt's full blocks
        n_full = len(prompt) // BS
        blocks = list(got) + [dk.kv_alloc_block(pool) for _ in range(n_full - len(got))]
        adopted = dk.prefix_index_insert(idx, pool, prompt, blocks)
        assert adopted == ref.store(list(prompt), blocks)
        # the request ends: its own references go, the cache's stay
        for b in blocks[len(got):]:
            dk.kv_release_block(pool, b)
        assert dk.prefix_index_size(idx) == len(ref.entries)
    # every cached block is held exactly once (by the index), every other block is free
    held = set(ref.entries.values())
    assert dk.kv_free_blocks(pool) == 400 - len(held)
    for b in held:
        assert dk.kv_refcount(pool, b) == 1
    dk.prefix_index_destroy(idx, pool)
    assert dk.kv_free_blocks(pool) == 400
    dk.destroy_kv_pool(pool)


def test_lru_eviction_order_and_pins():
    pool = make_pool(16)
    idx = dk.prefix_index_create(BS)

    def cached(prompt):
        """Stores a prompt whose blocks nobody keeps using; returns its blocks."""
        n = len(prompt) // BS
        hit = list(dk.prefix_index_match(idx, prompt, n))
        blocks = hit + [dk.kv_alloc_block(pool) for _ in range(n - len(hit))]
        dk.prefix_index_insert(idx, pool, prompt, blocks)
        for b in blocks[len(hit):]:
            dk.kv_release_block(pool, b)
        return blocks

    a = np.arange(48, dtype=np.int32)                       # chain a0 -> a1 -> a2
    b = np.concatenate([a[:16], 100 + np.arange(16)]).astype(np.int32)   # a0 -> b1
    c = (200 + np.arange(16)).astype(np.int32)              # c0
    ba, bb, bc = cached(a), cached(b), cached(c)
    assert ba[0] == bb[0] and dk.prefix_index_size(idx) == 5
    # touch chain a (a lookup marks its entries as just used); c and b1 are older now
    assert list(dk.prefix_index_match(idx, a, 3)) == ba
    # a request still uses b1: it must not be dropped
    dk.kv_retain_block(pool, bb[1])
    # victims: only entries without cached successors and without users, oldest first.
    # order of last use: b1 (pinned), c0, then a0,a1,a2 (a0 has successors)
    assert dk.prefix_index_evict_lru(idx, pool) == bc[0]
    assert dk.prefix_index_evict_lru(idx, pool) == ba[2]
    assert dk.prefix_index_evict_lru(idx, pool) == ba[1]
    # a0 still has the successor b1, b1 is pinned: nothing can go
    with pytest.raises(dk.DecodeKitError) as e:
        dk.prefix_index_evict_lru(idx, pool)
    assert e.value.status == "DK_E_POOL_EXHAUSTED"
    dk.kv_release_block(pool, bb[1])
    assert dk.prefix_index_evict_lru(idx, pool) == bb[1]
    assert dk.prefix_index_evict_lru(idx, pool) == ba[0]
    assert dk.prefix_index_size(idx) == 0 and dk.kv_free_blocks(pool) == 16
    # a dropped chain is gone from lookups
    assert len(dk.prefix_index_match(idx, a, 3)) == 0
    dk.prefix_index_destroy(idx, pool)
    dk.destroy_kv_pool(pool)


def test_engine_argument_checks_on_the_host():
    shape = W.CONFIGS["tiny"]
    cfg = dk.DkModelConfig.from_shape(shape)
    ptrs, keep = fake_weights(shape)
    m = dk.create_model(cfg, ptrs)
    pool = make_pool(8)
    ok = dk.EngineConfig(4, 8, 16, 1)
    need = dk.engine_device_bytes(m, ok)
    assert need > 0 and need % 256 == 0
    for bad in (dk.EngineConfig(0, 8, 16, 1), dk.EngineConfig(65, 8, 16, 1), dk.EngineConfig(4, 0, 16, 1),
                dk.EngineConfig(4, 8, 0, 1), dk.EngineConfig(4, 8, 65, 1)):
        with pytest.raises(dk.DecodeKitError) as e:
            dk.engine_device_bytes(m, bad)
        assert e.value.status == "DK_E_INVALID_ARG"
    with pytest.raises(dk.DecodeKitError) as e:
        dk.engine_create(m, pool, ok, 0x1000, need - 1)
    assert e.value.status == "DK_E_WORKSPACE_TOO_SMALL"
    with pytest.raises(dk.DecodeKitError) as e:
        dk.engine_create(m, pool, ok, 0x1001, need)
    assert "aligned" in str(e.value)
    eng = dk.engine_create(m, pool, ok, 0x1000, need)        # the arena is not touched before a step
    with pytest.raises(dk.DecodeKitError):
        dk.engine_submit(eng, np.zeros(0, np.int32), 4)
    with pytest.raises(dk.DecodeKitError):
        dk.engine_submit(eng, np.zeros(4, np.int32), 0)
    with pytest.raises(dk.DecodeKitError) as e:
        dk.engine_submit(eng, np.zeros(100, np.int32), 30)   # 129 positions > 8 blocks
    assert "exceed" in str(e.value)
    rid = dk.engine_submit(eng, np.zeros(100, np.int32), 29)
    toks, state, reused = dk.engine_poll(eng, rid)
    assert len(toks) == 0 and state == "pending" and reused == 0
    with pytest.raises(dk.DecodeKitError):
        dk.engine_forget(eng, rid)                            # still pending
    with pytest.raises(dk.DecodeKitError):
        dk.engine_poll(eng, rid + 1)
    st = dk.engine_stats(eng)
    assert st["pending"] == 1 and st["active"] == 0 and st["cached_blocks"] == 0
    dk.engine_destroy(eng)
    dk.destroy_kv_pool(pool)
    dk.destroy_model(m)


def fake_weights(shape):
    """Weight pointers that are never dereferenced on the host."""
    layers = (dk.LayerWeights * shape.n_layers)()
    for i in range(shape.n_layers):
        for name, _ in dk.LayerWeights._fields_:
            setattr(layers[i], name, 0x1000)
    return dk.WeightPtrs(0x1000, 0x1000, 0x1000, layers), layers
