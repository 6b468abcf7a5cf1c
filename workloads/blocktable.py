"""Block tables for a paged KV pool with shareable prefix blocks.

A sequence's cached tokens live in fixed-size blocks of a common pool; its
block table lists the physical block ids in logical order.  Sequences that
resumed from the same cached prefix (the paper's text prefix cache lookup,
Algorithm 2, returns a KV state and a start position) name the same physical
blocks for that prefix.  Physical ids come from a seeded shuffle so that code
which assumes contiguous placement fails.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class BlockLayout:
    block_size: int
    num_blocks: int
    tables: np.ndarray        # int32 [B, max_blocks]; -1 where unused
    contexts: np.ndarray      # int32 [B] tokens cached before the first step
    refcount: np.ndarray      # int32 [num_blocks]
    shared_prefix: int
    sharers: tuple

    @property
    def max_blocks(self) -> int:
        return self.tables.shape[1]

    def live_slot_mask(self) -> np.ndarray:
        """[num_blocks, block_size] bool: slots that hold a cached token."""
        m = np.zeros((self.num_blocks, self.block_size), dtype=bool)
        for b, T in enumerate(self.contexts):
            for t in range(int(T)):
                m[self.tables[b, t // self.block_size], t % self.block_size] = True
        return m

    def unique_live_tokens(self, extra: int = 0) -> int:
        """Cached tokens counted once per physical slot (shared prefix once)."""
        priv = int(sum(int(T) + extra for T in self.contexts))
        return priv - self.shared_prefix * max(0, len(self.sharers) - 1)


def draw_contexts(batch, lo, hi, shared_prefix, n_sharers, seed):
    """Context lengths: sharers (the first n_sharers rows) are drawn above the
    shared prefix so each has at least one private token."""
    g = np.random.Generator(np.random.Philox(key=np.array([seed, 0xC0FFEE], dtype=np.uint64)))
    ctx = np.empty(batch, dtype=np.int32)
    for b in range(batch):
        l = max(lo, shared_prefix + 1) if b < n_sharers else lo
        ctx[b] = g.integers(l, hi + 1)
    return ctx


def build_block_tables(contexts, block_size, steps, shared_prefix=0, n_sharers=0,
                       seed=3, spare_blocks=0) -> BlockLayout:
    """Tables with room for `steps` appended tokens per sequence.

    The first `n_sharers` sequences point at one set of physical blocks for
    their first `shared_prefix` tokens (a multiple of the block size, so no
    partly filled block is shared and no shared block is ever an append
    target)."""
    contexts = np.asarray(contexts, dtype=np.int32)
    B = len(contexts)
    assert shared_prefix % block_size == 0
    n_shared_blocks = shared_prefix // block_size
    sharers = tuple(range(n_sharers)) if n_shared_blocks else ()
    for b in sharers:
        assert contexts[b] > shared_prefix
    need = [(int(T) + steps + block_size - 1) // block_size for T in contexts]
    max_blocks = max(need)
    total = sum(need) - n_shared_blocks * max(0, len(sharers) - 1) + spare_blocks
    g = np.random.Generator(np.random.Philox(key=np.array([seed, 0xB10C], dtype=np.uint64)))
    ids = g.permutation(total).astype(np.int32)
    nxt = 0
    tables = np.full((B, max_blocks), -1, dtype=np.int32)
    refcount = np.zeros(total, dtype=np.int32)
    shared_ids = ids[nxt:nxt + n_shared_blocks] if sharers else ids[:0]
    nxt += len(shared_ids)
    for b in range(B):
        k = 0
        if b in sharers:
            tables[b, :n_shared_blocks] = shared_ids
            refcount[shared_ids] += 1
            k = n_shared_blocks
        m = need[b] - k
        tables[b, k:need[b]] = ids[nxt:nxt + m]
        refcount[ids[nxt:nxt + m]] += 1
        nxt += m
    return BlockLayout(block_size, total, tables, contexts.copy(), refcount,
                       shared_prefix if sharers else 0, sharers)


def layout_for(workload) -> BlockLayout:
    """The block layout of a named workload."""
    w = workload
    if w.contexts is not None:
        ctx = np.asarray(w.contexts, dtype=np.int32)
    else:
        ctx = draw_contexts(w.batch, w.context_range[0], w.context_range[1],
                            w.shared_prefix, w.n_sharers, w.seed_blocks)
    return build_block_tables(ctx, w.block_size, w.steps, w.shared_prefix, w.n_sharers,
                              seed=w.seed_blocks)
