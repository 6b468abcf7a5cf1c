"""Seeded bf16 bit patterns for weights, KV contexts and start tokens.

Every tensor is addressed by (seed, tensor name, chunk index) through a
counter-based generator (Philox), so any tensor can be regenerated on its own
and large models never need a second host copy.  All arrays are uint16 bf16 bit
patterns: data for both the CPU oracle and the HIP path, which each do their
own arithmetic on them.
"""
import os
import zlib
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .configs import ModelConfig

BF16_NAN_BITS = 0x7FC0
_CHUNK = 1 << 22          # elements per independently keyed chunk


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest, ties to even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> float32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _name_key(name: str) -> int:
    return zlib.crc32(name.encode()) | (len(name) << 32)


def _chunk_normal(seed, key, chunk, n, std, mean):
    bitgen = np.random.Philox(key=np.array([seed, key], dtype=np.uint64),
                              counter=np.array([0, 0, chunk, 0], dtype=np.uint64))
    g = np.random.Generator(bitgen)
    x = g.standard_normal(n, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return bf16_bits_from_f32(x)


_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        _POOL = ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1)))
    return _POOL


def normal_bf16(seed: int, name: str, shape, std: float = 1.0, mean: float = 0.0,
                out: np.ndarray = None) -> np.ndarray:
    """bf16(N(mean, std)) bit patterns of the given shape for (seed, name)."""
    n = int(np.prod(shape))
    res = out.reshape(-1) if out is not None else np.empty(n, dtype=np.uint16)
    assert res.size == n and res.dtype == np.uint16
    key = _name_key(name)
    nchunks = (n + _CHUNK - 1) // _CHUNK

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        res[lo:hi] = _chunk_normal(seed, key, c, hi - lo, std, mean)

    if nchunks <= 1:
        for c in range(nchunks):
            work(c)
    else:
        list(_pool().map(work, range(nchunks)))
    return res.reshape(shape)


def layer_tensor_shapes(cfg: ModelConfig):
    """name -> (shape, std, mean) for one layer.  Matrices are W[out, in]."""
    H, d = cfg.hidden, cfg.head_dim
    t = {
        "g_attn": ((H,), 0.02, 1.0),
        "wq": ((cfg.q_dim, H), 0.02, 0.0),
        "wk": ((cfg.kv_dim, H), 0.02, 0.0),
        "wv": ((cfg.kv_dim, H), 0.02, 0.0),
        "wo": ((H, cfg.q_dim), 0.02, 0.0),
        "g_mlp": ((H,), 0.02, 1.0),
    }
    if cfg.qk_norm:
        t["g_q"] = ((d,), 0.02, 1.0)
        t["g_k"] = ((d,), 0.02, 1.0)
    if cfg.n_experts:
        E, Fe = cfg.n_experts, cfg.expert_ffn
        t["w_router"] = ((E, H), 0.02, 0.0)
        t["w_gate"] = ((E, Fe, H), 0.02, 0.0)
        t["w_up"] = ((E, Fe, H), 0.02, 0.0)
        t["w_down"] = ((E, H, Fe), 0.02, 0.0)
    else:
        F = cfg.ffn
        t["w_gate"] = ((F, H), 0.02, 0.0)
        t["w_up"] = ((F, H), 0.02, 0.0)
        t["w_down"] = ((H, F), 0.02, 0.0)
    return t


def normal_bf16_many(seed: int, specs: dict) -> dict:
    """Several tensors at once: specs maps name -> (shape, std, mean).  Same
    values as one normal_bf16 call per name; all chunks share the thread pool."""
    outs, tasks = {}, []
    for name, (shape, std, mean) in specs.items():
        n = int(np.prod(shape))
        res = np.empty(n, dtype=np.uint16)
        outs[name] = res.reshape(shape)
        key = _name_key(name)
        for c in range((n + _CHUNK - 1) // _CHUNK):
            tasks.append((res, key, c, min(n, (c + 1) * _CHUNK) - c * _CHUNK, std, mean))

    def work(t):
        res, key, c, m, std, mean = t
        res[c * _CHUNK: c * _CHUNK + m] = _chunk_normal(seed, key, c, m, std, mean)

    list(_pool().map(work, tasks))
    return outs


def make_layer(cfg: ModelConfig, seed: int, layer: int):
    specs = {f"layer{layer}.{k}": v for k, v in layer_tensor_shapes(cfg).items()}
    out = normal_bf16_many(seed, specs)
    return {k.split(".", 1)[1]: v for k, v in out.items()}


def make_weights(cfg: ModelConfig, seed: int = 0, layers=None):
    """All weights of the model as uint16 bf16 bit patterns.

    Matrices are bf16(N(0, 0.02)); norm gains are bf16(1 + N(0, 0.02)) so that a
    missing or misplaced gain is visible.  `layers` limits which layers are
    generated (others are None), for models too large to hold at once.
    """
    V, H = cfg.vocab, cfg.hidden
    specs = {"embed": ((V, H), 0.02, 0.0), "g_final": ((H,), 0.02, 1.0)}
    if not cfg.tie_lm_head:
        specs["lm_head"] = ((V, H), 0.02, 0.0)
    want = range(cfg.n_layers) if layers is None else layers
    for l in want:
        for k, v in layer_tensor_shapes(cfg).items():
            specs[f"layer{l}.{k}"] = v
    t = normal_bf16_many(seed, specs)
    w = {"embed": t["embed"], "g_final": t["g_final"]}
    w["lm_head"] = t["embed"] if cfg.tie_lm_head else t["lm_head"]
    w["layers"] = [{k: t[f"layer{l}.{k}"] for k in layer_tensor_shapes(cfg)} if l in want else None
                   for l in range(cfg.n_layers)]
    return w


def pool_shape(cfg: ModelConfig, num_blocks: int, block_size: int):
    """KV pool dims: [layer][block][K|V][kv_head][slot][dim], dense, C order."""
    return (cfg.n_layers, num_blocks, 2, cfg.n_kv_heads, block_size, cfg.head_dim)


def fill_kv_pool(cfg: ModelConfig, layout, seed: int = 1, poison: bool = True) -> np.ndarray:
    """A KV pool whose live slots hold bf16(N(0,1)) and whose other slots hold
    a poison pattern (bf16 NaN) so that any read past a sequence's length, or
    of a block no table names, shows up in the result."""
    shp = pool_shape(cfg, layout.num_blocks, layout.block_size)
    pool = normal_bf16(seed, "kv_pool", shp, 1.0)
    if poison:
        live = layout.live_slot_mask()                    # [num_blocks, block_size] bool
        dead = ~live
        pool[:, dead[:, None, None, :].repeat(2, 1).repeat(cfg.n_kv_heads, 2)] = BF16_NAN_BITS
    return pool


def initial_tokens(cfg: ModelConfig, batch: int, seed: int = 2) -> np.ndarray:
    g = np.random.Generator(np.random.Philox(key=np.array([seed, _name_key("tokens")], dtype=np.uint64)))
    return g.integers(0, cfg.vocab, size=batch, dtype=np.int32)
