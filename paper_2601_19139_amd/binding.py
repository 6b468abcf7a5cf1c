"""ctypes binding of include/decodekit.h and include/dk_engine.h: same names
without the dk_ prefix, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DECODEKIT_LIBRARY names another build of the same library (the host-sanitizer build of the tests)
LIB_PATH = os.environ.get("DECODEKIT_LIBRARY") or os.path.join(_HERE, "libdecodekit.so")

STATUS = {0: "DK_OK", -1: "DK_E_INVALID_ARG", -2: "DK_E_POOL_EXHAUSTED", -3: "DK_E_BAD_BLOCK",
          -4: "DK_E_WORKSPACE_TOO_SMALL", -5: "DK_E_UNSUPPORTED_SHAPE", -6: "DK_E_HIP"}
STEP_ADVANCE = 1
STEP_PROFILE = 2
STEP_NO_FUSED = 4
KERNEL_CLASSES = ("embed", "gemv", "gemm", "attention", "moe_router", "moe_expert", "moe_combine", "argmax", "fused_step")


class DecodeKitError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"{STATUS.get(code, code)}: {text}")
        self.code = code
        self.status = STATUS.get(code, str(code))


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
        "qk_norm", "n_experts", "top_k", "expert_ffn", "tie_lm_head")] + [
        ("rms_eps", C.c_double), ("rope_theta", C.c_double)]

    @classmethod
    def from_shape(cls, cfg):
        """From any object with the fields of workloads.ModelConfig."""
        return cls(cfg.n_layers, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn,
                   cfg.vocab, int(cfg.qk_norm), cfg.n_experts, cfg.top_k, cfg.expert_ffn,
                   int(cfg.tie_lm_head), cfg.rms_eps, cfg.rope_theta)


LAYER_FIELDS = ("g_attn", "w_qkv", "g_q", "g_k", "w_o", "g_mlp", "w_gate", "w_up", "w_down",
                "w_router")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class WeightPtrs(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("g_final", C.c_void_p),
                ("layers", C.POINTER(LayerWeights))]


_SIGNATURES = {
    "dk_last_error": (C.c_char_p, []),
    "dk_version": (C.c_char_p, []),
    "dk_kv_pool_bytes": (C.c_int32, [C.POINTER(ModelConfig), C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]),
    "dk_create_kv_pool": (C.c_int32, [C.POINTER(ModelConfig), C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_void_p)]),
    "dk_destroy_kv_pool": (C.c_int32, [C.c_void_p]),
    "dk_kv_alloc_block": (C.c_int32, [C.c_void_p, C.POINTER(C.c_int32)]),
    "dk_kv_alloc_block_id": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_kv_retain_block": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_kv_release_block": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_kv_refcount": (C.c_int32, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]),
    "dk_kv_free_blocks": (C.c_int32, [C.c_void_p, C.POINTER(C.c_int32)]),
    "dk_kv_offset": (C.c_int32, [C.c_void_p] + [C.c_int32] * 6 + [C.POINTER(C.c_int64)]),
    "dk_kv_validate_tables": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]),
    "dk_append_kv": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                 C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_create_model": (C.c_int32, [C.POINTER(ModelConfig), C.POINTER(WeightPtrs), C.POINTER(C.c_void_p)]),
    "dk_create_model_q4": (C.c_int32, [C.POINTER(ModelConfig), C.POINTER(WeightPtrs), C.POINTER(C.c_void_p)]),
    "dk_destroy_model": (C.c_int32, [C.c_void_p]),
    "dk_workspace_bytes": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]),
    "dk_decode_step": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                   C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p,
                                   C.c_uint32, C.c_void_p]),
    "dk_decode_step_static": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]),
    "dk_prefill_chunk": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_workspace_reset": (C.c_int32, [C.c_void_p]),
    "dk_debug_set_wait_limit": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_debug_set_stage_stamps": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t]),
    "dk_fused_status": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_profile_read": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]),
    "dk_step_routing": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "dk_read_stream": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "dk_step_algorithmic_bytes": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                              C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_uint64)]),
}

class Sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_k", C.c_int32), ("top_p", C.c_float), ("seed", C.c_uint64)]


class EngineConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("max_batch", "max_blocks_per_seq", "prefill_chunk", "prefix_cache")]


class EngineStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("iterations", "decode_steps", "generated_tokens", "prefill_tokens",
                                          "reused_tokens", "evictions")] + [
        (n, C.c_int32) for n in ("cached_blocks", "active", "pending")]


_SIGNATURES.update({
    "dk_sample_scratch_bytes": (C.c_int32, [C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]),
    "dk_sample_tokens": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(Sampling), C.c_uint64, C.c_void_p,
                                     C.c_size_t, C.c_void_p, C.c_void_p]),
    "dk_gemm_plan_query": (C.c_int32, [C.c_int32] * 6 + [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "dk_prefix_index_create": (C.c_int32, [C.c_int32, C.POINTER(C.c_void_p)]),
    "dk_prefix_index_destroy": (C.c_int32, [C.c_void_p, C.c_void_p]),
    "dk_prefix_index_match": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                          C.POINTER(C.c_int32)]),
    "dk_prefix_index_insert": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                           C.POINTER(C.c_int32)]),
    "dk_prefix_index_evict_lru": (C.c_int32, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]),
    "dk_prefix_index_size": (C.c_int32, [C.c_void_p, C.POINTER(C.c_int32)]),
    "dk_engine_device_bytes": (C.c_int32, [C.c_void_p, C.POINTER(EngineConfig), C.POINTER(C.c_size_t)]),
    "dk_engine_create": (C.c_int32, [C.c_void_p, C.c_void_p, C.POINTER(EngineConfig), C.c_void_p, C.c_size_t,
                                     C.POINTER(C.c_void_p)]),
    "dk_engine_destroy": (C.c_int32, [C.c_void_p]),
    "dk_engine_submit": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                     C.POINTER(C.c_int64)]),
    "dk_engine_step": (C.c_int32, [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]),
    "dk_engine_set_sampling": (C.c_int32, [C.c_void_p, C.POINTER(Sampling)]),
    "dk_engine_poll": (C.c_int32, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                   C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "dk_engine_forget": (C.c_int32, [C.c_void_p, C.c_int64]),
    "dk_engine_get_stats": (C.c_int32, [C.c_void_p, C.POINTER(EngineStats)]),
})

EXPORTS = tuple(_SIGNATURES)
REQUEST_STATES = ("pending", "active", "done", "failed")
_LIB = None


def lib():
    """The loaded library.  Raises if it has not been built: there is no
    fallback path."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise DecodeKitError(-6, f"{LIB_PATH} is missing; build it with "
                                     "`python -m paper_2601_19139_amd.build`")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = L
    return _LIB


def last_error() -> str:
    return lib().dk_last_error().decode()


def version() -> str:
    return lib().dk_version().decode()


def _check(code):
    if code != 0:
        raise DecodeKitError(code, last_error())


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


# ---- pool -----------------------------------------------------------------
def kv_pool_bytes(cfg: ModelConfig, num_blocks: int, block_size: int) -> int:
    out = C.c_size_t()
    _check(lib().dk_kv_pool_bytes(C.byref(cfg), num_blocks, block_size, C.byref(out)))
    return out.value


def create_kv_pool(cfg: ModelConfig, num_blocks: int, block_size: int, dev_mem, dev_bytes: int):
    out = C.c_void_p()
    _check(lib().dk_create_kv_pool(C.byref(cfg), num_blocks, block_size, _ptr(dev_mem), dev_bytes,
                                   C.byref(out)))
    return out


def destroy_kv_pool(pool):
    _check(lib().dk_destroy_kv_pool(pool))


def kv_alloc_block(pool) -> int:
    out = C.c_int32()
    _check(lib().dk_kv_alloc_block(pool, C.byref(out)))
    return out.value


def kv_alloc_block_id(pool, block_id: int):
    _check(lib().dk_kv_alloc_block_id(pool, block_id))


def kv_retain_block(pool, block_id: int):
    _check(lib().dk_kv_retain_block(pool, block_id))


def kv_release_block(pool, block_id: int):
    _check(lib().dk_kv_release_block(pool, block_id))


def kv_refcount(pool, block_id: int) -> int:
    out = C.c_int32()
    _check(lib().dk_kv_refcount(pool, block_id, C.byref(out)))
    return out.value


def kv_free_blocks(pool) -> int:
    out = C.c_int32()
    _check(lib().dk_kv_free_blocks(pool, C.byref(out)))
    return out.value


def kv_offset(pool, layer, block, kv, head, slot, dim) -> int:
    out = C.c_int64()
    _check(lib().dk_kv_offset(pool, layer, block, kv, head, slot, dim, C.byref(out)))
    return out.value


def kv_validate_tables(pool, h_block_tables, h_seq_lens):
    """h_block_tables: host int32 [B, max_blocks] (numpy); h_seq_lens: host int32 [B]."""
    B, mb = h_block_tables.shape
    _check(lib().dk_kv_validate_tables(pool, _ptr(h_block_tables), mb, _ptr(h_seq_lens), B))


def append_kv(pool, layer, d_block_tables, d_seq_lens, d_k, d_v, stream=None):
    B, mb = d_block_tables.shape
    _check(lib().dk_append_kv(pool, layer, _ptr(d_block_tables), mb, _ptr(d_seq_lens), B,
                              _ptr(d_k), _ptr(d_v), _stream(stream)))


# ---- model ----------------------------------------------------------------
def create_model(cfg: ModelConfig, weights: WeightPtrs):
    out = C.c_void_p()
    _check(lib().dk_create_model(C.byref(cfg), C.byref(weights), C.byref(out)))
    return out


def create_model_q4(cfg: ModelConfig, weights: WeightPtrs):
    out = C.c_void_p()
    _check(lib().dk_create_model_q4(C.byref(cfg), C.byref(weights), C.byref(out)))
    return out


def destroy_model(model):
    _check(lib().dk_destroy_model(model))


def read_stream(d_buf, d_sink, stream=None):
    """Enqueues the read-only streaming kernel over the whole of d_buf (measurement aid)."""
    _check(lib().dk_read_stream(_ptr(d_buf), d_buf.numel() * d_buf.element_size(), _ptr(d_sink), _stream(stream)))


def gemm_plan_query(epilogue: int, N: int, K: int, B: int, four_bit: bool = False, compute_units: int = 0):
    """(waves per block or 0, K slices, estimated microseconds) of the batched GEMM the step would launch."""
    w, s, us = C.c_int32(), C.c_int32(), C.c_double()
    _check(lib().dk_gemm_plan_query(epilogue, N, K, B, int(four_bit), compute_units, C.byref(w), C.byref(s), C.byref(us)))
    return w.value, s.value, us.value


def workspace_bytes(model, max_B: int, max_blocks_per_seq: int) -> int:
    out = C.c_size_t()
    _check(lib().dk_workspace_bytes(model, max_B, max_blocks_per_seq, C.byref(out)))
    return out.value


def decode_step(model, pool, d_block_tables, d_seq_lens, d_tokens, d_workspace, d_logits,
                d_next_tokens, flags: int = 0, stream=None, workspace_bytes_: int = None):
    B, mb = d_block_tables.shape
    nbytes = workspace_bytes_ if workspace_bytes_ is not None else d_workspace.numel() * d_workspace.element_size()
    _check(lib().dk_decode_step(model, pool, _ptr(d_block_tables), mb, _ptr(d_seq_lens),
                                _ptr(d_tokens), B, _ptr(d_workspace), nbytes, _ptr(d_logits),
                                _ptr(d_next_tokens), flags, _stream(stream)))


STATIC_SCRATCH_BYTES = 64 << 20


def decode_step_static(model, pool, d_block_tables, d_seq_lens, d_tokens, d_logits, d_next_tokens,
                       flags: int = 0, stream=None):
    """dk_decode_step with the library's own fixed device scratch (allocates nothing)."""
    B, mb = d_block_tables.shape
    _check(lib().dk_decode_step_static(model, pool, _ptr(d_block_tables), mb, _ptr(d_seq_lens), _ptr(d_tokens), B,
                                       _ptr(d_logits), _ptr(d_next_tokens), flags, _stream(stream)))


def prefill_chunk(model, pool, d_block_table, start: int, d_tokens, d_workspace, workspace_bytes_: int,
                  d_logits, d_next_tokens, stream=None):
    """One prefill chunk of one sequence: d_block_table int32 [max_blocks], d_tokens int32 [n]."""
    _check(lib().dk_prefill_chunk(model, pool, _ptr(d_block_table), int(d_block_table.numel()), int(start),
                                  _ptr(d_tokens), int(d_tokens.numel()), _ptr(d_workspace), workspace_bytes_,
                                  _ptr(d_logits), _ptr(d_next_tokens), _stream(stream)))


STAGE_STAMPS = 16


def debug_set_stage_stamps(model, layer: int, d_stamps):
    """d_stamps: an int64 device tensor [blocks][STAGE_STAMPS], or None to switch the stamps off."""
    if d_stamps is None:
        _check(lib().dk_debug_set_stage_stamps(model, 0, None, 0))
    else:
        _check(lib().dk_debug_set_stage_stamps(model, layer, _ptr(d_stamps), d_stamps.numel() * d_stamps.element_size()))


def debug_set_wait_limit(model, polls: int):
    _check(lib().dk_debug_set_wait_limit(model, polls))


def workspace_reset(model):
    _check(lib().dk_workspace_reset(model))


def fused_status(model, d_workspace, stream=None):
    """(serial of the last persistent step that gave up waiting or 0, waits that ran out so far)."""
    out = (C.c_uint32 * 2)()
    _check(lib().dk_fused_status(model, _ptr(d_workspace), out, _stream(stream)))
    return out[0], out[1]


def profile_read(model, reset=True):
    """Per kernel class: (milliseconds, launches) summed over the profiled steps."""
    n = len(KERNEL_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(lib().dk_profile_read(model, ms, cnt, int(reset)))
    return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}


def step_routing(model, d_workspace, B, max_blocks_per_seq, n_layers, top_k, stream=None):
    """Experts chosen in the last decode step: numpy int32 [n_layers, B, top_k]."""
    import numpy as np
    out = np.empty((n_layers, B, top_k), dtype=np.int32)
    _check(lib().dk_step_routing(model, _ptr(d_workspace), B, max_blocks_per_seq, _ptr(out), _stream(stream)))
    return out


def step_algorithmic_bytes(model, pool, h_block_tables, h_seq_lens, with_logits=True,
                           distinct_experts_per_layer=None) -> int:
    B, mb = h_block_tables.shape
    out = C.c_uint64()
    _check(lib().dk_step_algorithmic_bytes(model, pool, _ptr(h_block_tables), mb, _ptr(h_seq_lens), B,
                                           int(with_logits), _ptr(distinct_experts_per_layer),
                                           C.byref(out)))
    return out.value


def sample_scratch_bytes(B: int, V: int) -> int:
    out = C.c_size_t()
    _check(lib().dk_sample_scratch_bytes(B, V, C.byref(out)))
    return out.value


def sample_tokens(d_logits, temperature: float, top_k: int, top_p: float, seed: int, step: int, d_scratch,
                  d_out, stream=None):
    """d_logits float32 [B, V]; d_scratch at least sample_scratch_bytes(B, V) bytes, 256-byte
    aligned; d_out int32 [B]."""
    B, V = d_logits.shape
    prm = Sampling(temperature, top_k, top_p, seed)
    _check(lib().dk_sample_tokens(_ptr(d_logits), B, V, C.byref(prm), step, _ptr(d_scratch),
                                  d_scratch.numel() * d_scratch.element_size(), _ptr(d_out), _stream(stream)))


# ---- prefix index and engine (dk_engine.h) ------------------------------------

def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def prefix_index_create(block_size: int = 16):
    out = C.c_void_p()
    _check(lib().dk_prefix_index_create(block_size, C.byref(out)))
    return out


def prefix_index_destroy(index, pool=None):
    _check(lib().dk_prefix_index_destroy(index, pool))


def prefix_index_match(index, tokens, max_blocks: int):
    """Block ids of the longest cached chain of `tokens` (at most max_blocks blocks)."""
    t = _i32(tokens)
    out = np.empty(max(1, max_blocks), dtype=np.int32)
    n = C.c_int32()
    _check(lib().dk_prefix_index_match(index, _ptr(t), t.size, max_blocks, _ptr(out), C.byref(n)))
    return out[:n.value].copy()


def prefix_index_insert(index, pool, tokens, blocks) -> int:
    t, b = _i32(tokens), _i32(blocks)
    assert t.size >= 16 * b.size
    n = C.c_int32()
    _check(lib().dk_prefix_index_insert(index, pool, _ptr(t), b.size, _ptr(b), C.byref(n)))
    return n.value


def prefix_index_evict_lru(index, pool) -> int:
    out = C.c_int32()
    _check(lib().dk_prefix_index_evict_lru(index, pool, C.byref(out)))
    return out.value


def prefix_index_size(index) -> int:
    out = C.c_int32()
    _check(lib().dk_prefix_index_size(index, C.byref(out)))
    return out.value


def engine_device_bytes(model, cfg: EngineConfig) -> int:
    out = C.c_size_t()
    _check(lib().dk_engine_device_bytes(model, C.byref(cfg), C.byref(out)))
    return out.value


def engine_create(model, pool, cfg: EngineConfig, d_arena, arena_bytes: int):
    out = C.c_void_p()
    _check(lib().dk_engine_create(model, pool, C.byref(cfg), _ptr(d_arena), arena_bytes, C.byref(out)))
    return out


def engine_destroy(engine):
    _check(lib().dk_engine_destroy(engine))


def engine_submit(engine, prompt, max_new_tokens: int, eos_token: int = -1) -> int:
    p = _i32(prompt)
    out = C.c_int64()
    _check(lib().dk_engine_submit(engine, _ptr(p), p.size, max_new_tokens, eos_token, C.byref(out)))
    return out.value


def engine_step(engine, stream=None) -> int:
    """One iteration of the scheduler; returns the number of requests still active or pending."""
    out = C.c_int32()
    _check(lib().dk_engine_step(engine, _stream(stream), C.byref(out)))
    return out.value


def engine_set_sampling(engine, temperature: float = None, top_k: int = 0, top_p: float = 1.0, seed: int = 0):
    """Sample every token generated from now on (temperature None: back to greedy)."""
    if temperature is None:
        _check(lib().dk_engine_set_sampling(engine, None))
        return
    prm = Sampling(temperature, top_k, top_p, seed)
    _check(lib().dk_engine_set_sampling(engine, C.byref(prm)))


def engine_poll(engine, request_id: int, capacity: int = 4096):
    """(tokens generated so far, state name, prompt tokens supplied by the prefix cache)."""
    buf = np.empty(capacity, dtype=np.int32)
    n, st, reused = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().dk_engine_poll(engine, request_id, _ptr(buf), capacity, C.byref(n), C.byref(st), C.byref(reused)))
    return buf[:min(n.value, capacity)].copy(), REQUEST_STATES[st.value], reused.value


def engine_forget(engine, request_id: int):
    _check(lib().dk_engine_forget(engine, request_id))


def engine_stats(engine) -> dict:
    s = EngineStats()
    _check(lib().dk_engine_get_stats(engine, C.byref(s)))
    return {n: getattr(s, n) for n, _ in EngineStats._fields_}

