"""ctypes front end of decode_oracle.c (argument marshalling only)."""
import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decode_oracle.c")
# ORACLE_SANITIZE=1 selects a build under AddressSanitizer and UndefinedBehaviorSanitizer (kept in a
# folder of its own; the process must then start with gcc's libasan preloaded - the tests do that)
_SANITIZE = os.environ.get("ORACLE_SANITIZE") == "1"
_BUILD = os.path.join(_HERE, "_build", "san") if _SANITIZE else os.path.join(_HERE, "_build")
_LOCK = threading.Lock()


def _lib_path(real: str) -> str:
    return os.path.join(_BUILD, f"liboracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile both builds of the oracle: arithmetic in double (the reference
    for every parity test) and in float (single precision; kept to show the
    two agree)."""
    os.makedirs(_BUILD, exist_ok=True)
    for real, flag in (("f64", []), ("f32", ["-DORC_REAL_FLOAT"])):
        out = _lib_path(real)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= os.path.getmtime(_SRC)):
            continue
        tmp = out + f".tmp{os.getpid()}"
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-fno-fast-math", "-ffp-contract=off", *flag, _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, out)


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
        "qk_norm", "n_experts", "top_k", "expert_ffn")] + [
        ("rms_eps", C.c_double), ("rope_theta", C.c_double)]


_LAYER_FIELDS = ("g_attn", "wq", "wk", "wv", "g_q", "g_k", "wo", "g_mlp",
                 "w_gate", "w_up", "w_down", "w_router")


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Oracle:
    """One compiled build of the oracle ('f64' or 'f32' arithmetic)."""

    def __init__(self, real: str = "f64"):
        with _LOCK:
            build()
        self.real = real
        self.lib = C.CDLL(_lib_path(real))
        L = self.lib
        L.orc_pool_offset.restype = C.c_int64
        L.orc_pool_offset.argtypes = [C.c_void_p] + [C.c_int32] * 8
        L.orc_argmax_f32.restype = C.c_int32
        L.orc_silu.restype = C.c_double
        L.orc_silu.argtypes = [C.c_double]
        L.orc_decode_step.restype = C.c_int
        assert L.orc_real_bytes() == (8 if real == "f64" else 4)

    # -- config / weights -------------------------------------------------
    @staticmethod
    def config(cfg) -> _Config:
        return _Config(cfg.n_layers, cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                       cfg.ffn, cfg.vocab, int(cfg.qk_norm), cfg.n_experts, cfg.top_k,
                       cfg.expert_ffn, cfg.rms_eps, cfg.rope_theta)

    @staticmethod
    def layer_struct(layer: dict) -> _Layer:
        s = _Layer()
        keep = []
        for n in _LAYER_FIELDS:
            a = layer.get(n)
            if a is not None:
                a = _u16(a)
                keep.append(a)
                setattr(s, n, a.ctypes.data)
        s._keep = keep
        return s

    # -- stages -----------------------------------------------------------
    def bf16_to_f32(self, bits):
        bits = _u16(bits)
        out = np.empty(bits.shape, dtype=np.float32)
        self.lib.orc_bf16_to_f32(_p(bits), C.c_int64(bits.size), _p(out))
        return out

    def f32_to_bf16(self, x):
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.empty(x.shape, dtype=np.uint16)
        self.lib.orc_f32_to_bf16(_p(x), C.c_int64(x.size), _p(out))
        return out

    def rmsnorm(self, x, gain_bits, eps):
        x = _f64(x)
        out = np.empty_like(x)
        self.lib.orc_rmsnorm(_p(x), C.c_int32(x.size), _p(_u16(gain_bits)), C.c_double(eps), _p(out))
        return out

    def matvec(self, W_bits, x):
        W_bits = _u16(W_bits)
        x = _f64(x)
        rows, cols = W_bits.shape
        assert x.shape == (cols,)
        y = np.empty(rows, dtype=np.float64)
        self.lib.orc_matvec(_p(W_bits), C.c_int64(rows), C.c_int64(cols), _p(x), _p(y))
        return y

    def matvec_q4(self, m: dict, x):
        """y = W x for a 4-bit matrix in canonical form (dict q / scale / bias)."""
        q = np.ascontiguousarray(m["q"], dtype=np.uint8)
        rows, cols = q.shape
        sc, bi = _u16(m["scale"]), _u16(m["bias"])
        assert sc.shape == bi.shape == (rows, cols // 64) and cols % 64 == 0
        x = _f64(x)
        assert x.shape == (cols,)
        y = np.empty(rows, dtype=np.float64)
        self.lib.orc_matvec_q4(_p(q), _p(sc), _p(bi), C.c_int64(rows), C.c_int64(cols), _p(x), _p(y))
        return y

    def rope(self, v, pos, theta):
        v = _f64(v).copy()
        self.lib.orc_rope(_p(v), C.c_int32(v.size), C.c_int32(pos), C.c_double(theta))
        return v

    def softmax(self, s):
        s = _f64(s)
        p = np.empty_like(s)
        self.lib.orc_softmax(_p(s), C.c_int32(s.size), _p(p))
        return p

    def silu(self, z):
        return self.lib.orc_silu(float(z))

    def pool_offset(self, cfg, num_blocks, block_size, layer, block, kv, head, slot, dim):
        c = self.config(cfg)
        return self.lib.orc_pool_offset(C.addressof(c), num_blocks, block_size, layer, block,
                                        kv, head, slot, dim)

    def append_kv(self, cfg, pool, block_size, layer, table_row, pos, k, v):
        c = self.config(cfg)
        assert pool.dtype == np.uint16 and pool.flags.c_contiguous
        t = _i32(table_row)
        self.lib.orc_append_kv(C.byref(c), _p(pool), C.c_int32(pool.shape[1]), C.c_int32(block_size),
                               C.c_int32(layer), _p(t), C.c_int32(pos), _p(_f64(k)), _p(_f64(v)))

    def attention(self, cfg, pool, block_size, layer, table_row, n_tokens, q, want_probs=False):
        c = self.config(cfg)
        assert pool.dtype == np.uint16 and pool.flags.c_contiguous
        t = _i32(table_row)
        q = _f64(q).reshape(-1)
        out = np.empty(cfg.n_q_heads * cfg.head_dim, dtype=np.float64)
        probs = np.empty((cfg.n_q_heads, n_tokens), dtype=np.float64) if want_probs else None
        self.lib.orc_attention(C.byref(c), _p(pool), C.c_int32(pool.shape[1]), C.c_int32(block_size),
                               C.c_int32(layer), _p(t), C.c_int32(n_tokens), _p(q), _p(out), _p(probs))
        out = out.reshape(cfg.n_q_heads, cfg.head_dim)
        return (out, probs) if want_probs else out

    def swiglu(self, wg, wu, wd, h):
        wg, wu, wd = _u16(wg), _u16(wu), _u16(wd)
        F, H = wg.shape
        h = _f64(h)
        out = np.empty(H, dtype=np.float64)
        self.lib.orc_swiglu(_p(wg), _p(wu), _p(wd), C.c_int32(H), C.c_int32(F), _p(h), _p(out))
        return out

    def moe(self, cfg, layer: dict, h):
        c = self.config(cfg)
        ls = self.layer_struct(layer)
        h = _f64(h)
        out = np.empty(cfg.hidden, dtype=np.float64)
        idx = np.empty(cfg.top_k, dtype=np.int32)
        wts = np.empty(cfg.top_k, dtype=np.float64)
        self.lib.orc_moe(C.byref(c), C.byref(ls), _p(h), _p(out), _p(idx), _p(wts))
        return out, idx, wts

    def argmax(self, v):
        v = np.ascontiguousarray(v, dtype=np.float32)
        return int(self.lib.orc_argmax_f32(_p(v), C.c_int32(v.size)))

    # -- sampling ---------------------------------------------------------
    def sample(self, logits, temperature, top_k, top_p, u):
        v = np.ascontiguousarray(logits, dtype=np.float32)
        self.lib.orc_sample.restype = C.c_int32
        return int(self.lib.orc_sample(_p(v), C.c_int32(v.size), C.c_double(temperature), C.c_int32(top_k),
                                       C.c_double(top_p), C.c_double(u)))

    def philox4x32_10(self, counter, key):
        c = (C.c_uint32 * 4)(*[int(x) for x in counter])
        k = (C.c_uint32 * 2)(*[int(x) for x in key])
        out = (C.c_uint32 * 4)()
        self.lib.orc_philox4x32_10(c, k, out)
        return tuple(int(x) for x in out)

    def sample_uniform(self, seed, step, row):
        self.lib.orc_sample_uniform.restype = C.c_double
        return float(self.lib.orc_sample_uniform(C.c_uint64(seed), C.c_uint64(step), C.c_uint32(row)))

    # -- whole step -------------------------------------------------------
    def route(self, cfg, w_router_bits, h, proposal=None, tie_tol=0.0):
        """The router alone: (experts int32 [k], weights [k], adopted, margin)."""
        c = self.config(cfg)
        h = _f64(h)
        idx = np.empty(cfg.top_k, dtype=np.int32)
        wts = np.empty(cfg.top_k, dtype=np.float64)
        adopted = C.c_int32(0)
        margin = C.c_double(0.0)
        prop = None if proposal is None else _i32(proposal)
        self.lib.orc_route.restype = None
        self.lib.orc_route(C.byref(c), _p(_u16(w_router_bits)), _p(h), _p(idx), _p(wts), _p(prop),
                           C.c_double(tie_tol), C.byref(adopted), C.byref(margin))
        return idx, wts, bool(adopted.value), margin.value

    def decode_step_tie(self, cfg, weights, pool, block_size, block_tables, seq_lens, tokens, proposal, tie_tol):
        """decode_step of a mixture-of-experts model (bf16 weights) with expert sets proposed for
        the router's near-ties: proposal int32 [L, B, top_k]; adopted only where it is a valid
        top-k set up to tie_tol (see decode_oracle.c).  Adds 'adopted' int32 [L, B] and 'margin'
        float64 [L, B] to the result."""
        c = self.config(cfg)
        assert pool.dtype == np.uint16 and pool.flags.c_contiguous and cfg.n_experts
        L = cfg.n_layers
        structs = (_Layer * L)()
        keep = []
        for i, lay in enumerate(weights["layers"]):
            s = self.layer_struct(lay)
            keep.append(s)
            structs[i] = s
        bt, sl, tk = _i32(block_tables), _i32(seq_lens), _i32(tokens)
        B = tk.size
        prop = _i32(proposal)
        assert prop.shape == (L, B, cfg.top_k)
        logits = np.empty((B, cfg.vocab), dtype=np.float32)
        nxt = np.empty(B, dtype=np.int32)
        experts = np.empty((L, B, cfg.top_k), dtype=np.int32)
        adopted = np.zeros((L, B), dtype=np.int32)
        margin = np.zeros((L, B), dtype=np.float64)
        self.lib.orc_decode_step_tie.restype = C.c_int
        rc = self.lib.orc_decode_step_tie(
            C.byref(c), structs, _p(_u16(weights["embed"])), _p(_u16(weights["g_final"])),
            _p(_u16(weights["lm_head"])), _p(pool), C.c_int32(pool.shape[1]), C.c_int32(block_size),
            _p(bt), C.c_int32(bt.shape[1]), _p(sl), _p(tk), C.c_int32(B),
            _p(logits), _p(nxt), _p(experts), _p(prop), C.c_double(tie_tol), _p(adopted), _p(margin))
        if rc != 0:
            raise ValueError(f"orc_decode_step_tie rejected its arguments (code {rc})")
        return {"next": nxt, "logits": logits, "experts": experts, "adopted": adopted, "margin": margin}

    def decode_step(self, cfg, weights, pool, block_size, block_tables, seq_lens, tokens,
                    want_logits=True, want_trace=False):
        """One decode step for every row of the batch.  `pool` (uint16,
        [L, NB, 2, nkv, bs, d]) is updated in place.  Returns a dict with
        'next' int32 [B], 'logits' float32 [B, V] (optional), 'trace_x',
        'experts' (optional)."""
        c = self.config(cfg)
        assert pool.dtype == np.uint16 and pool.flags.c_contiguous
        L = cfg.n_layers
        structs = (_Layer * L)()
        keep = []
        for i, lay in enumerate(weights["layers"]):
            s = self.layer_struct(lay)
            keep.append(s)
            structs[i] = s
        bt = _i32(block_tables)
        sl = _i32(seq_lens)
        tk = _i32(tokens)
        B = tk.size
        assert bt.shape[0] == B and sl.size == B
        logits = np.empty((B, cfg.vocab), dtype=np.float32) if want_logits else None
        nxt = np.empty(B, dtype=np.int32)
        trace = np.empty((L + 1, B, cfg.hidden), dtype=np.float32) if want_trace else None
        experts = (np.empty((L, B, cfg.top_k), dtype=np.int32)
                   if (want_trace and cfg.n_experts) else None)
        rc = self.lib.orc_decode_step(
            C.byref(c), structs, _p(_u16(weights["embed"])), _p(_u16(weights["g_final"])),
            _p(_u16(weights["lm_head"])), _p(pool), C.c_int32(pool.shape[1]), C.c_int32(block_size),
            _p(bt), C.c_int32(bt.shape[1]), _p(sl), _p(tk), C.c_int32(B),
            _p(logits), _p(nxt), _p(trace), _p(experts))
        if rc != 0:
            raise ValueError(f"orc_decode_step rejected its arguments (code {rc})")
        return {"next": nxt, "logits": logits, "trace_x": trace, "experts": experts}


    def decode_step_q4(self, cfg, qweights, pool, block_size, block_tables, seq_lens, tokens,
                       want_logits=True, want_trace=False):
        """decode_step for a model whose projections and lm_head are 4-bit (canonical
        dicts q / scale / bias in place of the bf16 matrices; expert matrices [E, N, K]
        as q [E, N, K], scale / bias [E, N, K/64]; the router stays bf16)."""
        c = self.config(cfg)
        assert pool.dtype == np.uint16 and pool.flags.c_contiguous
        L = cfg.n_layers
        names = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
        structs = (_Layer * L)()
        keep, mats = [], []
        for i, lay in enumerate(qweights["layers"]):
            s = self.layer_struct({k: v for k, v in lay.items() if k not in names})
            keep.append(s)
            structs[i] = s
            mats += [lay[n] for n in names]
        mats.append(qweights["lm_head"])
        n = len(mats)
        experts = (np.empty((L, len(tokens), cfg.top_k), dtype=np.int32)
                   if (want_trace and cfg.n_experts) else None)
        qs = [np.ascontiguousarray(m["q"], dtype=np.uint8) for m in mats]
        ss = [_u16(m["scale"]) for m in mats]
        bs = [_u16(m["bias"]) for m in mats]
        qp = (C.c_void_p * n)(*[a.ctypes.data for a in qs])
        sp = (C.c_void_p * n)(*[a.ctypes.data for a in ss])
        bp = (C.c_void_p * n)(*[a.ctypes.data for a in bs])
        bt = _i32(block_tables)
        sl = _i32(seq_lens)
        tk = _i32(tokens)
        B = tk.size
        assert bt.shape[0] == B and sl.size == B
        logits = np.empty((B, cfg.vocab), dtype=np.float32) if want_logits else None
        nxt = np.empty(B, dtype=np.int32)
        trace = np.empty((L + 1, B, cfg.hidden), dtype=np.float32) if want_trace else None
        self.lib.orc_decode_step_q4.restype = C.c_int
        rc = self.lib.orc_decode_step_q4(
            C.byref(c), structs, qp, sp, bp, _p(_u16(qweights["embed"])), _p(_u16(qweights["g_final"])),
            _p(pool), C.c_int32(pool.shape[1]), C.c_int32(block_size),
            _p(bt), C.c_int32(bt.shape[1]), _p(sl), _p(tk), C.c_int32(B),
            _p(logits), _p(nxt), _p(trace), _p(experts))
        if rc != 0:
            raise ValueError(f"orc_decode_step_q4 rejected its arguments (code {rc})")
        return {"next": nxt, "logits": logits, "trace_x": trace, "experts": experts}


_CACHE = {}


def oracle_f64() -> Oracle:
    if "f64" not in _CACHE:
        _CACHE["f64"] = Oracle("f64")
    return _CACHE["f64"]


def oracle_f32() -> Oracle:
    if "f32" not in _CACHE:
        _CACHE["f32"] = Oracle("f32")
    return _CACHE["f32"]
