"""Device-memory plumbing around the C ABI: uploads seeded bf16 bit patterns
into torch tensors, keeps them alive, and hands their addresses to the library.
No arithmetic of the decode path happens here."""
import ctypes as C

import numpy as np

from . import binding as dk
from .q4 import pack_q4


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise dk.DecodeKitError(-6, "no HIP device: the decode path has no CPU fallback")
    return torch


def _dev_bf16(bits: np.ndarray):
    """uint16 bf16 bit patterns (host) -> device tensor of the same bits."""
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda()


class DeviceModel:
    """Weights resident in HBM + the library's model handle.  q, k and v
    matrices are stored as one [(nq+2nkv)*d, H] matrix (rows q, then k, then v).

    Matrices given as dicts (q / scale / bias: the canonical 4-bit form) make a
    4-bit model: every projection and the lm_head must then be in that form."""

    def __init__(self, shape, weights: dict):
        self.shape = shape
        self.cfg = dk.ModelConfig.from_shape(shape)
        self.tensors = []
        keep = self.tensors.append
        self.q4 = isinstance(weights["lm_head"], dict)

        packed = {}
        if self.q4:
            # pack on a few threads (numpy releases the interpreter lock): seconds instead of minutes at 8B
            from concurrent.futures import ThreadPoolExecutor
            def flat(m):   # a stack of expert matrices [E, N, K] is packed as one matrix of E*N rows
                if m["q"].ndim == 2:
                    return m
                e, n, k = m["q"].shape
                return {"q": m["q"].reshape(e * n, k), "scale": m["scale"].reshape(e * n, -1),
                        "bias": m["bias"].reshape(e * n, -1), "_of": m}

            jobs = [(weights["lm_head"],)]
            for L in weights["layers"]:
                jobs += [(L["wq"], L["wk"], L["wv"]), (L["wo"],), (flat(L["w_gate"]),), (flat(L["w_up"]),),
                         (flat(L["w_down"]),)]
            with ThreadPoolExecutor(max_workers=8) as ex:
                for j, buf in zip(jobs, ex.map(lambda j: pack_q4(*j), jobs)):
                    packed[id(j[0].get("_of", j[0]))] = buf

        def up(*a):
            if self.q4 and isinstance(a[0], dict):
                t = _torch().from_numpy(packed.pop(id(a[0]))).cuda()
            else:
                t = _dev_bf16(a[0] if len(a) == 1 else np.concatenate(a, axis=0))
            keep(t)
            return t.data_ptr()

        embed = up(weights["embed"])
        lm_head = embed if weights["lm_head"] is weights["embed"] else up(weights["lm_head"])
        g_final = up(weights["g_final"])
        self._layers = (dk.LayerWeights * shape.n_layers)()
        for i, L in enumerate(weights["layers"]):
            s = self._layers[i]
            s.g_attn = up(L["g_attn"])
            s.w_qkv = up(L["wq"], L["wk"], L["wv"])
            s.g_q = up(L["g_q"]) if "g_q" in L else None
            s.g_k = up(L["g_k"]) if "g_k" in L else None
            s.w_o = up(L["wo"])
            s.g_mlp = up(L["g_mlp"])
            s.w_gate = up(L["w_gate"])
            s.w_up = up(L["w_up"])
            s.w_down = up(L["w_down"])
            s.w_router = up(L["w_router"]) if "w_router" in L else None
        self._ptrs = dk.WeightPtrs(embed, lm_head, g_final, self._layers)
        self.handle = (dk.create_model_q4 if self.q4 else dk.create_model)(self.cfg, self._ptrs)

    def close(self):
        if self.handle is not None:
            dk.destroy_model(self.handle)
            self.handle = None


class DeviceKV:
    """A KV pool in HBM (torch-owned memory) + the library's pool handle, with
    block ownership mirrored from a block layout (ids, shared prefixes)."""

    def __init__(self, dmodel: DeviceModel, layout, pool_bits: np.ndarray = None):
        torch = _torch()
        self.layout = layout
        nbytes = dk.kv_pool_bytes(dmodel.cfg, layout.num_blocks, layout.block_size)
        if pool_bits is not None:
            assert pool_bits.nbytes == nbytes
            self.mem = _dev_bf16(pool_bits)
        else:
            self.mem = torch.zeros(nbytes // 2, dtype=torch.int16, device="cuda")
        self.handle = dk.create_kv_pool(dmodel.cfg, layout.num_blocks, layout.block_size,
                                        self.mem, nbytes)
        # take every block a table names; a block named by several tables is shared
        for b in range(layout.tables.shape[0]):
            for bid in layout.tables[b]:
                bid = int(bid)
                if bid < 0:
                    continue
                if dk.kv_refcount(self.handle, bid) == 0:
                    dk.kv_alloc_block_id(self.handle, bid)
                else:
                    dk.kv_retain_block(self.handle, bid)
        self.block_tables = torch.from_numpy(np.ascontiguousarray(layout.tables)).cuda()

    def bits(self) -> np.ndarray:
        return self.mem.cpu().numpy().view(np.uint16)

    def close(self):
        if self.handle is not None:
            dk.destroy_kv_pool(self.handle)
            self.handle = None


class Decoder:
    """Buffers for repeated decode steps of a fixed batch."""

    def __init__(self, dmodel: DeviceModel, dkv: DeviceKV, seq_lens, tokens, want_logits=True):
        torch = _torch()
        self.m, self.kv = dmodel, dkv
        B, mb = dkv.layout.tables.shape
        self.B = B
        self.seq_lens = torch.from_numpy(np.ascontiguousarray(seq_lens, dtype=np.int32)).cuda()
        self.tokens = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).cuda()
        self.next = torch.empty(B, dtype=torch.int32, device="cuda")
        self.logits = (torch.empty((B, dmodel.shape.vocab), dtype=torch.float32, device="cuda")
                       if want_logits else None)
        self.ws_bytes = dk.workspace_bytes(dmodel.handle, B, mb)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device="cuda")
        self._ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256

    def fused_status(self):
        """(serial of the last persistent step that gave up waiting, waits that ran out) or None
        when no persistent step has used this decoder's workspace."""
        try:
            return dk.fused_status(self.m.handle, self._ws_ptr)
        except dk.DecodeKitError:
            return None

    def routing(self):
        """Experts chosen in the last step, int32 [n_layers, B, top_k] (MoE models)."""
        shape = self.m.shape
        return dk.step_routing(self.m.handle, self._ws_ptr, self.B, self.kv.layout.tables.shape[1],
                               shape.n_layers, shape.top_k)

    def step(self, flags: int = 0, stream=None):
        dk.decode_step(self.m.handle, self.kv.handle, self.kv.block_tables, self.seq_lens,
                       self.tokens, self._ws_ptr, self.logits, self.next, flags, stream,
                       workspace_bytes_=self.ws_bytes)


class Prefiller:
    """Buffers for chunked prefill of single sequences (chunks of up to `max_chunk` tokens)."""

    def __init__(self, dmodel: DeviceModel, dkv: DeviceKV, max_chunk: int = 64, want_logits=True):
        torch = _torch()
        self.m, self.kv = dmodel, dkv
        self.max_chunk = max_chunk
        mb = dkv.layout.tables.shape[1]
        self.ws_bytes = dk.workspace_bytes(dmodel.handle, max_chunk, mb)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device="cuda")
        self._ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256
        self.next = torch.empty(max_chunk, dtype=torch.int32, device="cuda")
        self.logits = (torch.empty((max_chunk, dmodel.shape.vocab), dtype=torch.float32, device="cuda")
                       if want_logits else None)

    def prefill(self, row: int, start: int, tokens, chunk: int = None, last_only: bool = False):
        """Feeds `tokens` (host ints) of sequence `row` of the layout, whose first `start`
        positions are already cached.  Returns (next tokens [n], logits [n, V] or None) on the
        host; with last_only, only the last chunk's (the other chunks skip the lm_head)."""
        torch = _torch()
        chunk = chunk or self.max_chunk
        assert 1 <= chunk <= self.max_chunk
        table = self.kv.block_tables[row]
        toks = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).cuda()
        nxt, lg = [], []
        for o in range(0, len(tokens), chunk):
            part = toks[o:o + chunk]
            n = int(part.numel())
            if last_only and o + chunk < len(tokens):
                dk.prefill_chunk(self.m.handle, self.kv.handle, table, start + o, part, self._ws_ptr,
                                 self.ws_bytes, None, None)
                continue
            dk.prefill_chunk(self.m.handle, self.kv.handle, table, start + o, part, self._ws_ptr, self.ws_bytes,
                             self.logits, self.next)
            nxt.append(self.next[:n].cpu().numpy().copy())
            if self.logits is not None:
                lg.append(self.logits[:n].cpu().numpy().copy())
        return np.concatenate(nxt), (np.concatenate(lg) if lg else None)

