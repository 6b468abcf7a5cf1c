"""Whole-step pins for the CPU oracle.

* brute force: an independent fp64 formulation of the decoder in torch matrix
  ops over dense, contiguous per-sequence caches (no block table, complex-number
  rotary embedding, library softmax-attention) must agree with the oracle;
* a block table whose prefix blocks are shared equals a contiguous copied cache
  bit for bit (resuming from a cached prefix - the paper's Algorithm 2 - must
  equal having the prefix privately);
* permuting physical block ids changes nothing, bit for bit;
* a batch of B equals B independent batch-1 runs, bit for bit (requests of the
  continuous batch do not interact - the paper's Algorithm 1);
* a step changes exactly L*B*2*nkv*d pool elements, at the addressed slots.
"""
import numpy as np
import pytest
import torch

import workloads as W
from workloads.blocktable import layout_for, build_block_tables


def t64(bits):
    return torch.from_numpy(W.f32_from_bf16_bits(bits).astype(np.float64))


def bf16_round(x: torch.Tensor) -> torch.Tensor:
    return x.float().to(torch.bfloat16).double()


def torch_rms(x, g, eps):
    return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + eps) * g


def torch_rope(x, pos, theta):
    d = x.shape[-1]
    ang = pos * theta ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    z = torch.complex(x[..., : d // 2], x[..., d // 2:]) * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], -1)


class TorchDecoder:
    """Dense-cache fp64 decoder for one sequence (independent second formulation)."""

    def __init__(self, cfg, w, K0, V0):
        self.cfg, self.w = cfg, w
        self.K = [k.clone() for k in K0]          # per layer [nkv, T, d]
        self.V = [v.clone() for v in V0]

    def step(self, token):
        c, w = self.cfg, self.w
        pos = self.K[0].shape[1]
        x = t64(w["embed"][token])
        for l, L in enumerate(w["layers"]):
            h = torch_rms(x, t64(L["g_attn"]), c.rms_eps)
            q = (t64(L["wq"]) @ h).view(c.n_q_heads, c.head_dim)
            k = (t64(L["wk"]) @ h).view(c.n_kv_heads, c.head_dim)
            v = (t64(L["wv"]) @ h).view(c.n_kv_heads, c.head_dim)
            if c.qk_norm:
                q = torch_rms(q, t64(L["g_q"]), c.rms_eps)
                k = torch_rms(k, t64(L["g_k"]), c.rms_eps)
            q, k = torch_rope(q, pos, c.rope_theta), torch_rope(k, pos, c.rope_theta)
            self.K[l] = torch.cat([self.K[l], bf16_round(k)[:, None, :]], 1)
            self.V[l] = torch.cat([self.V[l], bf16_round(v)[:, None, :]], 1)
            Kq = self.K[l].repeat_interleave(c.group, 0)
            Vq = self.V[l].repeat_interleave(c.group, 0)
            o = torch.nn.functional.scaled_dot_product_attention(q[:, None, :], Kq, Vq)[:, 0, :]
            x = x + t64(L["wo"]) @ o.reshape(-1)
            h = torch_rms(x, t64(L["g_mlp"]), c.rms_eps)
            if c.n_experts:
                p = torch.softmax(t64(L["w_router"]) @ h, 0)
                top = torch.topk(p, c.top_k)
                wt = top.values / top.values.sum()
                y = torch.zeros_like(x)
                for e, a in zip(top.indices.tolist(), wt):
                    act = torch.nn.functional.silu(t64(L["w_gate"][e]) @ h) * (t64(L["w_up"][e]) @ h)
                    y = y + a * (t64(L["w_down"][e]) @ act)
            else:
                act = torch.nn.functional.silu(t64(L["w_gate"]) @ h) * (t64(L["w_up"]) @ h)
                y = t64(L["w_down"]) @ act
            x = x + y
        logits = t64(w["lm_head"]) @ torch_rms(x, t64(w["g_final"]), c.rms_eps)
        return logits.numpy()


def dense_history(cfg, pool, lay, b):
    T, bs = int(lay.contexts[b]), lay.block_size
    K, V = [], []
    for l in range(cfg.n_layers):
        K.append(torch.stack([t64(pool[l, lay.tables[b, t // bs], 0, :, t % bs, :]) for t in range(T)], 1))
        V.append(torch.stack([t64(pool[l, lay.tables[b, t // bs], 1, :, t % bs, :]) for t in range(T)], 1))
    return K, V


def run_oracle(orc, cfg, w, pool, lay, tokens, steps, teacher=None):
    pool = pool.copy()
    sl = lay.contexts.copy()
    tok = np.asarray(tokens, dtype=np.int32).copy()
    outs = []
    for s in range(steps):
        r = orc.decode_step(cfg, w, pool, lay.block_size, lay.tables, sl, tok)
        outs.append(r)
        tok = r["next"] if teacher is None else teacher[s]
        sl = sl + 1
    return outs, pool


@pytest.mark.parametrize("wname", ["cfg0", "cfg0_moe"])
def test_brute_force_tiny(orc, wname):
    wl = W.WORKLOADS[wname]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, wl.seed_weights)
    pool = W.fill_kv_pool(cfg, lay, wl.seed_kv)           # dead slots are NaN: any over-read shows
    tokens = W.initial_tokens(cfg, wl.batch, wl.seed_tokens)
    outs, _ = run_oracle(orc, cfg, w, pool, lay, tokens, wl.steps)
    for b in range(wl.batch):
        dec = TorchDecoder(cfg, w, *dense_history(cfg, pool, lay, b))
        tok = int(tokens[b])
        for s in range(wl.steps):
            ref = dec.step(tok)
            got = outs[s]["logits"][b].astype(np.float64)
            rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
            assert rel < 1e-6, (wname, b, s, rel)          # float32 rounding of stored logits only
            assert int(outs[s]["next"][b]) == int(np.argmax(ref.astype(np.float32)))
            tok = int(outs[s]["next"][b])


def test_qk_norm_variant_brute_force(orc):
    base = W.CONFIGS["tiny"]
    cfg = W.ModelConfig(**{**base.as_dict(), "qk_norm": True, "rope_theta": 1e6, "n_q_heads": 6})
    lay = build_block_tables([19, 40, 1], 16, 3, seed=9)
    w = W.make_weights(cfg, 4)
    pool = W.fill_kv_pool(cfg, lay, 5)
    tokens = W.initial_tokens(cfg, 3, 6)
    outs, _ = run_oracle(orc, cfg, w, pool, lay, tokens, 3)
    for b in range(3):
        dec = TorchDecoder(cfg, w, *dense_history(cfg, pool, lay, b))
        tok = int(tokens[b])
        for s in range(3):
            ref = dec.step(tok)
            got = outs[s]["logits"][b].astype(np.float64)
            assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-6
            tok = int(outs[s]["next"][b])


def test_f32_build_agrees_with_f64(orc, orc32):
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    pool = W.fill_kv_pool(cfg, lay, 1)
    tokens = W.initial_tokens(cfg, wl.batch, 2)
    a, _ = run_oracle(orc, cfg, w, pool, lay, tokens, 4)
    teacher = [o["next"] for o in a]
    b, _ = run_oracle(orc32, cfg, w, pool, lay, tokens, 4, teacher=teacher)
    for x, y in zip(a, b):
        num = np.linalg.norm(x["logits"].astype(np.float64) - y["logits"], axis=1)
        assert np.all(num / np.linalg.norm(x["logits"], axis=1) < 2e-5)


def test_shared_prefix_equals_private_copy_bitwise(orc):
    cfg = W.CONFIGS["tiny"]
    bs, steps = 16, 3
    ctx = [50, 37, 33, 20]
    shared = build_block_tables(ctx, bs, steps, shared_prefix=32, n_sharers=3, seed=21)
    assert shared.refcount.max() == 3
    w = W.make_weights(cfg, 0)
    pool_s = W.fill_kv_pool(cfg, shared, 1)
    # private layout: same logical contents, every sequence owns all its blocks
    private = build_block_tables(ctx, bs, steps, seed=22)
    pool_p = np.full(W.pool_shape(cfg, private.num_blocks, bs), W.BF16_NAN_BITS, dtype=np.uint16)
    for b, T in enumerate(ctx):
        for t in range(T):
            pool_p[:, private.tables[b, t // bs], :, :, t % bs, :] = \
                pool_s[:, shared.tables[b, t // bs], :, :, t % bs, :]
    tokens = W.initial_tokens(cfg, 4, 2)
    a, _ = run_oracle(orc, cfg, w, pool_s, shared, tokens, steps)
    b_, _ = run_oracle(orc, cfg, w, pool_p, private, tokens, steps)
    for x, y in zip(a, b_):
        assert np.array_equal(x["logits"], y["logits"]) and np.array_equal(x["next"], y["next"])


def test_block_permutation_is_invisible_bitwise(orc):
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    pool = W.fill_kv_pool(cfg, lay, 1)
    perm = np.random.default_rng(3).permutation(lay.num_blocks).astype(np.int32)   # old id -> new id
    pool2 = np.empty_like(pool)
    pool2[:, perm] = pool
    lay2 = build_block_tables(lay.contexts, lay.block_size, wl.steps)
    lay2.tables = np.where(lay.tables >= 0, perm[np.maximum(lay.tables, 0)], -1).astype(np.int32)
    lay2.num_blocks = lay.num_blocks
    tokens = W.initial_tokens(cfg, wl.batch, 2)
    a, pa = run_oracle(orc, cfg, w, pool, lay, tokens, wl.steps)
    b, pb = run_oracle(orc, cfg, w, pool2, lay2, tokens, wl.steps)
    for x, y in zip(a, b):
        assert np.array_equal(x["logits"], y["logits"])
    assert np.array_equal(pb[:, perm].view(np.uint16), pa.view(np.uint16))


def test_batch_equals_independent_runs_bitwise(orc):
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    pool = W.fill_kv_pool(cfg, lay, 1)
    tokens = W.initial_tokens(cfg, wl.batch, 2)
    both, _ = run_oracle(orc, cfg, w, pool, lay, tokens, 4)
    for b in range(wl.batch):
        p = pool.copy()
        sl = lay.contexts[b:b + 1].copy()
        tok = tokens[b:b + 1].copy()
        for s in range(4):
            r = orc.decode_step(cfg, w, p, lay.block_size, lay.tables[b:b + 1], sl, tok)
            assert np.array_equal(r["logits"][0], both[s]["logits"][b])
            tok, sl = r["next"], sl + 1


def test_step_changes_exactly_the_appended_slots(orc):
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    pool = W.fill_kv_pool(cfg, lay, 1)           # target slots hold NaN bits beforehand
    before = pool.copy()
    tokens = W.initial_tokens(cfg, wl.batch, 2)
    orc.decode_step(cfg, w, pool, lay.block_size, lay.tables, lay.contexts, tokens)
    changed = np.argwhere(pool != before)
    assert len(changed) == cfg.n_layers * wl.batch * 2 * cfg.kv_dim
    want_slots = {(int(lay.tables[b, T // 16]), int(T % 16)) for b, T in enumerate(lay.contexts)}
    assert {(int(r[1]), int(r[4])) for r in changed} == want_slots
    # seq 0 has 32 cached tokens: its append lands in slot 0 of its third block
    assert (int(lay.tables[0, 2]), 0) in want_slots


def test_rejects_bad_arguments(orc):
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    pool = W.fill_kv_pool(cfg, lay, 1)
    with pytest.raises(ValueError):
        orc.decode_step(cfg, w, pool, 16, lay.tables, lay.contexts, np.array([0, cfg.vocab]))
    bad = lay.tables.copy()
    bad[1, 1] = 99
    with pytest.raises(ValueError):
        orc.decode_step(cfg, w, pool, 16, bad, lay.contexts, np.array([0, 1]))


def test_oracle_reproduces_stored_fixture(orc):
    """Drift detector: tests/golden/cfg0_oracle.json was written by
    tests/golden/make_golden.py from the oracle alone."""
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg0_oracle.json")
    gold = json.load(open(path))
    wl = W.WORKLOADS["cfg0"]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, wl.seed_weights)
    pool = W.fill_kv_pool(cfg, lay, wl.seed_kv)
    tokens = W.initial_tokens(cfg, wl.batch, wl.seed_tokens)
    outs, _ = run_oracle(orc, cfg, w, pool, lay, tokens, wl.steps)
    for o, g in zip(outs, gold["steps"]):
        assert [int(t) for t in o["next"]] == g["next"]
        assert np.allclose(o["logits"][:, :8], np.array(g["logits_0_8"]), rtol=1e-6, atol=1e-7)
