"""Pins for the 4-bit (group-wise affine) weight path of the CPU oracle.

The 4-bit format is the one of the quantised checkpoints the paper benchmarks
(evaluation setup: 4-bit models): groups of 64 columns, w = scale * q + bias.

* the matrix-vector product equals a library matmul over a matrix dequantised
  here, independently, in numpy;
* closed forms: scale 1 / bias 0 gives the integer dot product of the codes;
  scale 0 leaves bias * (sum of x over the group);
* a wrong group length, a transposed scale table or swapped scale / bias fail
  the closed forms above (each group gets its own scale and bias values);
* the whole step: a 4-bit model whose dequantised weights are exactly bf16
  numbers must give, bit for bit, what the (separately pinned) bf16 step gives
  for those bf16 weights - this fixes which 4-bit matrix feeds which
  projection, the matrix shapes and the lm_head;
* the quantiser used to prepare inputs reproduces its input within half a
  quantisation step.
"""
import numpy as np
import pytest

import workloads as W
from workloads.blocktable import layout_for, build_block_tables
from workloads.quant import quantize_q4, quantize_weights, MATRICES


def deq(m):
    s = W.f32_from_bf16_bits(m["scale"]).astype(np.float64)
    b = W.f32_from_bf16_bits(m["bias"]).astype(np.float64)
    return np.repeat(s, 64, axis=1) * m["q"].astype(np.float64) + np.repeat(b, 64, axis=1)


def random_q4(rng, n, k):
    """A canonical 4-bit matrix with distinct scale / bias per group."""
    q = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    scale = W.bf16_bits_from_f32(rng.uniform(0.001, 0.02, size=(n, k // 64)).astype(np.float32))
    bias = W.bf16_bits_from_f32(rng.uniform(-0.2, 0.0, size=(n, k // 64)).astype(np.float32))
    return {"q": q, "scale": scale, "bias": bias}


@pytest.mark.parametrize("n,k", [(1, 64), (37, 192), (130, 1024)])
def test_matvec_q4_equals_dense_matmul(orc, n, k):
    rng = np.random.default_rng(n * 1000 + k)
    m = random_q4(rng, n, k)
    x = rng.standard_normal(k)
    got = orc.matvec_q4(m, x)
    ref = deq(m) @ x
    assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(deq(m)).sum(axis=1).max() * np.abs(x).max())


def test_matvec_q4_closed_forms(orc):
    rng = np.random.default_rng(5)
    n, k = 9, 256
    q = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
    x = rng.integers(-4, 5, size=k).astype(np.float64)
    one = W.bf16_bits_from_f32(np.ones((n, k // 64), np.float32))
    zero = np.zeros((n, k // 64), np.uint16)
    # scale 1, bias 0: integer dot product, exact
    got = orc.matvec_q4({"q": q, "scale": one, "bias": zero}, x)
    assert np.array_equal(got, (q.astype(np.int64) @ x.astype(np.int64)).astype(np.float64))
    # scale 0: bias times the group sums of x; a different power of two per (row, group)
    e = rng.integers(-6, 3, size=(n, k // 64))
    bias = W.bf16_bits_from_f32((2.0 ** e).astype(np.float32))
    got = orc.matvec_q4({"q": q, "scale": zero, "bias": bias}, x)
    ref = ((2.0 ** e) * x.reshape(k // 64, 64).sum(axis=1)[None, :]).sum(axis=1)
    assert np.array_equal(got, ref)
    # a different power-of-two scale per (row, group), bias 0
    scale = W.bf16_bits_from_f32((2.0 ** e).astype(np.float32))
    got = orc.matvec_q4({"q": q, "scale": scale, "bias": zero}, x)
    part = (q.astype(np.int64).reshape(n, k // 64, 64) * x.astype(np.int64).reshape(1, k // 64, 64)).sum(axis=2)
    assert np.array_equal(got, ((2.0 ** e) * part).sum(axis=1))


def exact_q4_model(cfg, seed):
    """bf16 weights whose every projection is exactly representable in the 4-bit format, and
    that 4-bit form: w = 2^-e * (q - 8) with one exponent per group (scale 2^-e, bias -8 * 2^-e)."""
    rng = np.random.default_rng(seed)
    w = W.make_weights(cfg, seed)
    qw = {"embed": w["embed"], "g_final": w["g_final"], "layers": []}

    def make(shape):
        if len(shape) == 3:                      # a stack of expert matrices: row by row like one matrix
            e, n, k = shape
            bits, m = make((e * n, k))
            return bits.reshape(shape), {"q": m["q"].reshape(shape), "scale": m["scale"].reshape(e, n, k // 64),
                                         "bias": m["bias"].reshape(e, n, k // 64)}
        n, k = shape
        q = rng.integers(0, 16, size=(n, k), dtype=np.uint8)
        e = rng.integers(5, 8, size=(n, k // 64))
        s = (2.0 ** -e).astype(np.float32)
        dense = (np.repeat(s, 64, axis=1) * (q.astype(np.float32) - 8.0)).astype(np.float32)
        bits = W.bf16_bits_from_f32(dense)
        assert np.array_equal(W.f32_from_bf16_bits(bits), dense)          # exactly bf16
        return bits, {"q": q, "scale": W.bf16_bits_from_f32(s), "bias": W.bf16_bits_from_f32(-8.0 * s)}

    for L in w["layers"]:
        ql = dict(L)
        for name in MATRICES:
            L[name], ql[name] = make(L[name].shape)
        qw["layers"].append(ql)
    w["lm_head"], qw["lm_head"] = make(w["lm_head"].shape)
    return w, qw


def test_q4_step_equals_bf16_step_on_exactly_representable_weights(orc):
    wl = W.WORKLOADS["cfg0_q4"]
    cfg, lay = wl.cfg, layout_for(wl)
    w, qw = exact_q4_model(cfg, 11)
    pool_a = W.fill_kv_pool(cfg, lay, wl.seed_kv)
    pool_b = pool_a.copy()
    tok = W.initial_tokens(cfg, wl.batch, wl.seed_tokens)
    sl = lay.contexts.copy()
    for s in range(3):
        a = orc.decode_step(cfg, w, pool_a, lay.block_size, lay.tables, sl, tok, want_trace=True)
        b = orc.decode_step_q4(cfg, qw, pool_b, lay.block_size, lay.tables, sl, tok, want_trace=True)
        assert np.array_equal(a["logits"], b["logits"])
        assert np.array_equal(a["trace_x"], b["trace_x"])
        assert np.array_equal(a["next"], b["next"])
        assert np.array_equal(pool_a.view(np.uint16), pool_b.view(np.uint16))
        tok, sl = a["next"], sl + 1


def test_q4_moe_step_equals_bf16_step_on_exactly_representable_weights(orc):
    """Mixture of experts: the 4-bit gate / up / down stacks [E, N, K] feed the expert the (bf16) router
    chose; same experts, same logits, bit for bit, as the bf16 step on the same numbers."""
    cfg = W.ModelConfig(**{**W.CONFIGS["tiny_moe"].as_dict(), "expert_ffn": 128})
    lay = build_block_tables([33, 16, 5], 16, 3, seed=2)
    w, qw = exact_q4_model(cfg, 13)
    for L, QL in zip(w["layers"], qw["layers"]):
        assert L["w_gate"].shape == (cfg.n_experts, 128, cfg.hidden) and QL["w_router"] is L["w_router"]
    pool_a = W.fill_kv_pool(cfg, lay, 1)
    pool_b = pool_a.copy()
    tok = W.initial_tokens(cfg, 3, 2)
    sl = lay.contexts.copy()
    for s in range(3):
        a = orc.decode_step(cfg, w, pool_a, 16, lay.tables, sl, tok, want_trace=True)
        b = orc.decode_step_q4(cfg, qw, pool_b, 16, lay.tables, sl, tok, want_trace=True)
        assert np.array_equal(a["experts"], b["experts"])
        assert np.array_equal(a["logits"], b["logits"])
        assert np.array_equal(a["trace_x"], b["trace_x"])
        assert np.array_equal(pool_a, pool_b)
        tok, sl = a["next"], sl + 1


def test_q4_step_rejects_what_it_does_not_cover(orc):
    wl = W.WORKLOADS["cfg0"]                                  # ffn 688 is not a multiple of 64
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, 0)
    qw = {"embed": w["embed"], "g_final": w["g_final"], "lm_head": random_q4(np.random.default_rng(0), 8, 64),
          "layers": [{**L, **{n: random_q4(np.random.default_rng(0), 8, 64) for n in MATRICES}}
                     for L in w["layers"]]}
    pool = W.fill_kv_pool(cfg, lay, wl.seed_kv)
    with pytest.raises(ValueError):
        orc.decode_step_q4(cfg, qw, pool, lay.block_size, lay.tables, lay.contexts.copy(),
                           W.initial_tokens(cfg, wl.batch, 2))


def test_quantiser_round_trip_within_half_a_step():
    rng = np.random.default_rng(3)
    wb = W.bf16_bits_from_f32((rng.standard_normal((64, 512)) * 0.03).astype(np.float32))
    m = quantize_q4(wb)
    assert m["q"].max() <= 15 and m["q"].shape == (64, 512)
    w = W.f32_from_bf16_bits(wb).astype(np.float64)
    step = np.repeat(W.f32_from_bf16_bits(m["scale"]).astype(np.float64), 64, axis=1)
    # half a step, plus what rounding scale and bias to bf16 moves the grid (2^-8 relative each)
    assert np.all(np.abs(deq(m) - w) <= 0.5 * step + 2.0 ** -8 * (15 * step + np.abs(w).max()))
    # a constant group is reproduced exactly
    c = W.bf16_bits_from_f32(np.full((2, 64), 0.125, np.float32))
    assert np.array_equal(deq(quantize_q4(c)), np.full((2, 64), 0.125))


def test_quantize_weights_covers_every_projection():
    cfg = W.CONFIGS["tiny_q4"]
    qw = quantize_weights(W.make_weights(cfg, 0))
    for L in qw["layers"]:
        for n in MATRICES:
            assert set(L[n]) == {"q", "scale", "bias"}
        assert L["g_attn"].dtype == np.uint16
    assert qw["lm_head"]["q"].shape == (cfg.vocab, cfg.hidden)


def test_q4_oracle_reproduces_stored_fixture(orc):
    """Drift detector: tests/golden/cfg0_q4_oracle.json was written by tests/golden/make_golden.py from
    the oracle (and the input quantiser) alone."""
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg0_q4_oracle.json")
    gold = json.load(open(path))
    wl = W.WORKLOADS["cfg0_q4"]
    cfg, lay = wl.cfg, layout_for(wl)
    qw = quantize_weights(W.make_weights(cfg, wl.seed_weights))
    pool = W.fill_kv_pool(cfg, lay, wl.seed_kv)
    tok = W.initial_tokens(cfg, wl.batch, wl.seed_tokens)
    sl = lay.contexts.copy()
    for g in gold["steps"]:
        r = orc.decode_step_q4(cfg, qw, pool, wl.block_size, lay.tables, sl, tok)
        assert [int(t) for t in r["next"]] == g["next"]
        assert np.allclose(r["logits"][:, :8], np.array(g["logits_0_8"]), rtol=1e-6, atol=1e-7)
        tok, sl = r["next"], sl + 1
