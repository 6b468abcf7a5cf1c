"""GPU parity for 4-bit weights (group-wise affine, groups of 64 columns - the
precision of the checkpoints the paper benchmarks): the HIP decode step with a
packed 4-bit model, called through the C ABI, against the oracle's 4-bit step
on the same codes, scales and biases.

Both sides evaluate the same exact weights scale * q + bias, so the bars are
those of the bf16 path: logits within relative L2 1e-2 (contract) and 2e-4
(regression bound), greedy agreement, append addressing bit-exact.
"""
import numpy as np
import pytest

import workloads as W
from workloads.blocktable import layout_for, build_block_tables
from workloads.quant import quantize_weights
from gpu_common import run_both, run_sampled, check_parity, check_pool, check_pool_sampled

pytestmark = pytest.mark.gpu

TIGHT = 2e-4


@pytest.fixture(scope="module")
def dk():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    import paper_2601_19139_amd as dk
    dk.lib()
    return dk


def variant(base, **kw):
    return W.ModelConfig(**{**W.CONFIGS[base].as_dict(), **kw})


def test_cfg0_q4(dk, orc):
    wl = W.WORKLOADS["cfg0_q4"]                              # contexts 40, 16, 3, 0, 65
    shape, lay = wl.cfg, layout_for(wl)
    weights = quantize_weights(W.make_weights(shape, wl.seed_weights))
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    out = run_both(orc, shape, weights, lay, pool, tokens, wl.steps)
    worst, agree = check_parity(out)
    print(f"cfg0_q4: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT and agree == 1.0
    check_pool(out, pool, shape, lay, wl.steps)
    # free running, the kernels advancing their own tokens and lengths
    out2 = run_both(orc, shape, weights, lay, pool, tokens, wl.steps, teacher_forced=False,
                    gpu_flags=dk.STEP_ADVANCE)
    for g, o in zip(out2["gpu_next"], out2["orc_next"]):
        assert np.array_equal(g, o)


Q4_CASES = [
    # every batch size takes the matrix-core kernels: 1 row, the 16 / 32 / 48 / 64 row tiles
    ("batch1", W.CONFIGS["tiny_q4"], [37], 3),
    ("batch4_empty", W.CONFIGS["tiny_q4"], [0, 0, 15, 16], 2),
    ("batch16", W.CONFIGS["tiny_q4"], [5 + 9 * i for i in range(16)], 2),
    ("batch17_d128", variant("tiny_q4", head_dim=128, n_q_heads=8, n_kv_heads=2), [3 + 7 * i for i in range(17)], 2),
    ("batch33", W.CONFIGS["tiny_q4"], [1 + 3 * i for i in range(33)], 1),
    ("batch64", W.CONFIGS["tiny_q4"], [(11 * i) % 90 for i in range(64)], 1),
    # many row tiles per matrix (the kernels that give a wave 2 and 4 tiles), several K-steps per wave,
    # a vocabulary that is not a multiple of 16, no q/k norm, query groups of 3
    ("wide", variant("tiny_q4", hidden=1280, ffn=5376, vocab=70003, n_q_heads=6, head_dim=128, n_kv_heads=2,
                     qk_norm=False, n_layers=1), [19, 300, 64], 2),
    ("wide_batch24", variant("tiny_q4", hidden=1280, ffn=5376, vocab=70003, n_q_heads=12, head_dim=128,
                             n_kv_heads=2, n_layers=1), [2 + 5 * i for i in range(24)], 1),
    ("g3_d64", variant("tiny_q4", n_q_heads=6, n_kv_heads=2, hidden=384), [21, 64, 1], 2),
]


@pytest.mark.parametrize("name,shape,contexts,steps", Q4_CASES, ids=[c[0] for c in Q4_CASES])
def test_q4_shapes_and_edges(dk, orc, name, shape, contexts, steps):
    lay = build_block_tables(contexts, 16, steps, seed=23)
    weights = quantize_weights(W.make_weights(shape, 6))
    pool = W.fill_kv_pool(shape, lay, 7)
    tokens = W.initial_tokens(shape, len(contexts), 8)
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    worst, agree = check_parity(out)
    print(f"{name}: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT and agree == 1.0, (name, worst, agree)
    check_pool(out, pool, shape, lay, steps)


@pytest.mark.parametrize("heads,hidden,ffn", [((6, 2), 1536, 4096), ((8, 2), 2048, 8192)], ids=["g3", "g4"])
def test_q4_persistent_kernel_wide_classes(dk, orc, heads, hidden, ffn):
    """One row of a 4-bit model with query groups of 3 and 4: the wide classes of the persistent kernel
    with packed codes (must run as the persistent kernel, and meet the oracle)."""
    shape = variant("tiny_q4", hidden=hidden, ffn=ffn, vocab=2000, n_q_heads=heads[0], n_kv_heads=heads[1],
                    head_dim=128, qk_norm=True, n_layers=2)
    lay = build_block_tables([150], 16, 3, seed=31)
    weights = quantize_weights(W.make_weights(shape, 14))
    pool = W.fill_kv_pool(shape, lay, 15)
    tokens = W.initial_tokens(shape, 1, 16)
    out = run_both(orc, shape, weights, lay, pool, tokens, 3)
    assert out["fused_status"] == (0, 0), "the persistent kernel did not run (or gave up a wait)"
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0, (worst, agree)
    check_pool(out, pool, shape, lay, 3)


@pytest.mark.parametrize("contexts", [[37], [64, 5]], ids=["batch1", "batch2"])
def test_q4_both_paths_for_small_batches(dk, orc, contexts):
    """Batches of 1-2 rows take the single persistent kernel (vector-ALU dot products over the
    packed codes); with DK_STEP_NO_FUSED the same step runs kernel per stage on the matrix cores.
    Both must meet the oracle."""
    shape = W.CONFIGS["tiny_q4"]
    lay = build_block_tables(contexts, 16, 3, seed=29)
    weights = quantize_weights(W.make_weights(shape, 10))
    pool = W.fill_kv_pool(shape, lay, 11)
    tokens = W.initial_tokens(shape, len(contexts), 12)
    for flags in (0, dk.STEP_NO_FUSED):
        out = run_both(orc, shape, weights, lay, pool, tokens, 3, gpu_flags=flags)
        worst, agree = check_parity(out)
        assert worst < TIGHT and agree == 1.0, (flags, worst, agree)
        check_pool(out, pool, shape, lay, 3)


@pytest.mark.parametrize("batch", [20, 40, 64])
def test_q4_wide_batches_of_a_large_layer(dk, orc, batch):
    """From 17 rows on the gate/up pair of a large layer (here 10240 x 2048) runs, like the lm_head at every
    batch size, in the GEMM whose waves share one activation tile, with K cut in two across blocks."""
    shape = variant("tiny_q4", n_layers=1, hidden=2048, n_q_heads=16, n_kv_heads=8, head_dim=128, ffn=10240,
                    vocab=70003, rope_theta=1e6)
    contexts = [(29 * i) % 120 for i in range(batch)]
    lay = build_block_tables(contexts, 16, 2, seed=37)
    weights = quantize_weights(W.make_weights(shape, 15))
    pool = W.fill_kv_pool(shape, lay, 16)
    tokens = W.initial_tokens(shape, batch, 17)
    rows = (0, batch // 2, batch - 1)
    out = run_sampled(orc, shape, weights, lay, pool, tokens, 2, rows)
    worst, agree = check_parity(out)
    print(f"4-bit, batch {batch}: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT and agree == 1.0
    check_pool_sampled(out, pool, shape, lay, 2, rows)


Q4_MOE_CASES = [
    # hidden and expert width multiples of 128 and at least 512: the restructured expert kernels with packed
    # 4-bit expert stacks (down projection: the 768-wide and the generic variant), a crowded expert
    ("moe_768", variant("tiny_moe", hidden=1024, expert_ffn=768, n_experts=8, top_k=2), [2 + 3 * i for i in range(20)], 2),
    ("moe_512_crowded", variant("tiny_moe", hidden=1024, expert_ffn=512, n_experts=4, top_k=2), [1 + i for i in range(40)], 1),
    ("moe_batch1", variant("tiny_moe", hidden=512, expert_ffn=512, n_experts=8, top_k=2), [21], 3),
]


@pytest.mark.parametrize("name,shape,contexts,steps", Q4_MOE_CASES, ids=[c[0] for c in Q4_MOE_CASES])
def test_q4_mixture_of_experts(dk, orc, name, shape, contexts, steps):
    """4-bit expert stacks (the router stays bf16): same experts chosen, logits within the bound."""
    lay = build_block_tables(contexts, 16, steps, seed=41)
    weights = quantize_weights(W.make_weights(shape, 18))
    pool = W.fill_kv_pool(shape, lay, 19)
    tokens = W.initial_tokens(shape, len(contexts), 20)
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    for g, o in zip(out["gpu_experts"], out["orc_experts"]):
        assert np.array_equal(np.sort(g, axis=-1), np.sort(o, axis=-1)), name
    worst, agree = check_parity(out)
    print(f"{name}: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT and agree == 1.0, (name, worst, agree)
    check_pool(out, pool, shape, lay, steps)


def test_cfg4_shape_q4_sampled_rows(dk, orc):
    """The 30B-A3B mixture-of-experts shape (128 experts, top 8, expert width 768; cut to 4 layers) with
    4-bit weights at batch 16, ragged contexts with a shared 2048-token prefix: sampled rows."""
    wl = W.WORKLOADS["cfg4_l4"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = quantize_weights(W.make_weights(shape, wl.seed_weights))
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    rows = (1, 8, 14)
    out = run_sampled(orc, shape, weights, lay, pool, tokens, 1, rows)
    worst, agree = check_parity(out)
    print(f"cfg4_l4 shape, 4-bit: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f} on rows {rows}")
    assert worst < TIGHT
    check_pool_sampled(out, pool, shape, lay, 1, rows)


def test_q4_distinct_scales_and_biases_per_group(dk, orc):
    """Codes, scales and biases drawn independently (no relation to a bf16 matrix): a scale or bias
    taken from the wrong row, group or half of a K-step changes the logits by far more than the bound."""
    shape = W.CONFIGS["tiny_q4"]
    rng = np.random.default_rng(12)
    w = W.make_weights(shape, 1)

    def rnd(bits):
        n, k = bits.shape
        return {"q": rng.integers(0, 16, size=(n, k), dtype=np.uint8),
                "scale": W.bf16_bits_from_f32(rng.uniform(0.002, 0.02, size=(n, k // 64)).astype(np.float32)),
                "bias": W.bf16_bits_from_f32(rng.uniform(-0.16, -0.01, size=(n, k // 64)).astype(np.float32))}

    qw = {"embed": w["embed"], "g_final": w["g_final"], "lm_head": rnd(w["lm_head"]),
          "layers": [{k: (rnd(v) if k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down") else v)
                      for k, v in L.items()} for L in w["layers"]]}
    contexts = [9, 33, 70]
    lay = build_block_tables(contexts, 16, 2, seed=3)
    pool = W.fill_kv_pool(shape, lay, 2)
    tokens = W.initial_tokens(shape, len(contexts), 4)
    out = run_both(orc, shape, qw, lay, pool, tokens, 2)
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0, (worst, agree)


def test_q4_prefill_chunk_matches_token_by_token(dk, orc):
    """A prompt written by chunked prefill with 4-bit weights gives the logits of the oracle's
    token-by-token run."""
    import torch
    shape = W.CONFIGS["tiny_q4"]
    weights = quantize_weights(W.make_weights(shape, 9))
    P = 45
    lay = build_block_tables([0], 16, P + 1, seed=5)
    pool = W.fill_kv_pool(shape, lay, 3)
    prompt = np.random.default_rng(4).integers(0, shape.vocab, size=P).astype(np.int32)
    opool = pool.copy()
    ref = None
    for t in range(P):
        ref = orc.decode_step_q4(shape, weights, opool, 16, lay.tables, np.array([t], np.int32), prompt[t:t + 1])
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool)
    pf = dk.Prefiller(dm, dkv)
    nxt, logits = pf.prefill(0, 0, prompt, chunk=16)
    torch.cuda.synchronize()
    got = logits[-1].astype(np.float64)
    rel = np.linalg.norm(got - ref["logits"][0]) / np.linalg.norm(ref["logits"][0])
    assert rel < 2e-3, rel            # the bound of the prefill path (KV rounded to bf16 on both sides)
    assert int(nxt[-1]) == int(ref["next"][0])
    dkv.close()
    dm.close()


def test_cfg1_shape_q4_full_size(dk, orc):
    """The benchmark model shape (28 layers, hidden 1024, vocabulary 151936, context 512) with
    4-bit weights, every logit of the first steps."""
    wl = W.WORKLOADS["cfg1"]
    shape, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(shape, wl.seed_weights)
    if w["lm_head"] is w["embed"]:
        w = {**w, "lm_head": w["embed"].copy()}
    weights = quantize_weights(w)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    steps = 2
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    worst, agree = check_parity(out)
    print(f"cfg1 shape, 4-bit: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT
    check_pool(out, pool, shape, lay, steps)


def test_cfg3_shape_q4_sampled_rows(dk, orc):
    """The 8B shape (cut to 4 layers, so that quantising the weights takes seconds) at batch 16,
    context 4096, 4-bit weights: sampled rows against the oracle."""
    wl = W.WORKLOADS["cfg3_l4"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = quantize_weights(W.make_weights(shape, wl.seed_weights))
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    rows = (3, 12)
    out = run_sampled(orc, shape, weights, lay, pool, tokens, 1, rows)
    worst, agree = check_parity(out)
    print(f"cfg3 shape, 4-bit: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f} on rows {rows}")
    assert worst < TIGHT
    check_pool_sampled(out, pool, shape, lay, 1, rows)
