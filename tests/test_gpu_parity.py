"""GPU parity: the HIP decode path, called through the C ABI, against the CPU
oracle on the same seeded inputs.

Bars (stated for this path): KV-append / block-table addressing bit-exact;
logits within relative L2 1e-2 per row and step; greedy-token agreement >= 99 %
with the GPU fed the oracle's previous tokens (teacher-forced).  The measured
error is around 1e-5, so the tests also assert a much tighter bound to catch
regressions in accumulation precision.
"""
import numpy as np
import pytest

import workloads as W
from workloads.blocktable import layout_for, build_block_tables
from gpu_common import (run_both, run_sampled, free_run, check_parity, parity_stats, free_running_report,
                        log_result, check_pool, check_pool_sampled, rel_l2, TIE_TOL)

pytestmark = pytest.mark.gpu

TIGHT = 2e-4       # regression bound; the contract bound is 1e-2


@pytest.fixture(scope="module")
def dk():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    import paper_2601_19139_amd as dk
    dk.lib()                       # raises if the HIP library is not built
    return dk


def variant(base, **kw):
    return W.ModelConfig(**{**W.CONFIGS[base].as_dict(), **kw})


def test_append_kv_bit_exact(dk, orc):
    import torch
    wl = W.WORKLOADS["cfg0"]
    shape, lay = wl.cfg, layout_for(wl)
    before = np.full(W.pool_shape(shape, lay.num_blocks, 16), W.BF16_NAN_BITS, dtype=np.uint16)
    weights = W.make_weights(shape, 0)
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, before)
    opool = before.copy()
    sl = np.array([32, 17], dtype=np.int32)          # row 0 lands in slot 0 of a fresh block
    d_sl = torch.from_numpy(sl).cuda()
    for layer in range(shape.n_layers):
        k = W.normal_bf16(40 + layer, "k", (2, shape.n_kv_heads, shape.head_dim))
        v = W.normal_bf16(50 + layer, "v", (2, shape.n_kv_heads, shape.head_dim))
        dk.append_kv(dkv.handle, layer, dkv.block_tables, d_sl,
                     torch.from_numpy(k.view(np.int16)).cuda(), torch.from_numpy(v.view(np.int16)).cuda())
        for b in range(2):
            orc.append_kv(shape, opool, 16, layer, lay.tables[b], int(sl[b]),
                          W.f32_from_bf16_bits(k[b]).reshape(-1), W.f32_from_bf16_bits(v[b]).reshape(-1))
    torch.cuda.synchronize()
    got = dkv.bits().reshape(before.shape)
    assert np.array_equal(got, opool)
    assert int((got != before).sum()) == shape.n_layers * 2 * 2 * shape.kv_dim
    dkv.close()
    dm.close()


def test_cfg0_eight_steps(dk, orc):
    wl = W.WORKLOADS["cfg0"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)           # dead slots are NaN
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    out = run_both(orc, shape, weights, lay, pool, tokens, wl.steps)
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0
    check_pool(out, pool, shape, lay, wl.steps)
    # free running with the kernel advancing its own tokens and lengths
    out2 = run_both(orc, shape, weights, lay, pool, tokens, wl.steps, teacher_forced=False,
                    gpu_flags=dk.STEP_ADVANCE)
    for g, o in zip(out2["gpu_next"], out2["orc_next"]):
        assert np.array_equal(g, o)


CASES = [
    # name, shape, contexts, steps
    ("qk_norm_g3_d64", variant("tiny", qk_norm=True, n_q_heads=6, rope_theta=1e6), [19, 40, 1], 3),
    ("empty_context", variant("tiny"), [0, 0], 2),
    ("block_boundaries", variant("tiny", qk_norm=True), [15, 16, 31, 32], 3),
    ("d128_g4", variant("tiny", head_dim=128, n_q_heads=8, n_kv_heads=2, qk_norm=True), [70, 5], 2),
    ("d128_g8_mha_kv1", variant("tiny", head_dim=128, n_q_heads=8, n_kv_heads=1), [33], 2),
    ("g1_mha", variant("tiny", n_q_heads=2, n_kv_heads=2), [21, 64], 2),
    ("g5_d128", variant("tiny", head_dim=128, n_q_heads=10, n_kv_heads=2, qk_norm=True), [90, 3, 257], 2),
    ("g7_d64", variant("tiny", n_q_heads=7, n_kv_heads=1), [40, 300], 2),
    ("g5_batch16", variant("tiny", head_dim=128, n_q_heads=5, n_kv_heads=1), [2 + 21 * i for i in range(16)], 2),
    ("g7_batch9", variant("tiny", n_q_heads=14, n_kv_heads=2, qk_norm=True), [7 + 40 * i for i in range(9)], 2),
    ("multi_chunk_ragged", variant("tiny", qk_norm=True), [300, 65, 128, 7, 191], 3),
    ("batch7", variant("tiny"), [3, 50, 17, 80, 1, 64, 33], 2),
    ("odd_sizes", variant("tiny", hidden=264, ffn=1000, vocab=1003), [29, 12], 2),
    # batches above 4 rows take the matrix-core GEMM path (rows padded to 16, 32, 48, 64)
    ("batch16", variant("tiny", qk_norm=True), [5 + 9 * i for i in range(16)], 2),
    ("batch5_odd_sizes", variant("tiny", hidden=264, ffn=1000, vocab=1003), [29, 12, 0, 77, 16], 2),
    ("batch20_d128", variant("tiny", head_dim=128, n_q_heads=8, n_kv_heads=2, qk_norm=True),
     [3 + 7 * i for i in range(20)], 2),
    ("batch40", variant("tiny"), [1 + 3 * i for i in range(40)], 1),
    ("batch64", variant("tiny", qk_norm=True), [(11 * i) % 90 for i in range(64)], 1),
]


@pytest.mark.parametrize("name,shape,contexts,steps", CASES, ids=[c[0] for c in CASES])
def test_shapes_and_edges(dk, orc, name, shape, contexts, steps):
    lay = build_block_tables(contexts, 16, steps, seed=17)
    weights = W.make_weights(shape, 3)
    pool = W.fill_kv_pool(shape, lay, 4)
    tokens = W.initial_tokens(shape, len(contexts), 5)
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0, (name, worst, agree)
    check_pool(out, pool, shape, lay, steps)


@pytest.mark.parametrize("wname,steps", [("cfg0", 8), ("cfg1", 4)])
def test_persistent_and_kernel_per_stage_paths_agree(dk, orc, wname, steps):
    """Batches of 1-2 rows of the small dense shapes run as one persistent
    kernel; the same step as a chain of kernels (DK_STEP_NO_FUSED) must pass the
    same parity bars and give the same tokens."""
    wl = W.WORKLOADS[wname]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    fused = run_both(orc, shape, weights, lay, pool, tokens, steps)
    chain = run_both(orc, shape, weights, lay, pool, tokens, steps, gpu_flags=dk.STEP_NO_FUSED)
    assert fused["fused_status"] == (0, 0), "the persistent kernel did not run (or gave up a wait)"
    assert chain["fused_status"] is None
    for out in (fused, chain):
        worst, agree = check_parity(out)
        assert worst < TIGHT and agree == 1.0
        check_pool(out, pool, shape, lay, steps)
    for a, b in zip(fused["gpu_logits"], chain["gpu_logits"]):
        assert rel_l2(a, b).max() < 5e-5          # each is ~1e-5 from the oracle
    # the persistent kernel repeats bit for bit
    again = run_both(orc, shape, weights, lay, pool, tokens, steps)
    for a, b in zip(fused["gpu_logits"], again["gpu_logits"]):
        assert np.array_equal(a, b)


def test_persistent_kernel_gives_up_cleanly(dk, orc):
    """Every wait of the persistent kernel is bounded.  With the bound forced down to one poll
    (a host-side test hook) the kernel still runs to its end, marks the step invalid (token -1,
    nothing advanced, status words set) and the next step with the normal bound is right again."""
    import torch
    wl = W.WORKLOADS["cfg0"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool)
    dec = dk.Decoder(dm, dkv, lay.contexts, tokens)
    dk.debug_set_wait_limit(dm.handle, 1)
    dec.step(flags=dk.STEP_ADVANCE)
    torch.cuda.synchronize()
    assert (dec.next.cpu().numpy() == -1).all()
    assert np.array_equal(dec.seq_lens.cpu().numpy(), lay.contexts)          # not advanced
    assert np.array_equal(dec.tokens.cpu().numpy(), tokens)
    serial, gave_up = dec.fused_status()
    assert serial != 0 and gave_up > 0
    dk.debug_set_wait_limit(dm.handle, 0)                                     # back to the default
    dec.step()
    torch.cuda.synchronize()
    opool = pool.copy()
    r = orc.decode_step(shape, weights, opool, 16, lay.tables, lay.contexts, tokens)
    assert np.array_equal(dec.next.cpu().numpy(), r["next"])
    assert rel_l2(dec.logits.cpu().numpy(), r["logits"]).max() < TIGHT
    assert np.array_equal(dkv.bits().reshape(pool.shape) != pool, opool != pool)   # the slot was rewritten
    dkv.close()
    dm.close()


FUSED_CASES = [
    # contexts around the 64-token attention chunks of the persistent kernel, for both of its
    # shape classes (head_dim 64 and 128, query groups of 2), one and two rows
    ("d64_chunk_edges", variant("tiny", qk_norm=True), [63, 64], 3),
    ("d64_one_row_long", variant("tiny"), [700], 2),
    ("d64_empty_and_long", variant("tiny", qk_norm=True), [0, 830], 2),
    ("d128_chunk_edges", variant("tiny", head_dim=128, n_q_heads=4, n_kv_heads=2, qk_norm=True), [127, 65], 3),
    ("d128_one_row", variant("tiny", head_dim=128, n_q_heads=4, n_kv_heads=2), [129], 2),
    ("d128_wide", variant("tiny", head_dim=128, n_q_heads=16, n_kv_heads=8, hidden=1024, ffn=3072, vocab=2000,
                          qk_norm=True), [1, 513], 2),
    # the wide classes (one row): query groups of 3 and 4 - two result elements per thread in the chunk
    # merge -, hidden up to 4096, rows of up to 12288 columns; contexts over several chunks, and one
    # long enough that a block takes more than one attention item (8 kv heads x 40 chunks > 256 blocks)
    ("g3_3b_layer", variant("tiny", n_layers=2, head_dim=128, n_q_heads=24, n_kv_heads=8, hidden=3072, ffn=8192,
                            vocab=3001, rope_theta=5e5), [333], 2),
    ("g3_narrow", variant("tiny", head_dim=128, n_q_heads=6, n_kv_heads=2, hidden=1536, ffn=4000, vocab=1500,
                          qk_norm=True), [64], 3),
    ("g4_8b_layer", variant("tiny", n_layers=2, head_dim=128, n_q_heads=32, n_kv_heads=8, hidden=4096, ffn=12288,
                            vocab=3001, qk_norm=True, rope_theta=1e6), [130], 2),
    ("g4_many_items", variant("tiny", head_dim=128, n_q_heads=32, n_kv_heads=8, hidden=2048, ffn=4096, vocab=1000,
                              qk_norm=True), [2555], 2),
]


@pytest.mark.parametrize("name,shape,contexts,steps", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_persistent_kernel_edges(dk, orc, name, shape, contexts, steps):
    lay = build_block_tables(contexts, 16, steps, seed=23)
    weights = W.make_weights(shape, 6)
    pool = W.fill_kv_pool(shape, lay, 7)
    tokens = W.initial_tokens(shape, len(contexts), 8)
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    assert out["fused_status"] == (0, 0), "the persistent kernel did not run (or gave up a wait)"
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0, (name, worst, agree)
    check_pool(out, pool, shape, lay, steps)


def test_shared_prefix_blocks(dk, orc):
    shape = variant("tiny", qk_norm=True)
    ctx = [100, 70, 65, 90, 20]
    lay = build_block_tables(ctx, 16, 3, shared_prefix=64, n_sharers=4, seed=23)
    assert lay.refcount.max() == 4
    weights = W.make_weights(shape, 6)
    pool = W.fill_kv_pool(shape, lay, 7)
    tokens = W.initial_tokens(shape, len(ctx), 8)
    out = run_both(orc, shape, weights, lay, pool, tokens, 3)
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0
    check_pool(out, pool, shape, lay, 3)


def test_batch_rows_do_not_interact_and_runs_repeat(dk, orc):
    """A request joining or leaving the batch must not change another request's
    tokens (the continuous-batching loop of the paper's Algorithm 1)."""
    import torch
    shape = variant("tiny", qk_norm=True)
    ctx = [37, 90, 16]
    lay = build_block_tables(ctx, 16, 2, seed=31)
    weights = W.make_weights(shape, 9)
    pool = W.fill_kv_pool(shape, lay, 10)
    tokens = W.initial_tokens(shape, 3, 11)
    full = run_both(orc, shape, weights, lay, pool, tokens, 2)
    again = run_both(orc, shape, weights, lay, pool, tokens, 2)
    for a, b in zip(full["gpu_logits"], again["gpu_logits"]):
        assert np.array_equal(a, b), "two runs of the same step differ bit for bit"
    for b in range(3):
        sub = build_block_tables(ctx[b:b + 1], 16, 2, seed=31)
        sub.tables = lay.tables[b:b + 1].copy()
        sub.num_blocks = lay.num_blocks
        one = run_both(orc, shape, weights, sub, pool, tokens[b:b + 1], 2)
        for s in range(2):
            r = rel_l2(one["gpu_logits"][s][0], full["gpu_logits"][s][b])
            assert r < 1e-5
            assert one["gpu_next"][s][0] == full["gpu_next"][s][b]


def test_argmax_ties_take_the_lowest_index(dk, orc):
    shape = variant("tiny")
    lay = build_block_tables([5, 9], 16, 1, seed=3)
    weights = W.make_weights(shape, 12)
    lm = np.zeros_like(weights["lm_head"])
    lm[700] = weights["lm_head"][3]
    lm[300] = weights["lm_head"][3]
    lm[1023] = weights["lm_head"][3]
    weights = dict(weights, lm_head=lm)
    pool = W.fill_kv_pool(shape, lay, 13)
    out = run_both(orc, shape, weights, lay, pool, np.array([1, 2], dtype=np.int32), 1)
    assert np.array_equal(out["gpu_next"][0], out["orc_next"][0])
    assert set(out["orc_next"][0]) <= {0, 300}


def test_logits_optional(dk, orc):
    import torch
    wl = W.WORKLOADS["cfg0"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, 0)
    pool = W.fill_kv_pool(shape, lay, 1)
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool)
    dec = dk.Decoder(dm, dkv, lay.contexts, W.initial_tokens(shape, 2, 2), want_logits=False)
    dec.step()
    torch.cuda.synchronize()
    r = orc.decode_step(shape, weights, pool.copy(), 16, lay.tables, lay.contexts,
                        W.initial_tokens(shape, 2, 2))
    assert np.array_equal(dec.next.cpu().numpy(), r["next"])
    dkv.close()
    dm.close()


def test_cfg1_full_size(dk, orc):
    """The benchmark workload at full size (28 layers, vocabulary 151936, context 512) for its
    whole configured length: every logit of all 128 steps, teacher-forced, so the 99 % greedy
    agreement bar is measured on 128 tokens; the context grows from 512 to 639 and crosses eight
    block boundaries.  Also reported (not graded): the GPU decoding on its own tokens against the
    oracle on its own."""
    wl = W.WORKLOADS["cfg1"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    steps = wl.steps
    assert steps == 128
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    check_parity(out)
    st = parity_stats(out)
    dm = dk.DeviceModel(shape, weights)
    free = free_run(dk, dm, lay, pool, tokens, steps)
    dm.close()
    fr_agree, fr_first = free_running_report(free, out["orc_next"])
    # 128 steps on the kernel's own appended k/v: logits drift to ~1e-4 from the oracle, and with
    # them the share of appended values that round to the neighbouring bf16 (see check_pool)
    flips = check_pool(out, pool, shape, lay, steps, max_flips=0.08)
    log_result(f"cfg1 full size: {st['tokens']} tokens teacher-forced, greedy agreement {st['agree']:.4f}, "
               f"logits rel-L2 worst {st['worst']:.3e} mean {st['mean']:.3e}; free-running agreement "
               f"{fr_agree:.3f}, first divergence at step {fr_first}; appended values one bf16 step off: {flips:.4f}")
    assert st["tokens"] == 128 and st["agree"] >= 0.99
    assert st["worst"] < TIGHT


@pytest.mark.parametrize("wname", ["b1_3b", "b1_8b"])
def test_single_request_on_the_larger_shapes_full_size(dk, orc, wname):
    """One request alone on the 3B and 8B shapes at full size (28 / 36 layers, context 512): the wide
    classes of the persistent kernel (query groups of 3 and 4, two result elements per thread in the
    chunk merge, rows of 8192 / 12288 columns), 12 steps teacher-forced across a block boundary, every
    logit against the oracle; the kernel-per-stage path must give the same tokens."""
    wl = W.WORKLOADS[wname]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    steps = 12
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    assert out["fused_status"] == (0, 0), "the persistent kernel did not run (or gave up a wait)"
    check_parity(out)
    st = parity_stats(out)
    check_pool(out, pool, shape, lay, steps)
    log_result(f"{wname} full size (persistent kernel): {st['tokens']} tokens teacher-forced, greedy agreement "
               f"{st['agree']:.4f}, logits rel-L2 worst {st['worst']:.3e} mean {st['mean']:.3e}")
    assert st["tokens"] == steps and st["agree"] == 1.0 and st["worst"] < TIGHT
    staged = run_both(orc, shape, weights, lay, pool, tokens, 2, gpu_flags=dk.STEP_NO_FUSED)
    for a, b in zip(staged["gpu_next"], out["gpu_next"][:2]):
        assert np.array_equal(a, b)


# rows: sharers of the prefix and non-sharers; rows x steps >= 128 compared tokens per workload
FULL_SIZE = [("cfg2", (0, 2, 5, 7, 8, 10, 13, 15), 16), ("cfg3", (1, 6, 11, 14), 32),
             ("cfg4_l4", (1, 8, 14), 2), ("cfg4", (0, 5, 9, 15), 32)]


@pytest.mark.parametrize("wname,rows,steps", FULL_SIZE, ids=[c[0] for c in FULL_SIZE])
def test_batch16_full_size_sampled_rows(dk, orc, wname, rows, steps):
    """The batch-16 workloads at full size (Llama-3.2-3B shape with ragged contexts and a shared
    1024-token prefix; Qwen3-8B shape, context 4096; the Qwen3-30B-A3B mixture-of-experts shape
    with all 48 layers, 128 experts, top 8, ragged contexts and a shared 2048-token prefix): the
    GPU decodes all 16 rows, the oracle the sampled rows, teacher-forced, for enough steps that
    rows x steps >= 128 tokens stand behind the 99 % greedy-agreement bar; every logit of those
    rows is compared, and append addressing is checked for all rows.  The 8B rows start at a block
    boundary (4096) and cross another at 4112.  cfg4_l4 is the mixture-of-experts shape cut to 4
    layers (5 GB of weights instead of 61), kept as a quick check.  Mixture-of-experts models: the
    top-k choice of a router is an integer decided by floating point, and with random experts one
    swapped expert changes everything behind it; over 48 layers x 128 tokens a handful of choices
    fall between two probabilities closer than float32 resolves.  There the kernel's set is proposed
    to the oracle, which adopts it only if it is a valid top-k set up to TIE_TOL (count and margins
    are reported; any choice beyond the tolerance fails the test).  Reported, not graded: the GPU
    decoding the configured number of steps on its own tokens against the oracle on its own."""
    wl = W.WORKLOADS[wname]
    shape, lay = wl.cfg, layout_for(wl)
    if wl.n_sharers:
        n_sh = sum(r < wl.n_sharers for r in rows)
        assert 0 < n_sh < len(rows)                       # sharers and non-sharers are sampled
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    out = run_sampled(orc, shape, weights, lay, pool, tokens, steps, rows, free_steps=wl.steps, tie_tol=TIE_TOL)
    if shape.n_experts:
        routed = shape.n_layers * len(rows) * steps
        worst_tie = max([m for *_, m in out["ties"]], default=0.0)
        log_result(f"{wname}: router near-ties: {len(out['ties'])} of {routed} (layer, row, step) choices differed "
                   f"from the oracle's own within the tolerance {TIE_TOL:g} and were adopted (largest margin "
                   f"{worst_tie:.2e}); refused (beyond the tolerance): {out['tie_refused'][:4]}")
        assert not out["tie_refused"], "the kernel chose an expert the oracle does not rank within the tolerance"
        assert len(out["ties"]) <= 0.01 * routed
    check_parity(out)
    st = parity_stats(out)
    fr_agree, fr_first = free_running_report(out["free_next"], out["orc_next"], rows)
    boundary = sum(int((int(lay.contexts[r]) + s) % 16 == 0) for r in rows for s in range(steps))
    log_result(f"{wname} full size: {st['tokens']} tokens teacher-forced (rows {rows} x {steps} steps, "
               f"{boundary} of them opening a block), greedy agreement {st['agree']:.4f}, logits rel-L2 worst "
               f"{st['worst']:.3e} mean {st['mean']:.3e}; free-running ({wl.steps} steps run, {steps} compared) "
               f"agreement {fr_agree:.3f}, first divergence at step {fr_first}")
    assert st["tokens"] == len(rows) * steps and st["agree"] >= 0.99
    if wname != "cfg4_l4":
        assert st["tokens"] >= 128 and boundary > 0
    # regression bound: 2e-4 as everywhere; the 48-layer mixture of experts reaches 2.7e-4 after 32 steps
    # on its own appended k/v (twice the depth of the other shapes, expert weights renormalised from float32
    # probabilities), so its bound is 5e-4 - the contract (1e-2) is held by check_parity above
    assert st["worst"] < (5e-4 if wname == "cfg4" else TIGHT)
    for f in out["free_next"]:
        assert ((f >= 0) & (f < shape.vocab)).all()
    # appended values: one bf16 step plus ten times the drift of the float32 values behind them,
    # which follows the logits' (1e-4 elsewhere, up to 2.7e-4 for the 48-layer mixture of experts)
    check_pool_sampled(out, pool, shape, lay, steps, rows, drift=3e-3 if wname == "cfg4" else 1e-4)


@pytest.mark.parametrize("batch", [16, 20, 40, 64])
def test_wide_batches_of_a_large_layer(dk, orc, batch):
    """Large layer matrices run, from 16 rows on, in the GEMM whose waves share one activation
    tile in LDS, with K cut across blocks and the last block to arrive adding the slices in slice
    order (the lm_head joins from 17 rows on, with one slice).  One layer with matrices large enough
    to take each of those paths (q/k/v 6144 x 2048, gate/up 20480 x 2048, down 2048 x 20480,
    vocabulary 70003), two steps so that the tickets are used twice; sampled rows against the
    oracle.  Which block arrives last varies from run to run, the sums must not: a second run from
    the same state gives the same bits."""
    shape = variant("tiny", n_layers=1, hidden=2048, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=20480,
                    vocab=70003, qk_norm=True, rope_theta=1e6)
    contexts = [(37 * i) % 150 for i in range(batch)]
    lay = build_block_tables(contexts, 16, 2, seed=31)
    weights = W.make_weights(shape, 12)
    pool = W.fill_kv_pool(shape, lay, 13)
    tokens = W.initial_tokens(shape, batch, 14)
    rows = (0, batch // 2, batch - 1)
    out = run_sampled(orc, shape, weights, lay, pool, tokens, 2, rows)
    worst, agree = check_parity(out)
    print(f"batch {batch}: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}")
    assert worst < TIGHT and agree == 1.0
    check_pool_sampled(out, pool, shape, lay, 2, rows)
    again = run_sampled(orc, shape, weights, lay, pool, tokens, 2, rows)
    for a, b in zip(out["gpu_logits"], again["gpu_logits"]):
        assert np.array_equal(a, b)
    assert np.array_equal(out["gpu_pool"], again["gpu_pool"])


@pytest.mark.parametrize("hidden,heads,ffn,batch", [(2560, (32, 8), 9728, 16), (2560, (32, 8), 9728, 48),
                                                    (5120, (40, 8), 17408, 16), (5120, (40, 8), 17408, 33)])
def test_layer_shapes_outside_the_calibration(dk, orc, hidden, heads, ffn, batch):
    """Which GEMM kernel (and how many K slices) a matrix takes comes from a cost estimate whose
    constants were fitted on four model shapes; one layer of two shapes it never saw (hidden 2560 /
    ffn 9728, hidden 5120 / ffn 17408), at 16 rows and above, against the oracle on sampled rows, and
    bit-repeatable like every K-sliced sum."""
    shape = variant("tiny", n_layers=1, hidden=hidden, n_q_heads=heads[0], n_kv_heads=heads[1], head_dim=128, ffn=ffn,
                    vocab=32003, qk_norm=True, rope_theta=1e6)
    # (contexts of at least 40 tokens: with an empty context the attention output IS the new token's v,
    # rounded to bf16 from float32 here and from float64 in the oracle, and one differently rounded value
    # of a 5120-wide layer shows in that row's logits at 4e-4 - the empty-context cases of
    # test_shapes_and_edges cover that at its own bound)
    contexts = [40 + (29 * i) % 130 for i in range(batch)]
    lay = build_block_tables(contexts, 16, 2, seed=41)
    weights = W.make_weights(shape, 22)
    pool = W.fill_kv_pool(shape, lay, 23)
    tokens = W.initial_tokens(shape, batch, 24)
    rows = (0, batch // 2, batch - 1)
    qkv = (heads[0] + 2 * heads[1]) * 128
    plans = [dk.gemm_plan_query(e, n, k, batch) for e, n, k in ((0, qkv, hidden), (1, hidden, heads[0] * 128),
                                                               (2, ffn, hidden), (1, hidden, ffn))]
    print(f"hidden {hidden} batch {batch}: plans (waves, slices, est us) q|k|v, o, gate/up, down: {plans}", flush=True)
    assert any(w for w, _, _ in plans)          # the K-sliced kernel is among them
    out = run_sampled(orc, shape, weights, lay, pool, tokens, 2, rows)
    worst, agree = check_parity(out)
    print(f"hidden {hidden} batch {batch}: worst rel-L2 {worst:.3e}, greedy agreement {agree:.3f}", flush=True)
    assert worst < TIGHT and agree == 1.0, (worst, agree)
    check_pool_sampled(out, pool, shape, lay, 2, rows)
    again = run_sampled(orc, shape, weights, lay, pool, tokens, 2, rows)
    for a, b in zip(out["gpu_logits"], again["gpu_logits"]):
        assert np.array_equal(a, b)
    assert np.array_equal(out["gpu_pool"], again["gpu_pool"])


MOE_CASES = [
    ("cfg0_moe", W.CONFIGS["tiny_moe"], [33, 16, 5], 4),
    ("moe_batch1", W.CONFIGS["tiny_moe"], [21], 3),
    ("moe_32x4_batch16", variant("tiny_moe", n_experts=32, top_k=4, expert_ffn=104), [3 + 5 * i for i in range(16)], 2),
    # 40 rows over 4 experts: some expert serves more than 16 rows (several column passes)
    ("moe_crowded", variant("tiny_moe", n_experts=4, top_k=2, head_dim=128, n_q_heads=4, n_kv_heads=1),
     [1 + 2 * i for i in range(40)], 1),
    # hidden and expert width multiples of 128: the restructured expert kernels (8 waves x 1 row
    # tile for gate/up; 6 or 4 waves x 4 row tiles for down), with a crowded expert as well
    ("moe_wide_768", variant("tiny_moe", hidden=1024, expert_ffn=768, n_experts=8, top_k=2),
     [2 + 3 * i for i in range(20)], 2),
    ("moe_wide_512", variant("tiny_moe", hidden=1024, expert_ffn=512, n_experts=4, top_k=2),
     [1 + i for i in range(40)], 1),
]


@pytest.mark.parametrize("name,shape,contexts,steps", MOE_CASES, ids=[c[0] for c in MOE_CASES])
def test_mixture_of_experts(dk, orc, name, shape, contexts, steps):
    """Softmax router, top-k (ties to the lower index), renormalised weights,
    expert SwiGLU: logits and the routing itself against the oracle."""
    lay = build_block_tables(contexts, 16, steps, seed=41)
    weights = W.make_weights(shape, 14)
    pool = W.fill_kv_pool(shape, lay, 15)
    tokens = W.initial_tokens(shape, len(contexts), 16)
    out = run_both(orc, shape, weights, lay, pool, tokens, steps)
    worst, agree = check_parity(out)
    assert worst < TIGHT and agree == 1.0, (name, worst, agree)
    check_pool(out, pool, shape, lay, steps)
    same = total = 0
    for g, o in zip(out["gpu_experts"], out["orc_experts"]):
        same += int((np.sort(g, -1) == np.sort(o, -1)).all(-1).sum())
        total += g.shape[0] * g.shape[1]
    # a near-tie in the router may legitimately pick another expert; with these
    # seeds none does
    assert same == total, f"{name}: routing differs on {total - same} of {total} (layer, row) pairs"


@pytest.mark.parametrize("batch", [2, 20])
def test_decode_step_replays_in_a_hip_graph(dk, orc, batch):
    """The kernel-per-stage step keeps no host state between calls and enqueues only kernels, so a
    caller can capture it in a HIP graph (the persistent kernel alternates buffer sets on the host and
    is excluded with DK_STEP_NO_FUSED).  Eight replays, with eager work and synchronisation between
    them, must give the tokens of eight eager steps, and the last one the oracle's logits."""
    import torch
    shape = variant("tiny", qk_norm=True, vocab=70003 if batch > 16 else 1024)
    contexts = [(13 * i) % 70 for i in range(batch)]
    steps = 8
    lay = build_block_tables(contexts, 16, steps + 1, seed=43)
    weights = W.make_weights(shape, 20)
    pool = W.fill_kv_pool(shape, lay, 21)
    tokens = W.initial_tokens(shape, batch, 22)
    flags = dk.STEP_ADVANCE | dk.STEP_NO_FUSED
    dm = dk.DeviceModel(shape, weights)

    def fresh():
        dkv = dk.DeviceKV(dm, lay, pool)
        return dkv, dk.Decoder(dm, dkv, lay.contexts, tokens)

    dkv, dec = fresh()
    eager = []
    for _ in range(steps):
        dec.step(flags=flags)
        torch.cuda.synchronize()
        eager.append(dec.next.cpu().numpy().copy())
    eager_logits = dec.logits.cpu().numpy().copy()
    dkv.close()

    dkv, dec = fresh()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        dec.step(flags=flags, stream=stream.cuda_stream)          # step 0 eagerly (also the one-time set-up calls)
        stream.synchronize()
        got = [dec.next.cpu().numpy().copy()]
        graph.capture_begin()
        dec.step(flags=flags, stream=stream.cuda_stream)
        graph.capture_end()
    scratch = torch.zeros(1 << 20, device="cuda")
    for _ in range(steps - 1):
        graph.replay()
        torch.cuda.synchronize()
        got.append(dec.next.cpu().numpy().copy())
        scratch += 1.0                                            # the program's own eager work between replays
        torch.cuda.synchronize()
    for a, b in zip(eager, got):
        assert np.array_equal(a, b)
    assert np.array_equal(dec.logits.cpu().numpy(), eager_logits)  # same kernels, same order: bit for bit
    assert np.array_equal(dec.seq_lens.cpu().numpy(), lay.contexts + steps)
    # and the replayed chain is the oracle's: teacher-free comparison of the last step's logits
    opool, sl, tok = pool.copy(), lay.contexts.copy(), tokens.copy()
    agree = True
    for k in range(steps):
        r = orc.decode_step(shape, weights, opool, 16, lay.tables, sl, tok)
        agree = agree and np.array_equal(r["next"], got[k])
        sl, tok = sl + 1, r["next"]
    assert agree, "free-running greedy tokens left the oracle's path (no near-tie expected with this seed)"
    assert rel_l2(dec.logits.cpu().numpy(), r["logits"]).max() < 1e-3
    dkv.close()
    dm.close()
