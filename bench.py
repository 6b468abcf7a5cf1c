#!/usr/bin/env python3
"""Decode-step benchmark on one MI355X.

A "step" is one call of the decode step over the whole batch: embedding,
every layer (q/k/v projection, head norm + rotary embedding + KV append,
ragged paged attention, output projection, SwiGLU MLP), final norm, lm_head
and greedy argmax - one new token for each of the B sequences.  Inputs
(weights, KV pool, block tables, tokens) are resident in HBM before the timed
region.  Prints one JSON line: the contract fields, `roofline` (the dominant kernel
class against the published HBM peak and against a read-only streaming kernel
measured on the spot), `step_roofline` (the whole step), per-kernel times, the
batch-16 figure of the same model (batch-1 workloads), in the default run the
batch-16 workloads `cfg2`, `cfg3` and `cfg4_l4` timed the same way (their own keys),
and the CPU oracle's rate.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

# HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (scaled by a plain copy
# kernel: x2.0 and x1.0 to KiB), see profiles/decode_step_cfg1_hbm_counters.md.
# Quoted only while the library reports the kernel revision they were taken on.
MEASURED_TRAFFIC = {("cfg1", "fused_step"): ("fused r9", 1290928457),      # the whole step, one launch
                    ("cfg1", "gemv"): ("gemv r3", 10805373)}             # --kernel-per-stage


def cpu_baseline(shape, weights, layout, pool_bits, tokens, budget_s=12.0, max_steps=64, max_rows=2):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    the first `max_rows` rows of the batch (rows do not interact), free-running
    greedy steps until about `budget_s` seconds have passed."""
    import numpy as np
    from oracle import oracle_f64
    orc = oracle_f64()
    step = orc.decode_step_q4 if isinstance(weights["lm_head"], dict) else orc.decode_step
    rows = list(range(min(max_rows, len(tokens))))
    pool = pool_bits.copy()
    sl = layout.contexts[rows].copy()
    tok = np.asarray(tokens, dtype=np.int32)[rows].copy()
    tables = layout.tables[rows]
    step(shape, weights, pool, layout.block_size, tables, sl, tok, want_logits=False)   # warm-up
    sl, n, t0 = sl + 1, 0, time.perf_counter()
    while n < max_steps and (n == 0 or time.perf_counter() - t0 < budget_s):
        r = step(shape, weights, pool, layout.block_size, tables, sl, tok, want_logits=False)
        tok, sl, n = r["next"], sl + 1, n + 1
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": round(n * len(rows) / dt, 3), "unit": "tok/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} greedy steps of {len(rows)} of the {len(tokens)} rows of the same workload "
                      f"(fp64 C loops, OpenMP over rows of a matrix)"}


def dtype_name(args):
    return "bf16" if args.weights == "bf16" else "bf16 activations and KV, 4-bit weights (fp32 accumulation)"


def make_model_weights(args, W, shape, seed):
    """Seeded weights of the shape; with --weights q4 the projections and the lm_head quantised to 4 bits."""
    weights = W.make_weights(shape, seed)
    if args.weights == "q4":
        from workloads.quant import quantize_weights
        if weights["lm_head"] is weights["embed"]:
            weights = {**weights, "lm_head": weights["embed"].copy()}   # the embedding table stays bf16
        weights = quantize_weights(weights)
    return weights


def read_ceiling(dk, torch):
    """Read-only bandwidth of a plain streaming kernel on this device (dk_read_stream over 2 GiB that no
    cache holds, best of five launches): the practical ceiling next to the published peak."""
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    best = None
    for _ in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dk.read_stream(buf, sink)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    del buf
    return (2 << 30) / (best * 1e-3) / 1e9


def batch16_line(args, wl, dk, W, np, torch, dm, tok_s_batch1):
    """The same model with 16 concurrent sequences of the workload's context length (private caches):
    the other end of the paper's 1 -> 16 concurrent-request sweep.  Reported beside the batch-1 figure."""
    from workloads.blocktable import build_block_tables
    shape = wl.cfg
    ctx, B, span = int(wl.contexts[0]), 16, 64
    lay = build_block_tables([ctx] * B, wl.block_size, span, seed=wl.seed_blocks)
    pool_bits = W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False)
    dkv = dk.DeviceKV(dm, lay, pool_bits)
    dec = dk.Decoder(dm, dkv, lay.contexts, W.initial_tokens(shape, B, wl.seed_tokens), want_logits=True)
    d_ctx0, d_tok0 = dec.seq_lens.clone(), dec.tokens.clone()
    steps = min(args.steps, span)

    def run(n):
        dec.seq_lens.copy_(d_ctx0)
        dec.tokens.copy_(d_tok0)
        for _ in range(n):
            dec.step(flags=dk.STEP_ADVANCE)

    run(min(args.warmup, span))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    mean_ctx = (lay.contexts + (steps - 1) // 2).astype(np.int32)
    alg = dk.step_algorithmic_bytes(dm.handle, dkv.handle, lay.tables, mean_ctx, with_logits=True)
    tok_s = B * steps / wall
    out = {"workload": f"{shape.name} decode, batch {B}, context {ctx} growing, private caches, greedy",
           "value": round(tok_s, 2), "unit": "tok/s", "steps": steps, "ms_per_step": round(wall * 1e3 / steps, 5),
           "vs_batch1": round(tok_s / tok_s_batch1, 2), "algorithmic_bytes_per_step": int(alg),
           "achieved_GBs": round(alg / (wall / steps) / 1e9, 1),
           "frac": round(alg / (wall / steps) / 1e9 / HBM_PEAK_GBS, 4)}
    dkv.close()
    return out


def bench_prefill(args, wl, dk, W, np, torch):
    """Chunked prefill of one P-token prompt (next row after the decode step; not the headline metric)."""
    from workloads.blocktable import build_block_tables
    shape, P, chunk = wl.cfg, args.prefill, 64
    lay = build_block_tables([0], 16, P + 1, seed=wl.seed_blocks)
    weights = make_model_weights(args, W, shape, wl.seed_weights)
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False))
    pre = dk.Prefiller(dm, dkv, max_chunk=chunk, want_logits=False)
    toks = torch.from_numpy(W.initial_tokens(shape, P, wl.seed_tokens)).cuda()
    table = dkv.block_tables[0]

    def one_prompt():
        for o in range(0, P, chunk):
            part = toks[o:o + chunk]
            last = o + chunk >= P                     # only the last chunk's prediction is needed
            dk.prefill_chunk(dm.handle, dkv.handle, table, o, part, pre._ws_ptr, pre.ws_bytes, None,
                             pre.next if last else None)

    for _ in range(max(1, args.warmup // 4)):
        one_prompt()
    torch.cuda.synchronize()
    reps = max(1, args.steps // 8)
    t0 = time.perf_counter()
    for _ in range(reps):
        one_prompt()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / reps
    n_chunks = (P + chunk - 1) // chunk
    # per chunk: every dense weight once; the sequence's cached K/V once; the chunk's own K/V written
    kv_tok = shape.n_layers * 2 * shape.n_kv_heads * shape.head_dim * 2
    head = shape.vocab * shape.hidden * 2
    alg = sum(shape.dense_weight_bytes() - (0 if o + chunk >= P else head) + min(o + chunk, P) * kv_tok
              for o in range(0, P, chunk))
    # the method's own arithmetic: two flops per weight of the projections and token (the lm_head for the last
    # token only), and per layer and token 4 * n_q_heads * head_dim flops per cached position it attends to
    flops = 2.0 * ((shape.dense_weight_bytes() - head) / 2) * P + 2.0 * (head / 2) \
        + 4.0 * shape.n_layers * shape.n_q_heads * shape.head_dim * (P * (P + 1) / 2)
    print(json.dumps({
        "metric": "prefill_tok_per_s", "value": round(P / wall, 1), "unit": "tok/s", "n_gpus": 1,
        "steps": reps, "ms_per_step": round(wall * 1e3, 4), "higher_is_better": True, "dtype": dtype_name(args),
        "data": "synthetic (seeded random-init weights)",
        "config": {"workload": f"{shape.name}: one {P}-token prompt into an empty cache, {chunk} tokens per chunk",
                   "chunks": n_chunks},
        "roofline": {"bound": "hbm", "achieved": round(alg / wall / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(alg / wall / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "note": "weights are streamed once per 64-token chunk (the decode kernels with the rows "
                             "of one sequence); a compute-bound large-tile prefill is not built"},
        # the same run against the matrix cores' dense bf16 peak (what a compute-bound prefill would be held to)
        "mfma_roofline": {"bound": "mfma", "achieved": round(flops / wall / 1e12, 2), "peak": 2500.0, "unit": "TFLOP/s",
                          "frac": round(flops / wall / 1e12 / 2500.0, 4), "flops_per_prompt": int(flops)}}))


def bench_serve(args, wl, dk, W, np, torch):
    """The scheduler end to end: C requests submitted at once, run until all are done."""
    shape, C, P, NEW, STEM = wl.cfg, args.serve, 512, 128, 256
    assert 1 <= C <= 64
    weights = make_model_weights(args, W, shape, wl.seed_weights)
    dm = dk.DeviceModel(shape, weights)
    per_seq = (P + NEW + 15) // 16 + 1
    n_blocks = C * per_seq + 64
    nbytes = dk.kv_pool_bytes(dm.cfg, n_blocks, 16)
    pool_t = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    pool = dk.create_kv_pool(dm.cfg, n_blocks, 16, pool_t, nbytes)
    cfg = dk.EngineConfig(C, per_seq, 64, 1)
    need = dk.engine_device_bytes(dm.handle, cfg)
    arena = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(wl.seed_tokens)
    stem = rng.integers(0, shape.vocab, size=STEM)
    prompts = [np.concatenate([stem, rng.integers(0, shape.vocab, size=P - STEM)]).astype(np.int32) for _ in range(C)]

    def run():
        eng = dk.engine_create(dm.handle, pool, cfg, (arena.data_ptr() + 255) // 256 * 256, need)
        if args.sampled:
            dk.engine_set_sampling(eng, 0.8, 50, 0.9, seed=7)
        ids = [dk.engine_submit(eng, p, NEW) for p in prompts]
        t0 = time.perf_counter()
        dk.engine_step(eng)                      # admission: prefix lookup + prefill of all C prompts, first decode step
        t1 = time.perf_counter()
        while dk.engine_step(eng) > 0:
            pass
        t2 = time.perf_counter()
        st = dk.engine_stats(eng)
        assert all(dk.engine_poll(eng, i)[1] == "done" for i in ids)
        dk.engine_destroy(eng)
        return t1 - t0, t2 - t1, st

    run()                                        # warm-up
    admit_s, gen_s, st = run()
    gen_tokens = st["generated_tokens"] - 2 * C  # tokens of the steady decode phase (after the first iteration)
    print(json.dumps({
        "metric": "engine_aggregate_decode_tok_per_s", "value": round(gen_tokens / gen_s, 1), "unit": "tok/s",
        "n_gpus": 1, "higher_is_better": True, "dtype": dtype_name(args), "data": "synthetic (seeded random-init weights)",
        "config": {"workload": f"{shape.name}: {C} concurrent requests, {P}-token prompts sharing a {STEM}-token "
                               f"stem, {NEW} new tokens each, continuous batching with prefix cache"
                               + (", sampled (temperature 0.8, top-k 50, top-p 0.9)" if args.sampled else ", greedy"),
                   "concurrency": C},
        "ms_per_decode_iteration": round(gen_s * 1e3 / max(1, st["decode_steps"] - 1), 4),
        "admission_ms": round(admit_s * 1e3, 2),
        "prefill_tokens": st["prefill_tokens"], "reused_prompt_tokens": st["reused_tokens"],
        "whole_run_tok_per_s": round(st["generated_tokens"] / (admit_s + gen_s), 1),
        "paper_context": "paper: 4.3x aggregate throughput at 16 concurrent requests vs 1 (Apple M4 Max); "
                         "other hardware, context only"}))
    dk.destroy_kv_pool(pool)


def bench_ttft(args, wl, dk, W, np, torch):
    """Time to first token of a prompt whose 512-token prefix is / is not in the prefix cache."""
    shape, PREFIX, OWN = wl.cfg, 512, 32
    weights = make_model_weights(args, W, shape, wl.seed_weights)
    dm = dk.DeviceModel(shape, weights)
    per_seq = (PREFIX + OWN + 15) // 16 + 2
    n_blocks = 16 * per_seq
    nbytes = dk.kv_pool_bytes(dm.cfg, n_blocks, 16)
    pool_t = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    pool = dk.create_kv_pool(dm.cfg, n_blocks, 16, pool_t, nbytes)
    cfg = dk.EngineConfig(1, per_seq, 64, 1)
    need = dk.engine_device_bytes(dm.handle, cfg)
    arena = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(wl.seed_tokens)
    miss, hit = [], []
    for rep in range(6):                                  # the first repetition warms up
        eng = dk.engine_create(dm.handle, pool, cfg, (arena.data_ptr() + 255) // 256 * 256, need)
        prefix = rng.integers(0, shape.vocab, size=PREFIX)
        for out in (miss, hit):                           # same prefix twice: the second finds it cached
            prompt = np.concatenate([prefix, rng.integers(0, shape.vocab, size=OWN)]).astype(np.int32)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            rid = dk.engine_submit(eng, prompt, 1)
            dk.engine_step(eng)                           # returns when the first token is on the host
            dt = time.perf_counter() - t0
            toks, state, reused = dk.engine_poll(eng, rid)
            assert state == "done" and len(toks) == 1 and reused == (PREFIX if out is hit else 0)
            if rep:
                out.append(dt)
        dk.engine_destroy(eng)
    m, h = float(np.median(miss)), float(np.median(hit))
    print(json.dumps({
        "metric": "ttft_ms", "value": round(h * 1e3, 3), "unit": "ms", "higher_is_better": False, "n_gpus": 1,
        "dtype": dtype_name(args), "data": "synthetic (seeded random-init weights)",
        "config": {"workload": f"{shape.name}: {PREFIX}-token shared prefix + {OWN} own tokens, first token, "
                               f"through the engine (prefix cache hit vs miss)"},
        "ttft_miss_ms": round(m * 1e3, 3), "ttft_hit_ms": round(h * 1e3, 3), "speedup": round(m / h, 2),
        "paper_context": "paper: 245 ms -> 42 ms (5.8x) on Qwen3-4B, 4-bit, Apple M4 Max; other hardware and "
                         "model, context only"}))
    dk.destroy_kv_pool(pool)


def measure_decode(args, wl, dk, W, np, torch, steps, warmup, ceiling=None):
    """Times `steps` decode steps of a workload (inputs resident in HBM beforehand; wall clock around
    the timed steps with a device synchronisation on both sides, HIP events on the launch stream for
    the device time), then profiles a few more steps kernel by kernel.  Returns everything the
    report needs; the model stays alive in the result for follow-up measurements."""
    from workloads.blocktable import layout_for
    shape, lay = wl.cfg, layout_for(wl)
    weights = make_model_weights(args, W, shape, wl.seed_weights)
    router_bytes = shape.n_layers * shape.n_experts * shape.hidden * 2    # routers stay bf16
    weight_bytes = shape.dense_weight_bytes()                             # attention, dense MLP, lm_head, routers
    one_expert_bytes = shape.expert_bytes()
    if args.weights == "q4":
        def q4(b):                                                        # 4 bits + (scale, bias) per 64 weights
            return b // 4 + b // 128 * 4
        weight_bytes = q4(weight_bytes - router_bytes) + router_bytes
        one_expert_bytes = q4(one_expert_bytes)
    pool_bits = W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False)
    tokens0 = W.initial_tokens(shape, wl.batch, wl.seed_tokens)

    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool_bits)
    dec = dk.Decoder(dm, dkv, lay.contexts, tokens0, want_logits=True)
    d_ctx0 = dec.seq_lens.clone()
    d_tok0 = dec.tokens.clone()
    span = wl.steps                              # tokens of growth the block tables have room for

    path_flag = dk.STEP_NO_FUSED if args.kernel_per_stage else 0

    def restart():
        dec.seq_lens.copy_(d_ctx0)
        dec.tokens.copy_(d_tok0)

    def run(n):
        for i in range(n):
            if i % span == 0:
                restart()                        # back to the initial context (tables are sized for `span` steps)
            dec.step(flags=dk.STEP_ADVANCE | path_flag)   # greedy: the step feeds its token to the next one

    run(warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    run(steps)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = e0.elapsed_time(e1)

    ms_per_step = wall * 1e3 / steps
    tok_s = wl.batch * steps / wall

    # per-kernel times: a few more steps with start/stop events on every launch
    prof_steps = min(16, span)
    dk.profile_read(dm.handle, reset=True)
    restart()
    for _ in range(prof_steps):
        dec.step(flags=dk.STEP_ADVANCE | dk.STEP_PROFILE | path_flag)
    prof = dk.profile_read(dm.handle, reset=True)

    # algorithmic bytes of a step at the mean context of the timed steps
    n_in_span = min(steps, span)
    mean_ctx = (lay.contexts + (n_in_span - 1) // 2).astype(np.int32)
    distinct = None
    if shape.n_experts:
        routing = dec.routing()                                  # last profiled step
        distinct = np.array([len(np.unique(routing[l])) for l in range(shape.n_layers)], dtype=np.int32)
    alg_bytes = dk.step_algorithmic_bytes(dm.handle, dkv.handle, lay.tables, mean_ctx, with_logits=True,
                                          distinct_experts_per_layer=distinct)
    kv_bytes = dk.step_algorithmic_bytes(dm.handle, dkv.handle, lay.tables, mean_ctx, with_logits=False,
                                         distinct_experts_per_layer=distinct) \
        - weight_bytes - wl.batch * shape.hidden * 2 \
        - (int(distinct.sum()) * one_expert_bytes if distinct is not None else 0)
    expert_bytes = int(distinct.sum()) * one_expert_bytes if distinct is not None else 0
    class_bytes = {"gemv": weight_bytes - router_bytes, "gemm": weight_bytes - router_bytes,
                   "attention": kv_bytes, "moe_expert": expert_bytes, "moe_router": router_bytes,
                   "fused_step": alg_bytes}      # the persistent kernel is the whole step
    step_dev_s = dev_ms * 1e-3 / steps
    achieved_step = alg_bytes / step_dev_s / 1e9
    if ceiling is None:
        ceiling = read_ceiling(dk, torch)
    kernels = {}
    for k, (ms, cnt) in prof.items():
        if cnt:
            kernels[k] = {"launches_per_step": cnt // prof_steps, "avg_us": round(ms * 1e3 / cnt, 3),
                          "us_per_step": round(ms * 1e3 / prof_steps, 2)}
    dominant = max(kernels, key=lambda k: kernels[k]["us_per_step"])
    dom = kernels[dominant]
    dom_bytes_per_launch = class_bytes.get(dominant, 0) / dom["launches_per_step"]
    achieved = dom_bytes_per_launch / (dom["avg_us"] * 1e-6) / 1e9
    traffic = None
    rev, measured = MEASURED_TRAFFIC.get((wl.name, dominant), (None, None))
    if rev is not None and rev in dk.version() and args.weights == "bf16":   # counters were taken with bf16 weights
        traffic = measured

    return {"shape": shape, "lay": lay, "weights": weights, "pool_bits": pool_bits, "tokens0": tokens0, "dm": dm,
            "dkv": dkv, "dec": dec, "span": span, "ms_per_step": ms_per_step, "tok_s": tok_s, "alg_bytes": alg_bytes,
            "step_dev_s": step_dev_s, "achieved_step": achieved_step, "ceiling": ceiling, "kernels": kernels,
            "dominant": dominant, "dom": dom, "dom_bytes_per_launch": dom_bytes_per_launch, "achieved": achieved,
            "traffic": traffic, "distinct": distinct}


def extra_workload(args, name, dk, W, np, torch, ceiling):
    """A batch-16 workload of the task's list, timed like the headline one and reported compactly."""
    import gc
    wl = W.WORKLOADS[name]
    steps = min(args.steps, wl.steps)
    m = measure_decode(args, wl, dk, W, np, torch, steps, min(args.warmup, 8), ceiling)
    out = {"workload": f"{wl.name}: {m['shape'].name} decode, batch {wl.batch}, context "
                       f"{int(m['lay'].contexts.min())}..{int(m['lay'].contexts.max())} growing"
                       + (f", {wl.n_sharers} rows sharing a {wl.shared_prefix}-token prefix" if wl.n_sharers else ""),
           "value": round(m["tok_s"], 2), "unit": "tok/s", "steps": steps, "ms_per_step": round(m["ms_per_step"], 5),
           "algorithmic_bytes_per_step": int(m["alg_bytes"]),
           "step_frac": round(m["achieved_step"] / HBM_PEAK_GBS, 4), "step_achieved_GBs": round(m["achieved_step"], 1),
           "dominant_kernel": m["dominant"], "dominant_avg_launch_us": m["dom"]["avg_us"],
           "dominant_launches_per_step": m["dom"]["launches_per_step"],
           "dominant_algorithmic_bytes_per_launch": int(m["dom_bytes_per_launch"]),
           "dominant_frac": round(m["achieved"] / HBM_PEAK_GBS, 4),
           "kernels_us_per_step": {k: v["us_per_step"] for k, v in m["kernels"].items()}}
    if m["distinct"] is not None:
        out["distinct_experts_per_layer_mean"] = round(float(m["distinct"].mean()), 2)
    m["dkv"].close()
    m["dm"].close()
    m.clear()
    gc.collect()
    torch.cuda.empty_cache()
    return out


STAMP_NAMES = ("layer begins", "q|k|v rows handed over", "q|k|v of the attention item arrived", "chunk attention done",
               "merged attention output handed over (collecting blocks)", "attention output arrived",
               "x_mid rows handed over", "x_mid arrived", "activations handed over", "activations arrived",
               "x_out rows handed over", "next layer's input arrived")


def bench_stage_stamps(args, wl, dk, W, np, torch):
    """Where a layer of the persistent step kernel spends its time: every block stamps the device's
    100 MHz clock at the stage boundaries of one layer (dk_debug_set_stage_stamps); reported per
    boundary as microseconds since the earliest block began the layer - median, earliest and latest
    block - averaged over the timed steps."""
    from workloads.blocktable import layout_for
    shape, lay = wl.cfg, layout_for(wl)
    weights = make_model_weights(args, W, shape, wl.seed_weights)
    pool_bits = W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False)
    tokens0 = W.initial_tokens(shape, wl.batch, wl.seed_tokens)
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool_bits)
    dec = dk.Decoder(dm, dkv, lay.contexts, tokens0, want_logits=True)
    ctx0, tok0 = dec.seq_lens.clone(), dec.tokens.clone()
    n_blocks = torch.cuda.get_device_properties(0).multi_processor_count
    stamps = torch.zeros((n_blocks, dk.STAGE_STAMPS), dtype=torch.int64, device="cuda")
    layer = args.stamps
    for _ in range(args.warmup):
        dec.step(flags=dk.STEP_ADVANCE)
    torch.cuda.synchronize()
    if dec.fused_status() is None:
        print("bench.py --stamps: this workload does not run as the persistent kernel", file=sys.stderr)
        sys.exit(2)
    dk.debug_set_stage_stamps(dm.handle, layer, stamps)
    n = len(STAMP_NAMES)
    acc = np.zeros((3, n))
    step_names = ("kernel entry", "first layer begins", "lm_head begins", "lm_head rows streamed")
    acc_step = np.zeros((3, 4))
    steps = min(args.steps, wl.steps - 1)
    dec.seq_lens.copy_(ctx0)
    dec.tokens.copy_(tok0)
    for _ in range(steps):
        stamps.zero_()
        dec.step(flags=dk.STEP_ADVANCE)
        torch.cuda.synchronize()
        raw = stamps.cpu().numpy().astype(np.float64)
        t = raw[:, :n]
        t0 = t[:, 0].min()
        ts = raw[:, 12:16]
        ts0 = ts[:, 0].min()
        for i in range(4):
            acc_step[:, i] += ((np.median(ts[:, i]) - ts0) / 100.0, (ts[:, i].min() - ts0) / 100.0, (ts[:, i].max() - ts0) / 100.0)
        for i in range(n):
            col = t[:, i][t[:, i] > 0]                        # blocks that reached the boundary
            acc[:, i] += ((np.median(col) - t0) / 100.0, (col.min() - t0) / 100.0, (col.max() - t0) / 100.0)
    dk.debug_set_stage_stamps(dm.handle, 0, None)
    acc /= steps
    acc_step /= steps
    out = {"metric": "persistent_kernel_stage_stamps_us", "workload": wl.name, "layer": layer, "steps": steps,
           "blocks": int(n_blocks), "unit": "us since the first block began the layer",
           "boundaries": [{"boundary": STAMP_NAMES[i], "median": round(acc[0, i], 2), "earliest": round(acc[1, i], 2),
                           "latest": round(acc[2, i], 2)} for i in range(n)],
           "step": [{"boundary": step_names[i], "median": round(acc_step[0, i], 2), "earliest": round(acc_step[1, i], 2),
                     "latest": round(acc_step[2, i], 2)} for i in range(4)]}
    print(json.dumps(out))


def bench_sample(args, wl, dk, W, np, torch):
    """The sampler on synthetic logits (seeded normal, standard deviation 2.5) of the workload's vocabulary:
    microseconds per call of dk_sample_tokens on `--sample` rows, for four settings."""
    shape = wl.cfg
    B, V = args.sample, shape.vocab
    rng = np.random.default_rng(1)
    logits = torch.from_numpy((rng.normal(size=(B, V)) * 2.5).astype(np.float32)).cuda()
    scratch = torch.empty(dk.sample_scratch_bytes(B, V), dtype=torch.uint8, device="cuda")
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    settings = []
    for top_k, top_p in ((0, 1.0), (50, 1.0), (0, 0.9), (50, 0.9)):
        for i in range(args.warmup):
            dk.sample_tokens(logits, 0.8, top_k, top_p, 7, i, scratch, out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            dk.sample_tokens(logits, 0.8, top_k, top_p, 7, i, scratch, out)
        e1.record()
        torch.cuda.synchronize()
        settings.append({"top_k": top_k, "top_p": top_p, "us_per_call": round(e0.elapsed_time(e1) * 1e3 / args.steps, 2)})
    print(json.dumps({"metric": "sampler_us_per_call", "unit": "us", "rows": B, "vocab": V, "temperature": 0.8,
                      "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "settings": settings}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="default run only: skip the batch-16 workloads cfg2 / cfg3 / cfg4_l4 reported beside cfg1")
    ap.add_argument("--prefill", type=int, default=0, metavar="P",
                    help="measure chunked prefill instead: a P-token prompt of the workload's model shape "
                         "into an empty cache, 64 tokens per chunk (one step = one whole prompt)")
    ap.add_argument("--serve", type=int, default=0, metavar="C",
                    help="measure the continuous-batching engine instead: C concurrent requests of the "
                         "workload's model shape (512-token prompts with a shared 256-token stem, 128 new tokens)")
    ap.add_argument("--sampled", action="store_true",
                    help="with --serve: tokens drawn by the sampler (temperature 0.8, top-k 50, top-p 0.9) instead of greedy")
    ap.add_argument("--ttft", action="store_true",
                    help="measure time to first token through the engine with and without a prefix-cache hit "
                         "(512-token shared prefix + 32 own tokens, the shape of the paper's text prefix-cache table)")
    ap.add_argument("--weights", choices=("bf16", "q4"), default="bf16",
                    help="q4: the projections and the lm_head as 4-bit group-wise affine codes (groups of 64 "
                         "columns, bf16 scale and bias), the precision the paper benchmarks; dense workloads")
    ap.add_argument("--stamps", type=int, default=-1, metavar="L",
                    help="instead of timing steps: where layer L of the persistent step kernel spends its time "
                         "(device clock stamps of every block at the stage boundaries)")
    ap.add_argument("--sample", type=int, default=0, metavar="B",
                    help="measure the sampler (dk_sample_tokens) instead: B rows of logits over the workload's "
                         "vocabulary, temperature 0.8, with and without top-k 50 and top-p 0.9")
    ap.add_argument("--kernel-per-stage", action="store_true",
                    help="never take the single persistent kernel (small batches of small dense models)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    from workloads.blocktable import layout_for
    import paper_2601_19139_amd as dk

    dk.lib()                                    # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a HIP device"
    torch.cuda.set_device(0)

    wl = W.WORKLOADS[args.workload]
    if args.prefill:
        return bench_prefill(args, wl, dk, W, np, torch)
    if args.serve:
        return bench_serve(args, wl, dk, W, np, torch)
    if args.ttft:
        return bench_ttft(args, wl, dk, W, np, torch)
    if args.stamps >= 0:
        return bench_stage_stamps(args, wl, dk, W, np, torch)
    if args.sample:
        return bench_sample(args, wl, dk, W, np, torch)
    m = measure_decode(args, wl, dk, W, np, torch, args.steps, args.warmup)
    shape, lay, weights, pool_bits, tokens0, dm = (m[k] for k in ("shape", "lay", "weights", "pool_bits", "tokens0", "dm"))
    span, ms_per_step, tok_s, alg_bytes, step_dev_s = (m[k] for k in ("span", "ms_per_step", "tok_s", "alg_bytes", "step_dev_s"))
    achieved_step, ceiling, kernels, dominant, dom = (m[k] for k in ("achieved_step", "ceiling", "kernels", "dominant", "dom"))
    dom_bytes_per_launch, achieved, traffic, distinct = (m[k] for k in ("dom_bytes_per_launch", "achieved", "traffic", "distinct"))

    out = {
        "metric": "aggregate_decode_tok_per_s",
        "value": round(tok_s, 2),
        "unit": "tok/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype_name(args),
        "data": "synthetic (seeded random-init weights and KV of the named shape)",
        "config": {"workload": f"{wl.name}: {shape.name} decode, batch {wl.batch}, "
                               f"context {int(lay.contexts.min())}..{int(lay.contexts.max())} growing, "
                               f"block 16, greedy" + (", 4-bit weights" if args.weights == "q4" else ""),
                   "batch": wl.batch, "layers": shape.n_layers, "hidden": shape.hidden,
                   "vocab": shape.vocab},
        # the kernel class that takes most of the step; achieved = its algorithmic
        # bytes per launch / its mean launch duration (start/stop events per launch)
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel": dominant, "launches_per_step": dom["launches_per_step"],
                     "avg_launch_us": dom["avg_us"],
                     "algorithmic_bytes_per_launch": int(dom_bytes_per_launch),
                     # the same against what a plain read-only streaming kernel reaches on this device
                     "measured_read_ceiling": round(ceiling, 1), "frac_of_ceiling": round(achieved / ceiling, 4)},
        # the whole step (every launch): algorithmic bytes / device time of the timed region
        "step_roofline": {"achieved": round(achieved_step, 1), "frac": round(achieved_step / HBM_PEAK_GBS, 4),
                          "frac_of_ceiling": round(achieved_step / ceiling, 4),
                          "unit": "GB/s", "algorithmic_bytes_per_step": int(alg_bytes),
                          "device_ms_per_step": round(step_dev_s * 1e3, 5)},
        "kernels": kernels,
        "paper_context": "paper: up to 525 tok/s on Qwen3-0.6B (4-bit, Apple M4 Max, 546 GB/s); other hardware, not a target",
    }
    if distinct is not None:
        out["distinct_experts_per_layer_mean"] = round(float(distinct.mean()), 2)
    if wl.batch == 1 and wl.contexts:
        out["batch16"] = batch16_line(args, wl, dk, W, np, torch, dm, tok_s)
    if args.workload == "cfg1" and args.weights == "bf16" and not args.kernel_per_stage and not args.no_extra:
        # the batch-16 half of the metric on the task's batch-16 workloads (cfg4_l4: the 30B-A3B
        # mixture-of-experts shape cut to 4 layers, every kernel at its real size, 5 GB instead of 61)
        import gc
        m["dkv"].close()
        del m["dec"], m["dkv"]
        gc.collect()
        torch.cuda.empty_cache()
        for name in ("cfg2", "cfg3", "cfg4_l4"):
            out[name] = extra_workload(args, name, dk, W, np, torch, ceiling)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, weights, lay, pool_bits, tokens0,
                                           max_steps=min(64, span - 1))   # the tables have room for `span` tokens
    print(json.dumps(out))


if __name__ == "__main__":
    main()
