#!/usr/bin/env python3
"""Decode-step benchmark on one MI355X.

A "step" is one call of the decode step over the whole batch: embedding,
every layer (q/k/v projection, head norm + rotary embedding + KV append,
ragged paged attention, output projection, SwiGLU MLP), final norm, lm_head
and greedy argmax - one new token for each of the B sequences.  Inputs
(weights, KV pool, block tables, tokens) are resident in HBM before the timed
region.  Prints one JSON line.

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


def cpu_baseline(shape, weights, layout, pool_bits, tokens, budget_s=12.0, max_steps=64):
    """The CPU oracle, as it stands, on the same workload: free-running greedy
    steps until about `budget_s` seconds have passed."""
    import numpy as np
    from oracle import oracle_f64
    orc = oracle_f64()
    pool = pool_bits.copy()
    sl = layout.contexts.copy()
    tok = np.asarray(tokens, dtype=np.int32).copy()
    orc.decode_step(shape, weights, pool, layout.block_size, layout.tables, sl, tok)   # warm-up
    sl, n, t0 = sl + 1, 0, time.perf_counter()
    while n < max_steps and time.perf_counter() - t0 < budget_s:
        r = orc.decode_step(shape, weights, pool, layout.block_size, layout.tables, sl, tok,
                            want_logits=False)
        tok, sl, n = r["next"], sl + 1, n + 1
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": round(n * len(tok) / dt, 3), "unit": "tok/s", "cores": threads,
            "kind": "oracle", "sample": f"{n} greedy steps of the same workload (fp64 C loops, OpenMP rows)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1", file=sys.stderr)
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
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool_bits = W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False)
    tokens0 = W.initial_tokens(shape, wl.batch, wl.seed_tokens)

    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, lay, pool_bits)
    dec = dk.Decoder(dm, dkv, lay.contexts, tokens0, want_logits=True)
    d_ctx0 = dec.seq_lens.clone()
    d_tok0 = dec.tokens.clone()
    span = wl.steps                              # tokens of growth the block tables have room for

    def restart():
        dec.seq_lens.copy_(d_ctx0)
        dec.tokens.copy_(d_tok0)

    def run(n):
        for i in range(n):
            if i % span == 0:
                restart()                        # back to the initial context (tables are sized for `span` steps)
            dec.step(flags=dk.STEP_ADVANCE)      # greedy: the step feeds its token to the next one

    run(args.warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    run(args.steps)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = e0.elapsed_time(e1)

    ms_per_step = wall * 1e3 / args.steps
    tok_s = wl.batch * args.steps / wall

    # algorithmic bytes of a step at the mean context of the timed steps
    n_in_span = min(args.steps, span)
    mean_ctx = (lay.contexts + (n_in_span - 1) // 2).astype(np.int32)
    alg_bytes = dk.step_algorithmic_bytes(dm.handle, dkv.handle, lay.tables, mean_ctx, with_logits=True)
    step_dev_s = dev_ms * 1e-3 / args.steps
    achieved = alg_bytes / step_dev_s / 1e9

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
        "dtype": "bf16 weights/KV, f32 accumulate",
        "data": "synthetic (seeded random-init weights and KV of the named shape)",
        "config": {"workload": f"{wl.name}: {shape.name} decode, batch {wl.batch}, "
                               f"context {int(lay.contexts.min())}..{int(lay.contexts.max())}+, "
                               f"block 16, greedy",
                   "batch": wl.batch, "layers": shape.n_layers, "hidden": shape.hidden,
                   "vocab": shape.vocab},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "decode step (all launches of one step)",
                     "algorithmic_bytes_per_step": int(alg_bytes),
                     "device_ms_per_step": round(step_dev_s * 1e3, 5)},
        "paper_context": "paper: up to 525 tok/s on Qwen3-0.6B (4-bit, Apple M4 Max, 546 GB/s); other hardware, not a target",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, weights, lay, pool_bits, tokens0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
