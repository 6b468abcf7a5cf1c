"""Writes tests/golden/cfg0_oracle.json and cfg0_q4_oracle.json from the CPU oracle alone.

Run:  python tests/golden/make_golden.py
Each file stores the oracle's greedy tokens and a few logits for a tiny
workload (cfg0: 2 sequences, contexts 32 and 17, 8 free-running greedy steps;
cfg0_q4: 5 sequences with 4-bit weights made by workloads/quant.py, 6 steps).  The
paper prints no worked numeric example, so this is not a pin of the oracle; it
is a drift detector (any later change to the oracle's arithmetic shows up) and
a fixture whose every value comes from oracle/ only.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as W                      # noqa: E402
from workloads.blocktable import layout_for   # noqa: E402
from oracle import oracle_f64              # noqa: E402


def write(name, q4):
    orc = oracle_f64()
    wl = W.WORKLOADS[name]
    cfg, lay = wl.cfg, layout_for(wl)
    w = W.make_weights(cfg, wl.seed_weights)
    if q4:
        from workloads.quant import quantize_weights
        w = quantize_weights(w)
    step = orc.decode_step_q4 if q4 else orc.decode_step
    pool = W.fill_kv_pool(cfg, lay, wl.seed_kv)
    tok = W.initial_tokens(cfg, wl.batch, wl.seed_tokens)
    sl = lay.contexts.copy()
    steps = []
    for s in range(wl.steps):
        r = step(cfg, w, pool, wl.block_size, lay.tables, sl, tok)
        steps.append({
            "tokens_in": [int(t) for t in tok],
            "next": [int(t) for t in r["next"]],
            "logits_0_8": [[float(np.float32(v)) for v in r["logits"][b, :8]] for b in range(wl.batch)],
            "logits_l2": [float(np.linalg.norm(r["logits"][b].astype(np.float64))) for b in range(wl.batch)],
        })
        tok, sl = r["next"], sl + 1
    out = {"workload": name, "source": "oracle/decode_oracle.c (double build)", "steps": steps}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), f"{name}_oracle.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    write("cfg0", False)
    write("cfg0_q4", True)
