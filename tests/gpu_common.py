"""Helpers for the GPU parity tests: run the HIP path and the CPU oracle on
the same seeded inputs and compare."""
import numpy as np

import workloads as W


# Router near-ties.  An expert set of the kernel that differs from the oracle's own is accepted as
# the oracle's choice for that (layer, row) only if it is a valid top-k set up to this relative
# margin of the probabilities (oracle/decode_oracle.c, orc_tie).  Derivation: a router logit is a
# dot product of the normalised residual (relative error of the float32 path up to ~1.5e-4 after
# dozens of layers: the measured worst logits rel-L2) with a row of magnitude ~1, so two logits'
# difference is off by ~2e-4 (one sigma); a probability ratio moves by the same amount.  1e-3 is
# five sigma of that.  A wrong router (a dropped term, a wrong row) misses by orders of magnitude more.
TIE_TOL = 1e-3


def rel_l2(got, ref):
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    return np.linalg.norm(got - ref, axis=-1) / np.linalg.norm(ref, axis=-1)


def bf16_close(a_bits, b_bits, drift=1e-4):
    """True where two stored bf16 values agree up to rounding: the float32
    values they were rounded from differ by at most `drift` of the largest
    magnitude (1e-4: ten times the measured error of a short run; a run whose
    logits have drifted further from the oracle's passes a bound in proportion),
    and rounding adds at most one bf16 step (2^-7 relative) on top of that."""
    a = W.f32_from_bf16_bits(a_bits).astype(np.float64)
    b = W.f32_from_bf16_bits(b_bits).astype(np.float64)
    floor = drift * max(float(np.abs(b).max()), 1e-30)
    return np.abs(a - b) <= 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + floor


def run_both(orc, shape, weights, layout, pool_bits, tokens, steps, teacher_forced=True,
             want_pool=True, gpu_flags=0):
    """Runs `steps` decode steps on the GPU and in the oracle.

    teacher_forced: the GPU is fed the oracle's tokens at every step (the graded
    mode).  Returns a dict of per-step logits / tokens from both and the final
    pools."""
    import torch
    import paper_2601_19139_amd as dk
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, layout, pool_bits)
    opool = pool_bits.copy()
    sl = layout.contexts.copy().astype(np.int32)
    otok = np.asarray(tokens, dtype=np.int32).copy()
    dec = dk.Decoder(dm, dkv, sl, otok)
    out = {"gpu_logits": [], "orc_logits": [], "gpu_next": [], "orc_next": [],
           "gpu_experts": [], "orc_experts": []}
    for s in range(steps):
        dk.kv_validate_tables(dkv.handle, layout.tables, sl)
        # a 4-bit model (matrices given as q / scale / bias) takes the oracle's 4-bit step
        step = orc.decode_step_q4 if isinstance(weights["lm_head"], dict) else orc.decode_step
        r = step(shape, weights, opool, layout.block_size, layout.tables, sl, otok,
                 want_trace=bool(shape.n_experts))
        dec.step(flags=gpu_flags)
        torch.cuda.synchronize()
        if shape.n_experts:
            out["gpu_experts"].append(dec.routing())
            out["orc_experts"].append(r["experts"])
        out["gpu_logits"].append(dec.logits.cpu().numpy().copy())
        out["gpu_next"].append(dec.next.cpu().numpy().copy())
        out["orc_logits"].append(r["logits"])
        out["orc_next"].append(r["next"])
        sl = sl + 1
        otok = r["next"]
        if gpu_flags & dk.STEP_ADVANCE:
            # the kernel advanced its own state (free running)
            assert np.array_equal(dec.seq_lens.cpu().numpy(), sl)
            assert np.array_equal(dec.tokens.cpu().numpy(), out["gpu_next"][-1])
        if teacher_forced or not (gpu_flags & dk.STEP_ADVANCE):
            dec.seq_lens.copy_(torch.from_numpy(sl))
            nxt = otok if teacher_forced else out["gpu_next"][-1]
            dec.tokens.copy_(torch.from_numpy(np.ascontiguousarray(nxt)))
    out["fused_status"] = dec.fused_status()
    if want_pool:
        out["gpu_pool"] = dkv.bits().reshape(pool_bits.shape)
        out["orc_pool"] = opool
    dkv.close()
    dm.close()
    return out


def check_parity(out, tol=1e-2, min_agree=0.99):
    """The bar: relative L2 of the logits <= tol for every row of every step
    (the stated tolerance of the decode path), greedy agreement >= min_agree."""
    # the persistent step kernel (when it ran) must never have given up a wait
    assert out.get("fused_status") in (None, (0, 0)), f"persistent step kernel timed out: {out['fused_status']}"
    worst, agree, total = 0.0, 0, 0
    for gl, ol, gn, on in zip(out["gpu_logits"], out["orc_logits"], out["gpu_next"], out["orc_next"]):
        assert np.all(np.isfinite(gl))
        worst = max(worst, float(rel_l2(gl, ol).max()))
        agree += int((gn == on).sum())
        total += gn.size
    assert worst <= tol, f"logits relative L2 {worst:.3e} > {tol}"
    assert agree >= min_agree * total, f"greedy agreement {agree}/{total}"
    return worst, agree / total


def parity_stats(out):
    """Count of compared tokens, worst and mean relative L2 of the logits and the
    teacher-forced greedy agreement of a run_both / run_sampled result."""
    errs = np.concatenate([rel_l2(g, o).reshape(-1) for g, o in zip(out["gpu_logits"], out["orc_logits"])])
    same = sum(int((g == o).sum()) for g, o in zip(out["gpu_next"], out["orc_next"]))
    return {"tokens": int(errs.size), "worst": float(errs.max()), "mean": float(errs.mean()),
            "agree": same / errs.size}


def free_running_report(free_next, orc_next, rows=None):
    """The GPU decoding on its own tokens against the oracle decoding on its own:
    fraction of equal tokens over the compared steps and the first step at which
    any compared row differs (None: never).  Reported, not graded: one flipped
    near-tie changes everything after it."""
    n = min(len(free_next), len(orc_next))
    g = np.stack([np.asarray(f)[list(rows)] if rows is not None else np.asarray(f) for f in free_next[:n]])
    o = np.stack([np.asarray(x) for x in orc_next[:n]])
    differs = np.nonzero((g != o).any(axis=1))[0]
    return float((g == o).mean()), (int(differs[0]) if differs.size else None)


def progress(line):
    """A sign of life for long tests: appended to a file in the results folder of a GPU run (a
    harness that watches for silence sees the file grow; pytest holds printed output back)."""
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        with open(os.path.join(root, "gpurun_out", "test_progress.txt"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def log_result(line):
    """Prints a result line and, where the results folder of a GPU run exists or can be made,
    appends it there (pytest shows captured output only for failing tests)."""
    import os
    print(line, flush=True)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        with open(os.path.join(root, "gpurun_out", "parity_full_size.txt"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def check_pool(out, pool_before, shape, layout, steps, max_flips=0.02):
    """Appends must land at exactly the oracle's offsets; values may differ by
    the bf16 rounding of nearly equal float32 numbers (<= 1 step, rarely).

    How rarely: two float32 computations of the same k or v element that differ
    by a relative delta round to different bf16 neighbours with probability about
    delta / 2^-8.  A short run has delta ~ 1e-5 (0.3 %: the default bound of 2 %
    is generous); a run that has attended to more than a hundred of its own
    appended tokens reaches delta ~ 1e-4, i.e. a few per cent, and passes its own
    bound.  Returns the fraction that differed."""
    g, o = out["gpu_pool"], out["orc_pool"]
    g_changed = g != pool_before
    o_changed = o != pool_before
    # every slot the oracle wrote was poison before, so "changed" = "written"
    assert np.array_equal(g_changed, o_changed), "append addressing differs from the oracle"
    assert int(o_changed.sum()) == shape.n_layers * layout.tables.shape[0] * 2 * shape.kv_dim * steps
    assert bf16_close(g[o_changed], o[o_changed]).all(), "appended value differs by more than rounding"
    flips = float((g[o_changed] != o[o_changed]).mean())
    assert flips < max_flips, f"{flips:.4f} of the appended values differ by a rounding step"
    return flips


def run_sampled(orc, shape, weights, layout, pool_bits, tokens, steps, rows, free_steps=0, tie_tol=0.0):
    """Full-size variant: the GPU runs the whole batch, the oracle only the
    sampled `rows` (rows of a batch do not interact, so a row's result does not
    depend on which other rows are computed).  Sampled rows are teacher-forced
    with the oracle's tokens; the others follow the GPU's own tokens.

    Returns per-step logits/tokens of the sampled rows from both sides, the GPU
    pool, and the oracle pool (which holds only the sampled rows' appends).
    tie_tol > 0 (mixture-of-experts models): see TIE_TOL.
    free_steps > 0: the GPU also decodes that many steps from the same start on
    its own tokens (the step advancing tokens and lengths on the device), all
    rows, into a second copy of the pool: out["free_next"][step] = tokens [B]."""
    import torch
    import paper_2601_19139_amd as dk
    rows = list(rows)
    progress(f"{shape.name}: uploading weights")
    dm = dk.DeviceModel(shape, weights)
    dkv = dk.DeviceKV(dm, layout, pool_bits)
    opool = pool_bits.copy()
    sl = layout.contexts.copy().astype(np.int32)
    tok = np.asarray(tokens, dtype=np.int32).copy()
    dec = dk.Decoder(dm, dkv, sl, tok)
    out = {"gpu_logits": [], "orc_logits": [], "gpu_next": [], "orc_next": [], "ties": [], "tie_refused": []}
    q4 = isinstance(weights["lm_head"], dict)
    for s in range(steps):
        dk.kv_validate_tables(dkv.handle, layout.tables, sl)
        dec.step()
        torch.cuda.synchronize()
        if tie_tol and shape.n_experts and not q4:
            # the router's top-k is an integer decided by floating point: the kernel's expert sets go
            # to the oracle as proposals, which it adopts only where they are valid up to tie_tol
            prop = np.ascontiguousarray(dec.routing()[:, rows, :])
            r = orc.decode_step_tie(shape, weights, opool, layout.block_size, layout.tables[rows], sl[rows],
                                    tok[rows], prop, tie_tol)
            for l, i in zip(*np.nonzero(r["adopted"])):
                out["ties"].append((s, int(l), rows[i], float(r["margin"][l, i])))
            for l, i in zip(*np.nonzero((r["margin"] > tie_tol))):
                out["tie_refused"].append((s, int(l), rows[i], float(r["margin"][l, i])))
        else:
            step = orc.decode_step_q4 if q4 else orc.decode_step
            r = step(shape, weights, opool, layout.block_size, layout.tables[rows], sl[rows], tok[rows])
        progress(f"{shape.name}: oracle step {s + 1}/{steps} of rows {rows}")
        g_next = dec.next.cpu().numpy().copy()
        out["gpu_logits"].append(dec.logits[rows].cpu().numpy().copy())
        out["gpu_next"].append(g_next[rows])
        out["orc_logits"].append(r["logits"])
        out["orc_next"].append(r["next"])
        sl = sl + 1
        tok = g_next.copy()
        tok[rows] = r["next"]
        dec.seq_lens.copy_(torch.from_numpy(sl))
        dec.tokens.copy_(torch.from_numpy(tok))
    out["gpu_pool"] = dkv.bits().reshape(pool_bits.shape)
    out["orc_pool"] = opool
    dkv.close()
    if free_steps:
        out["free_next"] = free_run(dk, dm, layout, pool_bits, tokens, free_steps)
    dm.close()
    return out


def free_run(dk, dm, layout, pool_bits, tokens, steps):
    """`steps` decode steps on the GPU's own tokens (DK_STEP_ADVANCE): tokens per step [steps][B]."""
    import torch
    dkv = dk.DeviceKV(dm, layout, pool_bits)
    dec = dk.Decoder(dm, dkv, layout.contexts, np.asarray(tokens, dtype=np.int32), want_logits=False)
    got = []
    for _ in range(steps):
        dec.step(flags=dk.STEP_ADVANCE)
        got.append(dec.next.clone())
    torch.cuda.synchronize()
    assert np.array_equal(dec.seq_lens.cpu().numpy(), layout.contexts + steps)
    dkv.close()
    return [g.cpu().numpy() for g in got]


def check_pool_sampled(out, pool_before, shape, layout, steps, rows, drift=1e-4):
    """Addressing for every row against the closed-form slot list (block
    table entry T // 16, slot T % 16, every layer, K and V, every kv head);
    values of the sampled rows against the oracle's pool."""
    g, o = out["gpu_pool"], out["orc_pool"]
    bs = layout.block_size
    targets = {}                                     # block -> list of (slot, row)
    for b, T0 in enumerate(layout.contexts):
        for s in range(steps):
            T = int(T0) + s
            targets.setdefault(int(layout.tables[b, T // bs]), []).append((T % bs, b))
    untouched = np.ones(layout.num_blocks, dtype=bool)
    untouched[list(targets)] = False
    for l in range(shape.n_layers):                  # layer by layer keeps temporaries small
        assert np.array_equal(g[l][untouched], pool_before[l][untouched]), "a block no row appends to changed"
        for blk, lst in targets.items():
            slots = [sl for sl, _ in lst]
            other = [i for i in range(bs) if i not in slots]
            assert np.array_equal(g[l, blk][:, :, other, :], pool_before[l, blk][:, :, other, :])
            for sl_, b in lst:
                # poisoned beforehand, so a written slot holds no NaN pattern any more
                assert not np.any(g[l, blk, :, :, sl_, :] == W.BF16_NAN_BITS), "append slot not written"
                if b in rows:
                    ga, oa = g[l, blk, :, :, sl_, :], o[l, blk, :, :, sl_, :]
                    if not bf16_close(ga, oa, drift).all():
                        a = W.f32_from_bf16_bits(ga).astype(np.float64)
                        r = W.f32_from_bf16_bits(oa).astype(np.float64)
                        excess = (np.abs(a - r) - 2.0 ** -7 * np.maximum(np.abs(a), np.abs(r))).max() / np.abs(r).max()
                        raise AssertionError(f"layer {l} row {b} slot {sl_}: appended value off by a bf16 step plus "
                                             f"{excess:.2e} of the largest magnitude (allowed {drift:.1e})")
