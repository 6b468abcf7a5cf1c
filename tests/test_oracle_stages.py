"""Pins for every stage of the CPU oracle (oracle/decode_oracle.c).

None of these re-types the oracle's formula: each checks a stage against a
closed form, an invariant, a brute-force enumeration, a hand-worked value or a
library routine (numpy / torch CPU in fp64), chosen so that a dropped term, a
wrong sign or index, or a transposed operand fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

import workloads as W

RNG = np.random.default_rng(1234)


def bits(a):
    return W.bf16_bits_from_f32(np.asarray(a, dtype=np.float32))


def vals(b):
    return W.f32_from_bf16_bits(b).astype(np.float64)


# ------------------------------------------------------------------ bf16 --
def test_bf16_roundtrip_matches_torch(orc):
    x = np.concatenate([
        RNG.standard_normal(4096).astype(np.float32) * 3,
        np.array([0.0, -0.0, 1.0, -1.0, 1e-30, 3e38, np.inf, -np.inf], dtype=np.float32),
        # exact ties: 1 + 2^-8 lies halfway between two bf16 values (even below),
        # 1 + 3*2^-8 halfway (even above)
        np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8, -(1 + 2 ** -8), 2 + 2 ** -7], dtype=np.float32),
    ])
    got = orc.f32_to_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # hand-worked ties: 1+2^-8 -> 1.0 (0x3F80), 1+3*2^-8 -> 1+2^-6 (0x3F82)
    assert got[-4] == 0x3F80 and got[-3] == 0x3F82
    back = orc.bf16_to_f32(got)
    want_back = torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).float().numpy()
    assert np.array_equal(back, want_back)
    # the input generator's own conversion agrees bit for bit
    assert np.array_equal(W.bf16_bits_from_f32(x), want)


# --------------------------------------------------------------- RMSNorm --
def test_rmsnorm_closed_forms(orc):
    n = 96
    ones = bits(np.ones(n))
    # constant vector c with unit gain: c / sqrt(c^2 + eps)
    c, eps = 3.0, 0.25
    out = orc.rmsnorm(np.full(n, c), ones, eps)
    assert np.allclose(out, c / math.sqrt(c * c + eps), rtol=1e-14)
    # mean square of the output is ms / (ms + eps)
    x = RNG.standard_normal(n)
    out = orc.rmsnorm(x, ones, eps)
    ms = np.mean(x * x)
    assert np.isclose(np.mean(out * out), ms / (ms + eps), rtol=1e-12)
    # scale invariance as eps -> 0, and sign preserved
    a = orc.rmsnorm(x, ones, 0.0)
    b = orc.rmsnorm(7.5 * x, ones, 0.0)
    assert np.allclose(a, b, rtol=1e-13)
    assert np.all(np.sign(a) == np.sign(x))
    # gain is applied elementwise (not summed, not shifted)
    g = bits(1 + 0.5 * RNG.standard_normal(n))
    assert np.allclose(orc.rmsnorm(x, g, eps), out * vals(g), rtol=1e-13)
    # the mean is over n, not a sum: doubling the vector by repetition keeps values
    x2 = np.concatenate([x, x])
    assert np.allclose(orc.rmsnorm(x2, bits(np.ones(2 * n)), eps)[:n], out, rtol=1e-13)


# ---------------------------------------------------------------- matvec --
def test_matvec_matches_numpy_and_orientation(orc):
    rows, cols = 37, 53
    Wb = bits(RNG.standard_normal((rows, cols)))
    x = RNG.standard_normal(cols)
    y = orc.matvec(Wb, x)
    assert np.allclose(y, vals(Wb) @ x, rtol=1e-12, atol=1e-13)
    # orientation: a unit vector picks a column of W
    e = np.zeros(cols)
    e[5] = 1.0
    assert np.array_equal(orc.matvec(Wb, e), vals(Wb)[:, 5])


# ------------------------------------------------------------------ RoPE --
def test_rope_hand_worked_and_invariants(orc):
    # d = 4, theta = 100: pairs (0,2) and (1,3); frequencies 1 and 100^(-1/2) = 0.1
    v = np.array([1.0, 2.0, 3.0, 4.0])
    out = orc.rope(v, pos=2, theta=100.0)
    a0, a1 = 2.0, 0.2
    want = np.array([1 * math.cos(a0) - 3 * math.sin(a0), 2 * math.cos(a1) - 4 * math.sin(a1),
                     3 * math.cos(a0) + 1 * math.sin(a0), 4 * math.cos(a1) + 2 * math.sin(a1)])
    assert np.allclose(out, want, rtol=1e-14)
    d = 64
    x = RNG.standard_normal(d)
    assert np.array_equal(orc.rope(x, 0, 1e4), x)                    # position 0 = identity
    assert np.isclose(np.linalg.norm(orc.rope(x, 977, 1e6)), np.linalg.norm(x), rtol=1e-13)
    # the inner product depends only on the position difference
    k = RNG.standard_normal(d)
    a = orc.rope(x, 40, 1e4) @ orc.rope(k, 13, 1e4)
    b = orc.rope(x, 40 + 500, 1e4) @ orc.rope(k, 13 + 500, 1e4)
    assert np.isclose(a, b, rtol=1e-10)
    # complex-number formulation: (x_i + i x_{i+d/2}) * exp(i pos theta^(-2i/d))
    z = (x[: d // 2] + 1j * x[d // 2:]) * np.exp(1j * 123 * 5e5 ** (-2.0 * np.arange(d // 2) / d))
    assert np.allclose(orc.rope(x, 123, 5e5), np.concatenate([z.real, z.imag]), rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------- softmax --
def test_softmax_rows_sum_to_one_and_shift_invariance(orc, orc32):
    s = RNG.standard_normal(301) * 10
    p = orc.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-12 and np.all(p > 0)
    assert abs(orc32.softmax(s).sum() - 1.0) < 1e-6
    assert np.allclose(orc.softmax(s + 1000.0), p, rtol=1e-9)        # max-subtracted: no overflow
    assert np.allclose(orc.softmax(np.full(7, 3.3)), 1 / 7)
    assert np.allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), rtol=1e-12)
    # ratio of two entries is exp of the score difference
    assert np.isclose(p[3] / p[9], math.exp(s[3] - s[9]), rtol=1e-12)


# ----------------------------------------------------------- pool layout --
def test_pool_offset_enumeration(orc):
    cfg = W.CONFIGS["tiny"]
    NB, bs = 5, 16
    shape = W.pool_shape(cfg, NB, bs)
    flat = np.arange(int(np.prod(shape)), dtype=np.int64).reshape(shape)
    seen = set()
    for idx in np.ndindex(*shape[:-1]):
        for dim in (0, 1, cfg.head_dim - 1):
            off = orc.pool_offset(cfg, NB, bs, *idx, dim)
            assert off == flat[idx + (dim,)]
            seen.add(off)
    assert len(seen) == int(np.prod(shape[:-1])) * 3
    # a (block, K|V, head) tile is one contiguous run of bs*d elements
    assert orc.pool_offset(cfg, NB, bs, 1, 3, 1, 1, bs - 1, cfg.head_dim - 1) - \
        orc.pool_offset(cfg, NB, bs, 1, 3, 1, 1, 0, 0) == bs * cfg.head_dim - 1


def test_append_changes_exactly_the_addressed_slots(orc):
    cfg = W.CONFIGS["tiny"]
    bs, NB = 16, 6
    pool = np.full(W.pool_shape(cfg, NB, bs), W.BF16_NAN_BITS, dtype=np.uint16)   # no value can collide
    before = pool.copy()
    table = np.array([4, 1, 5], dtype=np.int32)
    k = RNG.standard_normal(cfg.kv_dim)
    v = RNG.standard_normal(cfg.kv_dim)
    pos, layer = 37, 1                                  # block index 2 -> id 5, slot 5
    orc.append_kv(cfg, pool, bs, layer, table, pos, k, v)
    changed = np.argwhere(pool != before)
    assert len(changed) == 2 * cfg.kv_dim
    assert set(map(tuple, changed[:, :2])) == {(layer, 5)}
    assert set(changed[:, 4]) == {5}
    kb = bits(k).reshape(cfg.n_kv_heads, cfg.head_dim)
    vb = bits(v).reshape(cfg.n_kv_heads, cfg.head_dim)
    assert np.array_equal(pool[layer, 5, 0, :, 5, :], kb)
    assert np.array_equal(pool[layer, 5, 1, :, 5, :], vb)


# ------------------------------------------------------------- attention --
def _contiguous_kv(cfg, pool, bs, layer, table, n):
    """K, V of logical positions 0..n-1 gathered with numpy indexing: [nkv, n, d]."""
    K = np.stack([vals(pool[layer, table[t // bs], 0, :, t % bs, :]) for t in range(n)], 1)
    V = np.stack([vals(pool[layer, table[t // bs], 1, :, t % bs, :]) for t in range(n)], 1)
    return K, V


@pytest.mark.parametrize("model,n_tokens", [("tiny", 45), ("tiny", 16), ("qwen3_0p6b", 70)])
def test_attention_matches_torch_sdpa(orc, model, n_tokens):
    base = W.CONFIGS[model]
    cfg = W.ModelConfig(**{**base.as_dict(), "n_layers": 2, "vocab": 8})
    bs, NB = 16, 9
    pool = W.normal_bf16(11, "p", W.pool_shape(cfg, NB, bs))
    table = np.array([7, 2, 8, 0, 5], dtype=np.int32)
    q = RNG.standard_normal((cfg.n_q_heads, cfg.head_dim))
    out, probs = orc.attention(cfg, pool, bs, 1, table, n_tokens, q, want_probs=True)
    K, V = _contiguous_kv(cfg, pool, bs, 1, table, n_tokens)
    G = cfg.group
    Kq = torch.from_numpy(np.repeat(K, G, axis=0))      # [nq, n, d]: head h uses kv head h // G
    Vq = torch.from_numpy(np.repeat(V, G, axis=0))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[:, None, :], Kq, Vq)[:, 0, :].numpy()
    assert np.allclose(out, ref, rtol=1e-10, atol=1e-12)
    assert np.allclose(probs.sum(1), 1.0, atol=1e-12)   # softmax rows sum to 1


def test_attention_special_cases(orc):
    cfg = W.CONFIGS["tiny"]
    bs, NB = 16, 4
    pool = W.normal_bf16(12, "p", W.pool_shape(cfg, NB, bs))
    table = np.array([3, 1], dtype=np.int32)
    q = RNG.standard_normal((cfg.n_q_heads, cfg.head_dim))
    # single-token context returns that token's V row, per kv head, exactly
    out = orc.attention(cfg, pool, bs, 0, table, 1, q)
    for h in range(cfg.n_q_heads):
        assert np.array_equal(out[h], vals(pool[0, 3, 1, h // cfg.group, 0, :]))
    # all keys zero -> uniform weights -> mean of V
    p2 = pool.copy()
    p2[:, :, 0] = 0
    n = 21
    out = orc.attention(cfg, p2, bs, 0, table, n, q)
    _, V = _contiguous_kv(cfg, p2, bs, 0, table, n)
    for h in range(cfg.n_q_heads):
        assert np.allclose(out[h], V[h // cfg.group].mean(0), rtol=1e-12)
    # scaling: logits are q.k / sqrt(d) -- ratio of two probabilities is fixed by it
    out, probs = orc.attention(cfg, pool, bs, 0, table, 5, q, want_probs=True)
    K, _ = _contiguous_kv(cfg, pool, bs, 0, table, 5)
    want = math.exp((q[3] @ K[1, 0] - q[3] @ K[1, 4]) / math.sqrt(cfg.head_dim))
    assert np.isclose(probs[3, 0] / probs[3, 4], want, rtol=1e-10)
    # G = 1 (multi-head): every q head reads its own kv head
    mha = W.ModelConfig(**{**cfg.as_dict(), "n_q_heads": 2, "n_kv_heads": 2})
    out = orc.attention(mha, pool, bs, 0, table, 1, q[:2])
    assert np.array_equal(out[1], vals(pool[0, 3, 1, 1, 0, :]))


# ---------------------------------------------------------------- SwiGLU --
def test_swiglu(orc):
    assert orc.silu(0.0) == 0.0
    assert np.isclose(orc.silu(2.0), 2.0 / (1 + math.exp(-2.0)), rtol=1e-15)
    assert np.isclose(orc.silu(-3.0), -3.0 / (1 + math.exp(3.0)), rtol=1e-15)
    H, F = 24, 40
    wg, wu, wd = (bits(RNG.standard_normal(s)) for s in ((F, H), (F, H), (H, F)))
    h = RNG.standard_normal(H)
    out = orc.swiglu(wg, wu, wd, h)
    t = torch.from_numpy
    ref = t(vals(wd)) @ (torch.nn.functional.silu(t(vals(wg)) @ t(h)) * (t(vals(wu)) @ t(h)))
    assert np.allclose(out, ref.numpy(), rtol=1e-11, atol=1e-12)
    # zero gate projection -> zero output (gate and up are not swapped)
    assert np.all(orc.swiglu(np.zeros_like(wg), wu, wd, h) == 0)
    assert np.any(orc.swiglu(wg, np.zeros_like(wu), wd, h) == 0)


# ------------------------------------------------------------------- MoE --
def _moe_layer(cfg, seed):
    lay = W.generate.make_layer(cfg, seed, 0)
    return lay


def test_moe_reductions(orc):
    cfg = W.CONFIGS["tiny_moe"]
    lay = _moe_layer(cfg, 5)
    h = RNG.standard_normal(cfg.hidden)
    out, idx, wts = orc.moe(cfg, lay, h)
    assert abs(wts.sum() - 1.0) < 1e-12 and len(set(idx)) == cfg.top_k
    # numpy fp64 formulation: softmax over all experts, top-k, renormalise
    logits = vals(lay["w_router"]) @ h
    p = np.exp(logits - logits.max())
    p /= p.sum()
    order = sorted(range(cfg.n_experts), key=lambda e: (-p[e], e))[: cfg.top_k]
    assert list(idx) == order
    assert np.allclose(wts, p[order] / p[order].sum(), rtol=1e-12)
    ref = sum(w * orc.swiglu(lay["w_gate"][e], lay["w_up"][e], lay["w_down"][e], h)
              for e, w in zip(order, p[order] / p[order].sum()))
    assert np.allclose(out, ref, rtol=1e-11, atol=1e-13)
    # all experts identical -> equals that expert's dense MLP (weights sum to 1)
    same = dict(lay)
    for k in ("w_gate", "w_up", "w_down"):
        same[k] = np.repeat(lay[k][:1], cfg.n_experts, axis=0)
    out_same, _, _ = orc.moe(cfg, same, h)
    dense = orc.swiglu(lay["w_gate"][0], lay["w_up"][0], lay["w_down"][0], h)
    assert np.allclose(out_same, dense, rtol=1e-11, atol=1e-13)
    # top_k = n_experts -> the full soft mixture
    full = W.ModelConfig(**{**cfg.as_dict(), "top_k": cfg.n_experts})
    out_full, idx_full, wts_full = orc.moe(full, lay, h)
    assert sorted(idx_full) == list(range(cfg.n_experts))
    mix = sum(p[e] * orc.swiglu(lay["w_gate"][e], lay["w_up"][e], lay["w_down"][e], h)
              for e in range(cfg.n_experts))
    assert np.allclose(out_full, mix, rtol=1e-11, atol=1e-13)
    # equal router logits -> ties go to the lower expert index
    tie = dict(lay)
    tie["w_router"] = np.zeros_like(lay["w_router"])
    _, idx_tie, wts_tie = orc.moe(cfg, tie, h)
    assert list(idx_tie) == list(range(cfg.top_k)) and np.allclose(wts_tie, 1 / cfg.top_k)


def test_router_adopts_only_valid_proposals(orc):
    """A proposed expert set replaces the router's own top-k only where it is a valid top-k set up
    to the tolerance (every proposed expert within (1 - tol) of the best one left out); pinned against
    a numpy statement of that rule, an exact tie, and the whole step."""
    cfg = W.CONFIGS["tiny_moe"]
    lay = _moe_layer(cfg, 5)
    h = RNG.standard_normal(cfg.hidden)
    logits = vals(lay["w_router"]) @ h
    p = np.exp(logits - logits.max())
    p /= p.sum()
    order = sorted(range(cfg.n_experts), key=lambda e: (-p[e], e))
    own, runner = order[: cfg.top_k], order[cfg.top_k]
    idx, wts, adopted, margin = orc.route(cfg, lay["w_router"], h)
    assert list(idx) == own and not adopted and margin == 0.0
    # the own set in another order: nothing to adopt, nothing changes
    idx2, wts2, adopted, margin = orc.route(cfg, lay["w_router"], h, proposal=own[::-1], tie_tol=1.0)
    assert list(idx2) == own and np.array_equal(wts2, wts) and not adopted
    # the runner-up instead of the k-th: adopted exactly when the tolerance covers the margin
    prop = own[:-1] + [runner]
    want_margin = (p[own[-1]] - p[runner]) / p[own[-1]]
    assert want_margin > 1e-6                       # random logits: no accidental tie
    for tol, expect in ((want_margin * 0.99, False), (want_margin * 1.01, True)):
        idx3, wts3, adopted, margin = orc.route(cfg, lay["w_router"], h, proposal=prop, tie_tol=tol)
        assert adopted == expect and abs(margin - want_margin) < 1e-12
        chosen = sorted(prop, key=lambda e: (-p[e], e)) if expect else own
        assert list(idx3) == chosen
        assert np.allclose(wts3, p[chosen] / p[chosen].sum(), rtol=1e-12)
    # a proposal that leaves out the best expert for the worst: margin near 1, refused at any sane tolerance
    bad = own[1:] + [order[-1]]
    idx4, _, adopted, margin = orc.route(cfg, lay["w_router"], h, proposal=bad, tie_tol=1e-3)
    assert list(idx4) == own and not adopted and margin > 0.1
    # malformed proposals (repeated or out-of-range experts) are ignored
    for junk in ([own[0]] * cfg.top_k, [cfg.n_experts] + own[1:], [-1] + own[1:]):
        idx5, _, adopted, _ = orc.route(cfg, lay["w_router"], h, proposal=junk, tie_tol=1.0)
        assert list(idx5) == own and not adopted
    # an exact tie: two experts with the same router row; either set is valid at tolerance 0
    tie = dict(lay)
    wr = lay["w_router"].copy()
    a, b = own[-1], runner
    wr[b] = wr[a]
    tie["w_router"] = wr
    lo, hi = min(a, b), max(a, b)
    idx6, _, adopted, _ = orc.route(cfg, wr, h)
    assert lo in idx6 and hi not in idx6            # ties go to the lower index
    swapped = [e for e in idx6 if e != lo] + [hi]
    idx7, wts7, adopted, margin = orc.route(cfg, wr, h, proposal=swapped, tie_tol=0.0)
    assert adopted and margin == 0.0 and hi in idx7 and lo not in idx7


def test_step_with_adopted_proposal_equals_step_of_relabelled_model(orc):
    """Whole step.  Two experts of layer 1 get the same router row, an exact tie; the plain step
    takes the lower index.  Proposing the higher one (tolerance 0) must give, bit for bit, what the
    plain step gives on the model with those two experts' weights exchanged: the same probabilities
    in the same places, the other expert's matrices."""
    from workloads.blocktable import layout_for
    wl = W.WORKLOADS["cfg0_moe"]
    shape, lay = wl.cfg, layout_for(wl)
    weights = W.make_weights(shape, wl.seed_weights)
    pool = W.fill_kv_pool(shape, lay, wl.seed_kv, poison=False)
    tokens = W.initial_tokens(shape, wl.batch, wl.seed_tokens)

    def step(w, **kw):
        return orc.decode_step(shape, w, pool.copy(), 16, lay.tables, lay.contexts, tokens, want_trace=True, **kw)

    own = list(step(weights)["experts"][1][0])          # row 0, layer 1: largest probability first
    a = own[-1]
    b = next(e for e in range(shape.n_experts) if e not in own)
    lo, hi = min(a, b), max(a, b)
    L1 = weights["layers"][1]
    wr = L1["w_router"].copy()
    wr[b] = wr[a]
    tied = dict(weights, layers=[weights["layers"][0], dict(L1, w_router=wr)])
    base = step(tied)
    assert lo in base["experts"][1][0] and hi not in base["experts"][1][0]
    proposal = base["experts"].copy()
    proposal[1][0] = [hi if e == lo else e for e in base["experts"][1][0]]
    got = orc.decode_step_tie(shape, tied, pool.copy(), 16, lay.tables, lay.contexts, tokens, proposal, 0.0)
    assert got["adopted"].sum() == 1 and got["adopted"][1][0] == 1 and got["margin"][1][0] == 0.0
    assert hi in got["experts"][1][0] and lo not in got["experts"][1][0]
    swap = {k: L1[k].copy() for k in ("w_gate", "w_up", "w_down")}
    for k in swap:
        swap[k][[lo, hi]] = swap[k][[hi, lo]]
    relabelled = dict(weights, layers=[weights["layers"][0], dict(L1, w_router=wr, **swap)])
    want = step(relabelled)
    assert np.array_equal(got["logits"][0], want["logits"][0]) and got["next"][0] == want["next"][0]
    assert not np.array_equal(got["logits"][0], base["logits"][0])
    # a proposal equal to the own choice everywhere is the plain step, whatever the tolerance
    same = orc.decode_step_tie(shape, tied, pool.copy(), 16, lay.tables, lay.contexts, tokens, base["experts"], 1.0)
    assert same["adopted"].sum() == 0 and np.array_equal(same["logits"], base["logits"])
    # on the untied model the same proposal is no tie (margin above zero): refused at tolerance 0
    far = orc.decode_step_tie(shape, weights, pool.copy(), 16, lay.tables, lay.contexts, tokens,
                              step(weights)["experts"][:, :, ::-1].copy(), 0.0)
    assert far["adopted"].sum() == 0 and np.array_equal(far["logits"], step(weights)["logits"])


# ---------------------------------------------------------------- argmax --
def test_argmax_planted_and_ties(orc):
    v = RNG.standard_normal(1000).astype(np.float32)
    v[613] = 50.0
    assert orc.argmax(v) == 613
    v[77] = 50.0
    assert orc.argmax(v) == 77            # lowest index among equal maxima
    v[999] = 51.0
    assert orc.argmax(v) == 999
    assert orc.argmax(np.array([-5.0, -5.0, -7.0], dtype=np.float32)) == 0
