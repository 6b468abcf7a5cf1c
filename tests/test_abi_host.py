"""CPU-side tests of the C ABI: the library loads, exports every symbol the
header declares, and its host logic (block accounting, argument checks,
workspace sizing, byte accounting) behaves.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as W
from workloads.blocktable import layout_for
import paper_2601_19139_amd as dk
from paper_2601_19139_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):       # every header of the boundary
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(dk_[a-z_0-9]+)\s*\(", text))
    return sorted(syms)


def test_library_exports_every_declared_symbol():
    L = dk.lib()
    syms = header_symbols()
    assert len(syms) >= 19
    for s in syms:
        assert hasattr(L, s), s
    assert sorted(binding.EXPORTS) == syms           # the binding covers the whole header
    assert "gfx950" in dk.version()


def tiny_cfg():
    return dk.DkModelConfig.from_shape(W.CONFIGS["tiny"])


def test_pool_bytes_and_offset_formula():
    shape = W.CONFIGS["tiny"]
    cfg = tiny_cfg()
    nbytes = dk.kv_pool_bytes(cfg, 5, 16)
    assert nbytes == int(np.prod(W.pool_shape(shape, 5, 16))) * 2
    pool = dk.create_kv_pool(cfg, 5, 16, 0x1000, nbytes)      # memory is never touched on the host
    flat = np.arange(nbytes // 2).reshape(W.pool_shape(shape, 5, 16))
    for idx in [(0, 0, 0, 0, 0, 0), (1, 4, 1, 1, 15, 63), (1, 2, 0, 1, 7, 5), (0, 3, 1, 0, 9, 33)]:
        assert dk.kv_offset(pool, *idx) == flat[idx]
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_offset(pool, 2, 0, 0, 0, 0, 0)
    assert e.value.status == "DK_E_INVALID_ARG"
    dk.destroy_kv_pool(pool)


def test_block_accounting():
    cfg = tiny_cfg()
    pool = dk.create_kv_pool(cfg, 4, 16, 0x1000, dk.kv_pool_bytes(cfg, 4, 16))
    assert dk.kv_free_blocks(pool) == 4
    a, b = dk.kv_alloc_block(pool), dk.kv_alloc_block(pool)
    assert (a, b) == (0, 1)
    dk.kv_alloc_block_id(pool, 3)
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_alloc_block_id(pool, 3)
    assert e.value.status == "DK_E_BAD_BLOCK"
    dk.kv_retain_block(pool, a)                    # a second sequence shares block a
    assert dk.kv_refcount(pool, a) == 2
    dk.kv_release_block(pool, a)
    assert dk.kv_refcount(pool, a) == 1 and dk.kv_free_blocks(pool) == 1
    dk.kv_release_block(pool, a)
    assert dk.kv_refcount(pool, a) == 0 and dk.kv_free_blocks(pool) == 2
    with pytest.raises(dk.DecodeKitError):
        dk.kv_release_block(pool, a)               # already free
    with pytest.raises(dk.DecodeKitError):
        dk.kv_retain_block(pool, a)                # cannot share a free block
    assert dk.kv_alloc_block(pool) == 0            # lowest free id first
    assert dk.kv_alloc_block(pool) == 2
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_alloc_block(pool)
    assert e.value.status == "DK_E_POOL_EXHAUSTED" and "in use" in str(e.value)
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_refcount(pool, 4)
    assert e.value.status == "DK_E_BAD_BLOCK"
    dk.destroy_kv_pool(pool)


def test_validate_tables():
    wl = W.WORKLOADS["cfg2"]
    lay = layout_for(wl)
    cfg = dk.DkModelConfig.from_shape(wl.cfg)
    pool = dk.create_kv_pool(cfg, lay.num_blocks, 16, 0x1000, dk.kv_pool_bytes(cfg, lay.num_blocks, 16))
    for b in range(wl.batch):
        for bid in lay.tables[b]:
            if bid >= 0:
                if dk.kv_refcount(pool, int(bid)) == 0:
                    dk.kv_alloc_block_id(pool, int(bid))
                else:
                    dk.kv_retain_block(pool, int(bid))
    assert dk.kv_free_blocks(pool) == 0
    assert dk.kv_refcount(pool, int(lay.tables[0, 0])) == 8        # the shared 1024-token prefix
    dk.kv_validate_tables(pool, lay.tables, lay.contexts)
    # append into a shared block is refused
    bad_len = lay.contexts.copy()
    bad_len[0] = 1000
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_validate_tables(pool, lay.tables, bad_len)
    assert e.value.status == "DK_E_BAD_BLOCK" and "shared" in str(e.value)
    bad = lay.tables.copy()
    bad[3, 1] = lay.num_blocks
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_validate_tables(pool, bad, lay.contexts)
    assert "out of range" in str(e.value)
    bad = lay.tables.copy()
    bad[9, int(lay.contexts[9]) // 16] = bad[10, int(lay.contexts[10]) // 16]
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_validate_tables(pool, bad, lay.contexts)
    assert "another row" in str(e.value) or "shared" in str(e.value)
    too_long = lay.contexts.copy()
    too_long[2] = lay.max_blocks * 16
    with pytest.raises(dk.DecodeKitError) as e:
        dk.kv_validate_tables(pool, lay.tables, too_long)
    assert e.value.status == "DK_E_INVALID_ARG"
    dk.destroy_kv_pool(pool)


def fake_model(shape):
    cfg = dk.DkModelConfig.from_shape(shape)
    layers = (dk.LayerWeights * shape.n_layers)()
    for s in layers:
        for n in binding.LAYER_FIELDS:
            setattr(s, n, 0x1000)
    ptrs = dk.WeightPtrs(0x1000, 0x1000, 0x1000, layers)
    return cfg, ptrs, layers


def test_model_shape_checks_and_workspace():
    cfg, ptrs, _keep = fake_model(W.CONFIGS["qwen3_8b"])
    m = dk.create_model(cfg, ptrs)
    small = dk.workspace_bytes(m, 1, 40)
    big = dk.workspace_bytes(m, 16, 260)
    # (the largest part: the persistent kernel's two sets of hand-over buffers at batch 1, 78 MB for 4160 tokens)
    assert 0 < small < big < 128 << 20
    with pytest.raises(dk.DecodeKitError) as e:
        dk.workspace_bytes(m, 65, 40)
    assert e.value.status == "DK_E_INVALID_ARG"
    # decode_step argument checks fire before any launch
    pcfg = dk.DkModelConfig.from_shape(W.CONFIGS["tiny"])
    wrong_pool = dk.create_kv_pool(pcfg, 4, 16, 0x1000, dk.kv_pool_bytes(pcfg, 4, 16))
    tables = np.zeros((1, 4), dtype=np.int32)
    with pytest.raises(dk.DecodeKitError) as e:
        dk.decode_step(m, wrong_pool, tables, 0x1000, 0x1000, 0x1000, None, 0x1000, stream=0,
                       workspace_bytes_=1 << 30)
    assert "different model shape" in str(e.value)
    pool = dk.create_kv_pool(cfg, 4, 16, 0x1000, dk.kv_pool_bytes(cfg, 4, 16))
    with pytest.raises(dk.DecodeKitError) as e:
        dk.decode_step(m, pool, tables, 0x1000, 0x1000, 0x1000, None, 0x1000, stream=0,
                       workspace_bytes_=16)
    assert e.value.status == "DK_E_WORKSPACE_TOO_SMALL"
    with pytest.raises(dk.DecodeKitError) as e:
        dk.decode_step(m, pool, tables, 0x1000, 0x1000, 0x1001, None, 0x1000, stream=0,
                       workspace_bytes_=1 << 30)
    assert "aligned" in str(e.value)
    dk.destroy_model(m)
    for field, val, status in [("head_dim", 96, "DK_E_UNSUPPORTED_SHAPE"),
                               ("n_q_heads", 30, "DK_E_UNSUPPORTED_SHAPE"),
                               ("hidden", 4100, "DK_E_UNSUPPORTED_SHAPE"),
                               ("n_layers", 0, "DK_E_INVALID_ARG")]:
        c2, p2, _k2 = fake_model(W.CONFIGS["qwen3_8b"])
        setattr(c2, field, val)
        with pytest.raises(dk.DecodeKitError) as e:
            dk.create_model(c2, p2)
        assert e.value.status == status, field
    c3, p3, l3 = fake_model(W.CONFIGS["qwen3_8b"])
    l3[5].g_q = None
    with pytest.raises(dk.DecodeKitError) as e:
        dk.create_model(c3, p3)
    assert "layer 5" in str(e.value)


def test_workspace_covers_every_smaller_batch():
    """dk_workspace_bytes(model, B) is the need of the largest layout among batches 1..B (the layout
    changes with the batch size: persistent kernel up to 2 rows, vector-ALU path up to 4, matrix cores
    above, K-sliced GEMMs from 33 rows), so it never decreases with B."""
    for name in ("qwen3_0p6b", "qwen3_8b", "qwen3_30b_a3b_l4", "tiny"):
        cfg, ptrs, _keep = fake_model(W.CONFIGS[name])
        m = dk.create_model(cfg, ptrs)
        sizes = [dk.workspace_bytes(m, b, 40) for b in range(1, 65)]
        assert all(a <= b for a, b in zip(sizes, sizes[1:])), name
        dk.destroy_model(m)


def test_q4_model_checks_and_bytes():
    """dk_create_model_q4: dense shapes with every contraction length a multiple of 128; the
    algorithmic bytes count 4.5 bits per weight."""
    shape = W.CONFIGS["qwen3_8b"]
    cfg, ptrs, _keep = fake_model(shape)
    with pytest.raises(dk.DecodeKitError) as e:       # fake_model aliases lm_head and embed
        dk.create_model_q4(cfg, ptrs)
    assert e.value.status == "DK_E_INVALID_ARG"
    ptrs.lm_head = 0x2000
    m = dk.create_model_q4(cfg, ptrs)
    lay = layout_for(W.WORKLOADS["cfg3"])
    pool = dk.create_kv_pool(cfg, lay.num_blocks, 16, 0x1000, dk.kv_pool_bytes(cfg, lay.num_blocks, 16))
    got = dk.step_algorithmic_bytes(m, pool, lay.tables, lay.contexts, with_logits=False)
    n_weights = shape.dense_weight_bytes() // 2
    want = (n_weights // 2 + n_weights // 64 * 4
            + lay.unique_live_tokens(extra=1) * shape.kv_bytes_per_token() + 16 * shape.hidden * 2)
    assert got == want
    # every batch size takes the batched path: the workspace holds the bf16 hi/lo activations
    m16 = dk.create_model(cfg, ptrs)
    assert dk.workspace_bytes(m, 1, 40) > dk.workspace_bytes(m16, 1, 40)
    dk.destroy_model(m16)
    dk.destroy_kv_pool(pool)
    dk.destroy_model(m)
    for sname in ("tiny", "tiny_moe"):                # ffn 688; mixture of experts
        c2, p2, _k2 = fake_model(W.CONFIGS[sname])
        p2.lm_head = 0x2000
        with pytest.raises(dk.DecodeKitError) as e:
            dk.create_model_q4(c2, p2)
        assert e.value.status == "DK_E_UNSUPPORTED_SHAPE", sname


def test_pack_q4_layout():
    """The packed 4-bit layout, element by element against its description."""
    from paper_2601_19139_amd import pack_q4, q4_bytes
    rng = np.random.default_rng(1)
    N, K = 21, 256
    m = {"q": rng.integers(0, 16, size=(N, K), dtype=np.uint8),
         "scale": rng.integers(0, 65536, size=(N, K // 64), dtype=np.uint16),
         "bias": rng.integers(0, 65536, size=(N, K // 64), dtype=np.uint16)}
    buf = pack_q4(m)
    assert buf.dtype == np.uint8 and buf.size == q4_bytes(N, K) == N * K // 2 + 2 * 2 * 128
    words = buf[:N * K // 2].view("<u4").reshape(N, K // 128, 4, 4)
    sb = buf[N * K // 2:].view(np.uint16).reshape(2, K // 128, 4, 2, 4, 2)
    for _ in range(300):
        r, k = int(rng.integers(N)), int(rng.integers(K))
        step, s, lg, j = k // 128, (k % 128) // 32, (k % 32) // 8, k % 8
        nib = (int(words[r, step, lg, s]) >> (4 * j)) & 15
        assert nib == m["q"][r, k]
        t, lgr, i, h = r // 16, (r % 16) // 4, r % 4, (k % 128) // 64
        assert sb[t, step, lgr, h, i, 0] == m["scale"][r, k // 64]
        assert sb[t, step, lgr, h, i, 1] == m["bias"][r, k // 64]
    # stacking by rows equals packing the stacked matrix
    a = {k: v[:16] for k, v in m.items()}
    b = {k: v[16:] for k, v in m.items()}
    assert np.array_equal(pack_q4(a, b), buf)


@pytest.mark.parametrize("wname,expect_gb", [("cfg1", 1.251), ("cfg3", 24.80)])
def test_algorithmic_bytes_match_the_formula(wname, expect_gb):
    wl = W.WORKLOADS[wname]
    lay = layout_for(wl)
    cfg, ptrs, _keep = fake_model(wl.cfg)
    m = dk.create_model(cfg, ptrs)
    pool = dk.create_kv_pool(cfg, lay.num_blocks, 16, 0x1000, dk.kv_pool_bytes(cfg, lay.num_blocks, 16))
    got = dk.step_algorithmic_bytes(m, pool, lay.tables, lay.contexts, with_logits=False)
    want = (wl.cfg.dense_weight_bytes()
            + lay.unique_live_tokens(extra=1) * wl.cfg.kv_bytes_per_token()
            + wl.batch * wl.cfg.hidden * 2)
    assert got == want
    assert abs(got / 1e9 - expect_gb) < 0.01 * expect_gb
    dk.destroy_model(m)
    dk.destroy_kv_pool(pool)


def test_shared_prefix_counts_once_in_algorithmic_bytes():
    wl = W.WORKLOADS["cfg2"]
    lay = layout_for(wl)
    cfg, ptrs, _keep = fake_model(wl.cfg)
    m = dk.create_model(cfg, ptrs)
    pool = dk.create_kv_pool(cfg, lay.num_blocks, 16, 0x1000, dk.kv_pool_bytes(cfg, lay.num_blocks, 16))
    got = dk.step_algorithmic_bytes(m, pool, lay.tables, lay.contexts, with_logits=False)
    logical = int(sum(int(t) + 1 for t in lay.contexts))
    unique = logical - 7 * 1024
    assert got == wl.cfg.dense_weight_bytes() + unique * wl.cfg.kv_bytes_per_token() + 16 * wl.cfg.hidden * 2


def test_gemm_plan_follows_the_cost_model():
    """The batched-GEMM dispatch is the argmin of a cost estimate, not a table of shapes: properties
    that any shape must meet, checked on layer matrices of model shapes the calibration never saw
    (hidden 2560 / ffn 9728, hidden 5120 / ffn 17408) beside the ones it did."""
    STORE, RESID, SWIGLU = 0, 1, 2
    shapes = []
    for H, nq, nkv, F, V in ((1024, 16, 8, 3072, 151936), (3072, 24, 8, 8192, 128256), (4096, 32, 8, 12288, 151936),
                             (2560, 32, 8, 9728, 151936), (5120, 40, 8, 17408, 152064), (1536, 12, 2, 8960, 151936)):
        qkv, qd = (nq + 2 * nkv) * 128, nq * 128
        shapes += [(STORE, qkv, H), (RESID, H, qd), (SWIGLU, F, H), (RESID, H, F), (STORE, V, H)]
    for cus in (256, 128, 304):
        for epi, N, K in shapes:
            for B in (5, 16, 17, 32, 48, 64):
                w, s, us = dk.gemm_plan_query(epi, N, K, B, False, cus)
                tiles = (N + 15) // 16
                assert w in (0, 4, 8) and 1 <= s <= 8 and us > 0
                if w == 0:
                    assert s == 1
                    continue
                # instantiated block widths: 4 waves for residual projections (and the gate/up pair at 16 rows)
                assert (w == 4) == (epi == RESID or (epi == SWIGLU and B <= 16 and w == 4))
                row_blocks = (tiles + w - 1) // w
                assert s <= max(1, K // 512)                     # at least four K-steps per slice
                if row_blocks <= cus // 2:
                    assert row_blocks * s <= cus                  # one round of blocks
                if row_blocks >= 2 * cus:
                    assert s == 1                                 # many rounds already: no slices (the lm_head)
                # the estimate grows with the batch rows
                assert dk.gemm_plan_query(epi, N, K, 64, False, cus)[2] >= dk.gemm_plan_query(epi, N, K, 16, False, cus)[2] or w == 0
    # small matrices stay with the kernel whose waves split K; K off the 128 grid always does
    assert dk.gemm_plan_query(STORE, 4096, 1024, 16)[0] == 0
    assert dk.gemm_plan_query(RESID, 1024, 3072, 16)[0] == 0
    assert dk.gemm_plan_query(STORE, 6144, 4000, 32)[:2] == (0, 1)
    # the large ones do not
    assert dk.gemm_plan_query(SWIGLU, 12288, 4096, 16)[0] in (4, 8)
    assert dk.gemm_plan_query(RESID, 4096, 12288, 16)[0] == 4
    for bad in ((3, 64, 128, 16), (0, 0, 128, 16), (0, 64, 128, 4), (0, 64, 128, 65)):
        with pytest.raises(dk.DecodeKitError):
            dk.gemm_plan_query(*bad)
