"""The decode step through the entry point that allocates nothing
(dk_decode_step_static: the workspace is a fixed device array inside the
library) against the same steps through dk_decode_step with a caller-owned
workspace: same kernels, same order of additions, so the results must be the
same bits.  Two calls in a row share the array, the second with a smaller
input; a second model in between makes the library start the persistent
kernel's buffers over."""
import numpy as np
import pytest

import workloads as W
from workloads.blocktable import build_block_tables
from gpu_common import rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dk():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    import paper_2601_19139_amd as dk
    dk.lib()
    return dk


def variant(base, **kw):
    return W.ModelConfig(**{**W.CONFIGS[base].as_dict(), **kw})


class Case:
    def __init__(self, dk, shape, contexts, steps, seed):
        self.dk, self.shape, self.steps = dk, shape, steps
        self.lay = build_block_tables(contexts, 16, steps, seed=seed)
        self.weights = W.make_weights(shape, seed + 1)
        self.pool = W.fill_kv_pool(shape, self.lay, seed + 2)
        self.tokens = W.initial_tokens(shape, len(contexts), seed + 3)
        self.dm = dk.DeviceModel(shape, self.weights)

    def reference(self, flags=0):
        """`steps` steps through dk_decode_step (own workspace), the step advancing itself."""
        import torch
        dk = self.dk
        dkv = dk.DeviceKV(self.dm, self.lay, self.pool)
        dec = dk.Decoder(self.dm, dkv, self.lay.contexts, self.tokens)
        res = []
        for _ in range(self.steps):
            dec.step(flags=flags | dk.STEP_ADVANCE)
            torch.cuda.synchronize()
            res.append((dec.next.cpu().numpy().copy(), dec.logits.cpu().numpy().copy()))
        bits = dkv.bits().copy()
        dkv.close()
        return res, bits

    def start_static(self):
        import torch
        dk = self.dk
        self.dkv = dk.DeviceKV(self.dm, self.lay, self.pool)
        B = len(self.tokens)
        self.seq = torch.from_numpy(self.lay.contexts.astype(np.int32)).cuda()
        self.tok = torch.from_numpy(np.asarray(self.tokens, dtype=np.int32)).cuda()
        self.next = torch.empty(B, dtype=torch.int32, device="cuda")
        self.logits = torch.empty((B, self.shape.vocab), dtype=torch.float32, device="cuda")

    def static_step(self, flags=0):
        import torch
        dk = self.dk
        dk.decode_step_static(self.dm.handle, self.dkv.handle, self.dkv.block_tables, self.seq, self.tok,
                              self.logits, self.next, flags | dk.STEP_ADVANCE)
        torch.cuda.synchronize()
        return self.next.cpu().numpy().copy(), self.logits.cpu().numpy().copy()

    def close(self):
        self.dm.close()


def same(got, want, what):
    assert np.array_equal(got[0], want[0]), f"{what}: tokens differ"
    assert np.all(np.isfinite(got[1]))
    assert rel_l2(got[1], want[1]).max() <= 1e-6, f"{what}: logits differ"      # the stated bar is 1e-2
    assert np.array_equal(got[1], want[1]), f"{what}: same kernels, same order, yet other bits"


def test_static_scratch_step_matches_the_workspace_step(dk):
    # first call: 20 rows on the matrix-core path (GEMM tickets, attention partials, bf16 operand tiles)
    big = Case(dk, variant("tiny", head_dim=128, n_q_heads=8, n_kv_heads=2, qk_norm=True, vocab=5003),
               [3 + 7 * i for i in range(20)], 3, seed=61)
    # second call, smaller: 2 rows of the tiny model, which run as the persistent kernel and
    # keep hand-over buffers in the array from step to step
    small = Case(dk, variant("tiny", qk_norm=True), [63, 17], 4, seed=71)
    big_ref, big_bits = big.reference()
    small_ref, small_bits = small.reference()
    big.start_static()
    for s in range(big.steps):
        same(big.static_step(), big_ref[s], f"20 rows, step {s}")
    assert np.array_equal(big.dkv.bits(), big_bits)
    small.start_static()
    for s in range(2):
        same(small.static_step(), small_ref[s], f"2 rows, step {s}")
    # another model's step goes through the same array in between ...
    third = Case(dk, variant("tiny"), [40], 1, seed=81)
    third_ref, _ = third.reference()
    third.start_static()
    same(third.static_step(), third_ref[0], "1 row of another model")
    # ... and the first model continues where it was
    for s in range(2, small.steps):
        same(small.static_step(), small_ref[s], f"2 rows, step {s} (after another model)")
    assert np.array_equal(small.dkv.bits(), small_bits)
    for c in (big, small, third):
        c.dkv.close()
        c.close()


def test_static_scratch_refusals(dk):
    import torch
    c = Case(dk, variant("tiny"), [5, 9], 1, seed=91)
    c.start_static()
    with pytest.raises(dk.DecodeKitError) as e:
        dk.decode_step_static(c.dm.handle, c.dkv.handle, c.dkv.block_tables, c.seq, c.tok, c.logits, c.next,
                              dk.STEP_PROFILE)
    assert e.value.status == "DK_E_INVALID_ARG"
    # 40 layers, two rows and a table of 16 320 tokens (255 attention chunks per sequence): the two sets of
    # hand-over buffers of the persistent kernel (attention partials of every layer) exceed the array, so the
    # step runs one kernel per stage - and gives what dk_decode_step gives with DK_STEP_NO_FUSED
    deep = Case(dk, variant("tiny", n_layers=40, n_q_heads=8, n_kv_heads=4), [5, 9], 1, seed=92)
    deep.start_static()
    wide = torch.zeros((2, 1020), dtype=torch.int32, device="cuda")
    wide[:, :deep.dkv.block_tables.shape[1]] = deep.dkv.block_tables
    assert dk.workspace_bytes(deep.dm.handle, 2, 1020) > dk.STATIC_SCRATCH_BYTES
    # the reference: the same step (same table width) with a caller-owned workspace and DK_STEP_NO_FUSED,
    # on a second copy of the cache
    ref_kv = dk.DeviceKV(deep.dm, deep.lay, deep.pool)
    nbytes = dk.workspace_bytes(deep.dm.handle, 2, 1020)
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    ws_ptr = (ws.data_ptr() + 255) // 256 * 256
    r_next, r_logits = torch.empty_like(deep.next), torch.empty_like(deep.logits)
    dk.decode_step(deep.dm.handle, ref_kv.handle, wide, deep.seq.clone(), deep.tok.clone(), ws_ptr, r_logits, r_next,
                   dk.STEP_NO_FUSED, None, workspace_bytes_=nbytes)
    dk.decode_step_static(deep.dm.handle, deep.dkv.handle, wide, deep.seq, deep.tok, deep.logits, deep.next, 0)
    torch.cuda.synchronize()
    same((deep.next.cpu().numpy(), deep.logits.cpu().numpy()), (r_next.cpu().numpy(), r_logits.cpu().numpy()),
         "deep model, wide table")
    assert np.array_equal(deep.dkv.bits(), ref_kv.bits())
    ref_kv.close()
    deep.dkv.close()
    deep.close()
    torch.cuda.synchronize()
    c.dkv.close()
    c.close()
