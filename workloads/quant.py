"""4-bit weight-only quantisation of generated weights (input preparation).

Group-wise affine 4-bit, the scheme of the 4-bit MLX checkpoints the paper
benchmarks: every row of a matrix is cut into groups of 64 consecutive
columns; a group stores 64 codes q in 0..15 and two bf16 numbers, and stands
for the weights  scale * q + bias.  What the codes, scales and biases are is
decided here, once, from the seeded bf16 weights; what they MEAN (the
dequantisation and everything after it) is the method's arithmetic and lives
in the oracle and in the HIP kernels, each with its own code.

The canonical form is produced: q uint8 [N, K], scale / bias uint16 (bf16 bits)
[N, K/64].  The oracle reads it as it is; the library's own packed layout is
made from it by the library's Python front end.
"""
import numpy as np

from .generate import f32_from_bf16_bits

GROUP = 64


def _bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def quantize_q4(w_bits: np.ndarray) -> dict:
    """bf16 bit patterns [N, K] (K a multiple of 64) -> canonical 4-bit form.  A stack of expert
    matrices [E, N, K] is quantised row by row like one matrix and keeps its leading axis."""
    if w_bits.ndim == 3:
        E, N, K = w_bits.shape
        m = quantize_q4(w_bits.reshape(E * N, K))
        return {"q": m["q"].reshape(E, N, K), "scale": m["scale"].reshape(E, N, K // GROUP),
                "bias": m["bias"].reshape(E, N, K // GROUP)}
    N, K = w_bits.shape
    assert K % GROUP == 0
    w = f32_from_bf16_bits(w_bits).reshape(N, K // GROUP, GROUP)
    lo, hi = w.min(axis=2), w.max(axis=2)
    scale = (hi - lo) / 15.0
    scale[scale == 0.0] = 1.0
    scale_bits, bias_bits = _bf16_bits_rne(scale), _bf16_bits_rne(lo)
    s = f32_from_bf16_bits(scale_bits)[:, :, None]
    b = f32_from_bf16_bits(bias_bits)[:, :, None]
    q = np.clip(np.rint((w - b) / s), 0, 15).astype(np.uint8).reshape(N, K)
    return {"q": q, "scale": scale_bits, "bias": bias_bits}


MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def quantize_weights(weights: dict, threads: int = 8) -> dict:
    """The 4-bit version of a model's weights: every projection matrix (expert stacks included) and the
    lm_head in canonical 4-bit form (dict q/scale/bias); embedding, norm gains and routers stay bf16.  Matrices are
    quantised on a few threads (numpy releases the interpreter lock in its array loops)."""
    from concurrent.futures import ThreadPoolExecutor
    jobs = [(None, "lm_head", weights["lm_head"])]
    for i, L in enumerate(weights["layers"]):
        jobs += [(i, k, v) for k, v in L.items() if k in MATRICES]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        done = list(ex.map(lambda j: quantize_q4(j[2]), jobs))
    out = {"embed": weights["embed"], "g_final": weights["g_final"],
           "layers": [dict(L) for L in weights["layers"]]}
    for (i, k, _), m in zip(jobs, done):
        if i is None:
            out[k] = m
        else:
            out["layers"][i][k] = m
    return out
