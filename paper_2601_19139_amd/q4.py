"""Packing of 4-bit (group-wise affine) matrices into the layout the library streams.

Input is the canonical form of a matrix: codes q uint8 [N, K] in 0..15, scale and
bias as bf16 bit patterns uint16 [N, K/64]; the weight is scale * q + bias.  Layout
only: no arithmetic of the decode path happens here.
"""
import numpy as np

GROUP = 64


def pack_q4(*mats: dict) -> np.ndarray:
    """Canonical matrices with the same K, stacked by rows, in the library's layout:
    code words, then all scales, then all biases.

    Codes: per row, K/128 steps of 128 columns; a step is 16 little-endian 32-bit words
    [4 lane groups lg][4 sub-steps s]; word (lg, s) holds the 8 columns
    step*128 + s*32 + lg*8 + j:  nibble i (bits 4i..4i+3) is column j = 2i, nibble 4+i is
    column j = 2i+1  (i = 0..3)."""
    q = np.concatenate([m["q"] for m in mats], axis=0)
    N, K = q.shape
    assert K % 128 == 0
    v = q.reshape(N, K // 128, 4, 4, 4, 2).astype(np.uint32)       # [row][step][s][lg][i][parity]
    v = v.transpose(0, 1, 3, 2, 4, 5)                               # [row][step][lg][s][i][parity]
    shifts = (4 * np.arange(4, dtype=np.uint32))[:, None] + np.array([0, 16], dtype=np.uint32)[None, :]
    words = (v << shifts).sum(axis=(4, 5), dtype=np.uint32)         # [row][step][lg][s]
    scale = np.concatenate([m["scale"] for m in mats], axis=0)
    bias = np.concatenate([m["bias"] for m in mats], axis=0)
    return np.concatenate([words.astype("<u4").reshape(-1).view(np.uint8), scale.reshape(-1).view(np.uint8),
                           bias.reshape(-1).view(np.uint8)])


def q4_bytes(n: int, k: int) -> int:
    """Bytes of a packed [n, k] matrix: half a byte per weight plus two bf16 per group of 64."""
    return n * k // 2 + 2 * n * (k // GROUP) * 2
