"""Packing of 4-bit (group-wise affine) matrices into the layout the library streams.

Input is the canonical form of a matrix: codes q uint8 [N, K] in 0..15, scale and
bias as bf16 bit patterns uint16 [N, K/64]; the weight is scale * q + bias.  Layout
only: no arithmetic of the decode path happens here.
"""
import numpy as np

GROUP = 64


def pack_q4(*mats: dict) -> np.ndarray:
    """Canonical matrices with the same K, stacked by rows, as one packed matrix in the
    layout dk_create_model_q4 documents: N*K/2 bytes of codes, then per 16-row tile and
    128-column step 128 bytes of (scale, bias) pairs.  Returns uint8."""
    q = np.concatenate([np.asarray(m["q"], dtype=np.uint8) for m in mats], axis=0)
    scale = np.concatenate([np.asarray(m["scale"], dtype=np.uint16) for m in mats], axis=0)
    bias = np.concatenate([np.asarray(m["bias"], dtype=np.uint16) for m in mats], axis=0)
    N, K = q.shape
    if K % 128 or scale.shape != (N, K // GROUP) or bias.shape != scale.shape:
        raise ValueError("4-bit matrix: K must be a multiple of 128, scale/bias [N, K/64]")
    # codes: word (lg, s) of a step holds columns s*32 + lg*8 + j, column j in bits 4j..4j+3
    v = q.reshape(N, K // 128, 4, 4, 8).astype(np.uint32)          # [row][step][s][lg][j]
    v = v.transpose(0, 1, 3, 2, 4)                                  # [row][step][lg][s][j]
    words = (v << (4 * np.arange(8, dtype=np.uint32))).sum(axis=4, dtype=np.uint32)   # [row][step][lg][s]
    # scales and biases: [tile][step][lg][h][i][scale, bias] for row 16*tile + 4*lg + i
    tiles = (N + 15) // 16
    sb = np.zeros((tiles * 16, K // GROUP, 2), dtype=np.uint16)
    sb[:N, :, 0] = scale
    sb[:N, :, 1] = bias
    sb = sb.reshape(tiles, 4, 4, K // 128, 2, 2)                    # [tile][lg][i][step][h][sb]
    sb = sb.transpose(0, 3, 1, 4, 2, 5)                             # [tile][step][lg][h][i][sb]
    return np.concatenate([words.astype("<u4").reshape(-1).view(np.uint8),
                           np.ascontiguousarray(sb).reshape(-1).view(np.uint8)])


def q4_bytes(n: int, k: int) -> int:
    """Bytes of a packed [n, k] matrix."""
    return n * k // 2 + (n + 15) // 16 * (k // 128) * 128
