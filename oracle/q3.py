"""CPU reference for the 3-bit weight format — TEST INFRASTRUCTURE ONLY (tests/, the smoke check and bench.py's CPU
baseline may call it; the product never does).

The paper deploys 3-bit quantised models where memory is short (Sec. 5.3) without printing a bit layout; the format
here is this build's reading, chosen to mirror the 4-bit one: groups of 32 columns share an fp16 scale, a group's 32
codes u in 0..7 are laid end to end, 3 bits each, in three little-endian uint32 words (code c at bits 3c..3c+2 of the
96-bit string, so codes 10 and 21 straddle a word boundary), and the weight is (u - 4) * scale.

Everything below is the definition written out in numpy, in float64."""
import numpy as np


def unpack_q3(qweight: np.ndarray, m: int, k: int) -> np.ndarray:
    """uint32 [m, 3k/32] -> int8 [m,k] in -4..3."""
    assert k % 32 == 0 and qweight.shape == (m, 3 * k // 32) and qweight.dtype == np.uint32
    words = qweight.reshape(m, k // 32, 3).astype(np.uint64)
    out = np.empty((m, k // 32, 32), dtype=np.int8)
    for c in range(32):
        word, shift = divmod(3 * c, 32)
        v = words[:, :, word] >> np.uint64(shift)
        if shift > 29:                                   # the code continues in the next word
            v = v | (words[:, :, word + 1] << np.uint64(32 - shift))
        out[:, :, c] = (v & np.uint64(7)).astype(np.int8) - 4
    return out.reshape(m, k)


def dequantize_q3(qweight: np.ndarray, scales: np.ndarray, m: int, k: int) -> np.ndarray:
    """float64 [m,k]: (u - 4) * scale of the column's group."""
    assert scales.shape == (m, k // 32) and scales.dtype == np.uint16
    s = scales.view(np.float16).astype(np.float64)
    return unpack_q3(qweight, m, k).astype(np.float64) * np.repeat(s, 32, axis=1)


def dequant_matmul_q3(x: np.ndarray, qweight: np.ndarray, scales: np.ndarray, m: int, k: int) -> np.ndarray:
    """x float [n,k] -> float64 [n,m] = x W^T."""
    assert x.shape[1] == k
    return x.astype(np.float64) @ dequantize_q3(qweight, scales, m, k).T
