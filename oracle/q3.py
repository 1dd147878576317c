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


def decoder_layer_q3(dims, w, x, kcache: np.ndarray, vcache: np.ndarray, seqs) -> np.ndarray:
    """One decoder layer whose four matrices are 3-bit (canonical layout): the layer of Sec. 5.1's Llama-style models with the
    3-bit weights of Sec. 5.3, written as the sequence of its steps -- RMSNorm, QKV matmul, rotary embedding + KV append,
    causal attention over the cache, output projection + residual, RMSNorm, gate/up matmul, SwiGLU, down projection +
    residual -- each step being the package's own reference for it (the matmuls the definition above, in float64).
    w: mapping with '<mat>.q' uint32 [m, 3k/32], '<mat>.s' fp16 bits [m, k/32] for wqkv, wo, wgu, wdown and 'norm_attn',
    'norm_ffn' fp16 bits [H].  x: fp16 bits or float32 [n,H].  kcache / vcache float32, updated in place.  Returns float32 [n,H]."""
    from . import attention, rmsnorm, rope_append, swiglu
    x = np.ascontiguousarray(x)
    xf = x.view(np.float16).astype(np.float32) if x.dtype == np.uint16 else x.astype(np.float32)
    n, H = xf.shape
    h, g, d, F = dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.ffn
    assert H == dims.hidden

    def mm(v, name, m, k):
        return dequant_matmul_q3(v, w[name + ".q"], w[name + ".s"], m, k)

    xn = rmsnorm(xf, w["norm_attn"], dims.rms_eps)
    qkv = mm(xn, "wqkv", (h + 2 * g) * d, H).astype(np.float32)
    qkv = rope_append(qkv, dims, kcache, vcache, seqs)
    a = attention(np.ascontiguousarray(qkv[:, :h * d]), kcache, vcache, dims, seqs).reshape(n, h * d)
    x1 = xf.astype(np.float64) + mm(a, "wo", H, h * d)
    xn2 = rmsnorm(x1.astype(np.float32), w["norm_ffn"], dims.rms_eps)
    act = swiglu(mm(xn2, "wgu", 2 * F, H).astype(np.float32))
    return (x1 + mm(act, "wdown", H, F)).astype(np.float32)
