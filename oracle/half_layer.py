"""CPU reference of the decoder layer on plain fp16 weights -- TEST INFRASTRUCTURE ONLY (tests/, the smoke check and
bench.py's CPU baseline may call it; the product never does).

The fp16 models of the paper's LLM evaluation (Sec. 5.1) run the same Llama-style layer as the quantised ones with
unquantised matrices.  The reference is that layer written as the sequence of its steps, each step being this package's
own reference for it: RMSNorm, QKV matmul, rotary embedding + KV append, causal attention over the cache, output
projection + residual, RMSNorm, gate/up matmul, SwiGLU, down projection + residual.  Nothing is rounded between steps."""
import numpy as np


def decoder_layer_f16(dims, w, x, kcache: np.ndarray, vcache: np.ndarray, seqs) -> np.ndarray:
    """w: mapping with 'wqkv' [(h+2g)d, H], 'wo' [H, hd], 'wgu' [2F, H], 'wdown' [H, F] and 'norm_attn', 'norm_ffn' [H], all
    fp16 bit patterns.  x: fp16 bits or float32 [n,H].  kcache / vcache float32, updated in place.  Returns float32 [n,H]."""
    from . import attention, half_matmul, rmsnorm, rope_append, swiglu
    x = np.ascontiguousarray(x)
    xf = x.view(np.float16).astype(np.float32) if x.dtype == np.uint16 else x.astype(np.float32)
    n, H = xf.shape
    h, d = dims.n_heads, dims.head_dim
    assert H == dims.hidden
    xn = rmsnorm(xf, w["norm_attn"], dims.rms_eps)
    qkv = rope_append(half_matmul(xn, w["wqkv"]), dims, kcache, vcache, seqs)
    a = attention(np.ascontiguousarray(qkv[:, :h * d]), kcache, vcache, dims, seqs).reshape(n, h * d)
    x1 = xf + half_matmul(np.ascontiguousarray(a), w["wo"])
    act = swiglu(half_matmul(rmsnorm(x1, w["norm_ffn"], dims.rms_eps), w["wgu"]))
    return (x1 + half_matmul(act, w["wdown"])).astype(np.float32)
