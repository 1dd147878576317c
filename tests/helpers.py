"""Shared test plumbing: the same seeded host arrays go to the oracle (numpy) and to the GPU (torch)."""
import numpy as np

import oracle
import workloads as wl

ATOL, RTOL = 1e-2, 2e-2          # element passes if |gpu - ref| <= ATOL + RTOL * |ref|  (fp16 result vs fp32 oracle)


def assert_close(gpu, ref, what="", atol=ATOL, rtol=RTOL):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), what + ": non-finite GPU output"
    err = np.abs(gpu - ref)
    bad = err > atol + rtol * np.abs(ref)
    if bad.any():
        idx = np.unravel_index(np.argmax(err - rtol * np.abs(ref)), err.shape)
        raise AssertionError("%s: %d/%d outside tolerance, worst at %s gpu=%r ref=%r (max abs err %.3e)"
                             % (what, int(bad.sum()), bad.size, idx, gpu[idx], ref[idx], err.max()))
    return float(err.max())


def oracle_dims(shape: wl.LayerShape, cap: int) -> oracle.Dims:
    return oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps,
                       shape.rope_base, cap)


def oracle_weights(shape: wl.LayerShape, w) -> oracle.LayerWeights:
    mats = shape.matrices()
    return oracle.LayerWeights(*(oracle.QMat(w[n + ".q"], w[n + ".s"], *mats[n]) for n in ("wqkv", "wo", "wgu", "wdown")),
                               w["norm_attn"], w["norm_ffn"])


def device_layer(shape: wl.LayerShape, w, cap, slots=1, n_max=1, B_max=None):
    from paper_2311_02103_amd.runtime import DeviceLayer
    return DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                       ffn=shape.ffn, kv_capacity=cap, kv_slots=slots, n_max=n_max, B_max=B_max, rms_eps=shape.rms_eps,
                       rope_base=shape.rope_base)


def f32_cache(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(wl.f16_bits_to_f32(bits))
