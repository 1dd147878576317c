"""Seeded synthetic inputs for the int4 decoder-layer workloads.

This module serves BOTH the CPU oracle's tests and the HIP path's tests and
benchmark, so it holds none of the layer's arithmetic: it only draws random
tensors, turns fp32 weights into the packed storage format the layer consumes
(that is input preparation, the inverse of nothing the layer computes -- the
layer only ever *decodes*), and names the workload shapes.

Everything is a pure function of (seed, tensor id): the generator is numpy's
counter-based Philox keyed with those two integers, so any tensor can be
regenerated alone, on any machine, without materialising the whole model.

Stand-in statement: the paper evaluates trained Llama-family checkpoints
(Sec. 5.1, Sec. 5.3); none is available here, so weights are random
N(0, 0.02^2), activations and pre-filled cache entries N(0, 1), norm weights
1 + 0.1 N(0, 1) -- same shapes, dtypes and storage format as the real thing.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

GROUP = 32          # quantisation group along k
NIBBLES = 8         # codes per uint32 word


@dataclass(frozen=True)
class LayerShape:
    name: str
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_layers: int = 1
    vocab: int = 32000

    @property
    def qkv_rows(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    def matrices(self) -> Dict[str, Tuple[int, int]]:
        """name -> (m, k) of the four quantised matrices of one layer."""
        H, F = self.hidden, self.ffn
        return {"wqkv": (self.qkv_rows, H), "wo": (H, self.n_heads * self.head_dim),
                "wgu": (2 * F, H), "wdown": (H, F)}

    def params_per_layer(self) -> int:
        return sum(m * k for m, k in self.matrices().values())

    def packed_bytes_per_layer(self) -> int:
        return sum(m * (k // 2) + m * ((k + GROUP - 1) // GROUP) * 2 for m, k in self.matrices().values())

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2


TINY = LayerShape("tiny", hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=688)
LLAMA7B = LayerShape("llama2-7b", hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn=11008, n_layers=32)
LLAMA70B = LayerShape("llama2-70b", hidden=8192, n_heads=64, n_kv_heads=8, head_dim=128, ffn=28672, n_layers=80)

# tensor-id space: (layer * 16 + slot) for weights, fixed bases for the rest
_SLOT = {"wqkv": 0, "wo": 1, "wgu": 2, "wdown": 3, "norm_attn": 4, "norm_ffn": 5}
TID_X = 1 << 20          # + call index
TID_KV = 2 << 20         # + layer * 2 + {0: K, 1: V}
TID_LENS = 3 << 20
TID_EMBED = 4 << 20
TID_LMHEAD = (4 << 20) + 1
TID_FINAL_NORM = (4 << 20) + 2
TID_IDS = (4 << 20) + 3


def rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)]))


def normal_f32(seed: int, tensor_id: int, shape, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    a = rng(seed, tensor_id).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def normal_f16_bits(seed: int, tensor_id: int, shape, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """fp16 tensor returned as its uint16 bit patterns (the wire format of every fp16 buffer)."""
    return normal_f32(seed, tensor_id, shape, std, mean).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits).view(np.float16).astype(np.float32)


def pack_codes(codes: np.ndarray) -> np.ndarray:
    """codes uint8 [m,k] in 0..15 -> uint32 [m,k/8]; element c%8 goes to bits 4*(c%8)..+3."""
    m, k = codes.shape
    assert k % NIBBLES == 0
    c = codes.reshape(m, k // NIBBLES, NIBBLES).astype(np.uint32)
    word = np.zeros((m, k // NIBBLES), dtype=np.uint32)
    for j in range(NIBBLES):
        word |= c[:, :, j] << np.uint32(4 * j)
    return word


def quantize_q4(w: np.ndarray, group: int = GROUP) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric int4, `group` columns per scale along k (32 unless stated; last group short if it does not divide k).

    Per group: scale = fp16(max|w| / 7); codes = clamp(rint(w / scale), -7, 7) + 8,
    an all-zero group (scale 0) gets code 8 everywhere.  Returns
    (qweight uint32 [m,k/8], scales uint16 bits [m,ceil(k/group)])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    m, k = w.shape
    assert k % NIBBLES == 0
    G = (k + group - 1) // group
    pad = G * group - k
    wp = np.pad(w, ((0, 0), (0, pad))) if pad else w
    grp = wp.reshape(m, G, group)
    amax = np.abs(grp).max(axis=2)
    s16 = (amax / np.float32(7.0)).astype(np.float16)
    s32 = s16.astype(np.float32)
    safe = np.where(s32 > 0, s32, np.float32(1.0))
    q = np.rint(grp / safe[:, :, None])
    q = np.clip(q, -7, 7)
    q = np.where((s32 > 0)[:, :, None], q, 0.0)
    codes = (q + 8).astype(np.uint8).reshape(m, G * group)[:, :k]
    return pack_codes(np.ascontiguousarray(codes)), s16.view(np.uint16)


def _qmat_slab(seed: int, tensor_id: int, slab: int, rows: int, k: int, std: float, group: int = GROUP):
    # every slab has its own Philox counter block, so the result does not depend on how slabs are scheduled
    g = np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)], counter=[0, 0, int(slab) + 1, 0]))
    w = g.standard_normal(size=(rows, k), dtype=np.float32) * np.float32(std)
    return quantize_q4(w, group)


def qmat(seed: int, tensor_id: int, m: int, k: int, std: float = 0.02, group: int = GROUP) -> Tuple[np.ndarray, np.ndarray]:
    """One random quantised matrix N(0, std^2); generated in row slabs (bounded host memory, threads)."""
    slab_rows = max(1, (1 << 22) // k)
    jobs = [(seed, tensor_id, i, min(slab_rows, m - r0), k, std, group) for i, r0 in enumerate(range(0, m, slab_rows))]
    if len(jobs) == 1:
        parts = [_qmat_slab(*jobs[0])]
    else:
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
            parts = list(pool.map(lambda j: _qmat_slab(*j), jobs))
    return np.concatenate([p[0] for p in parts], axis=0), np.concatenate([p[1] for p in parts], axis=0)


def layer_weights(shape: LayerShape, seed: int, layer: int = 0, group: int = GROUP) -> Dict[str, np.ndarray]:
    """Host arrays of one layer: '<mat>.q' uint32, '<mat>.s' uint16, 'norm_attn'/'norm_ffn' uint16."""
    out: Dict[str, np.ndarray] = {}
    for name, (m, k) in shape.matrices().items():
        q, s = qmat(seed, layer * 16 + _SLOT[name], m, k, group=group)
        out[name + ".q"], out[name + ".s"] = q, s
    for name in ("norm_attn", "norm_ffn"):
        out[name] = normal_f16_bits(seed, layer * 16 + _SLOT[name], (shape.hidden,), std=0.1, mean=1.0)
    return out


def activations(shape: LayerShape, seed: int, call: int, n: int) -> np.ndarray:
    """fp16 bits [n, hidden], N(0,1)."""
    return normal_f16_bits(seed, TID_X + call, (n, shape.hidden))


def kv_prefill(shape: LayerShape, seed: int, slots: int, capacity: int, layer: int = 0):
    """Two fp16-bit caches [slots, capacity, g, d] filled with N(0,1) everywhere (callers
    treat only entries below each sequence's past length as meaningful)."""
    dims = (slots, capacity, shape.n_kv_heads, shape.head_dim)
    return (normal_f16_bits(seed, TID_KV + 2 * layer, dims), normal_f16_bits(seed, TID_KV + 2 * layer + 1, dims))


def uniform_lengths(seed: int, count: int, lo: int, hi: int, stream: int = 0) -> np.ndarray:
    """count integers uniform in [lo, hi] inclusive."""
    return rng(seed, TID_LENS + stream).integers(lo, hi + 1, size=count, dtype=np.int32)


def model_tensors(shape: LayerShape, seed: int, vocab: int) -> Dict[str, np.ndarray]:
    """Embedding and LM head fp16 bits [vocab, hidden], N(0, 0.02^2); final norm weight fp16 bits [hidden], 1 + 0.1 N(0,1)."""
    return {"embedding": normal_f16_bits(seed, TID_EMBED, (vocab, shape.hidden), std=0.02),
            "lm_head": normal_f16_bits(seed, TID_LMHEAD, (vocab, shape.hidden), std=0.02),
            "norm_final": normal_f16_bits(seed, TID_FINAL_NORM, (shape.hidden,), std=0.1, mean=1.0)}


def token_ids(seed: int, count: int, vocab: int, stream: int = 0) -> np.ndarray:
    """count token ids uniform in [0, vocab)."""
    return rng(seed, TID_IDS + 16 * stream).integers(0, vocab, size=count, dtype=np.int32)


# ---- 3-bit weights (same group of 32 columns, 96 bits = three words per group) --------------------------------------
def pack_codes3(codes: np.ndarray) -> np.ndarray:
    """codes uint8 [m,k] in 0..7, k % 32 == 0 -> uint32 [m, 3k/32]: the codes of a row laid end to end as one
    little-endian bit string, 3 bits each (code c of a group starts at bit 3c of the group's three words)."""
    m, k = codes.shape
    assert k % GROUP == 0 and codes.max(initial=0) <= 7
    bits = ((codes[:, :, None] >> np.arange(3, dtype=np.uint8)) & 1).astype(np.uint8).reshape(m, 3 * k)
    return np.packbits(bits, axis=1, bitorder="little").view("<u4").reshape(m, 3 * k // 32)


def quantize_q3(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric 3-bit, group 32 along k: scale = fp16(max|w| / 3) per group, codes = clamp(rint(w / scale), -3, 3) + 4.
    Returns (uint32 [m, 3k/32], fp16 bits [m, k/32])."""
    m, k = w.shape
    g = w.reshape(m, k // GROUP, GROUP).astype(np.float32)
    scale = (np.abs(g).max(axis=2) / 3.0).astype(np.float16)
    scale = np.where(scale == 0, np.float16(1.0), scale)
    codes = np.clip(np.rint(g / scale.astype(np.float32)[:, :, None]), -3, 3).astype(np.int8) + 4
    return pack_codes3(codes.reshape(m, k).astype(np.uint8)), scale.view(np.uint16)


def qmat3(seed: int, tensor_id: int, m: int, k: int, std: float = 0.02) -> Tuple[np.ndarray, np.ndarray]:
    """One random 3-bit matrix from N(0, std^2) weights."""
    w = rng(seed, tensor_id).standard_normal((m, k), dtype=np.float32) * np.float32(std)
    return quantize_q3(w)


def layer_weights3(shape: LayerShape, seed: int, layer: int = 0) -> Dict[str, np.ndarray]:
    """Host arrays of one layer on 3-bit weights (canonical layout): '<mat>.q' uint32 [m, 3k/32], '<mat>.s' uint16, and
    the two norm vectors, from the same weight distributions as layer_weights."""
    out: Dict[str, np.ndarray] = {}
    for name, (m, k) in shape.matrices().items():
        out[name + ".q"], out[name + ".s"] = qmat3(seed, layer * 16 + _SLOT[name], m, k)
    for name in ("norm_attn", "norm_ffn"):
        out[name] = normal_f16_bits(seed, layer * 16 + _SLOT[name], (shape.hidden,), std=0.1, mean=1.0)
    return out
