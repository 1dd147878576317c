"""ctypes face of the CPU oracle (oracle/relax_oracle.c).

TEST INFRASTRUCTURE ONLY: the test-suite, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module; the product path
(``paper_2311_02103_amd``) never does and shares nothing with it.

The functions here only marshal numpy arrays into the C calls; every piece of
arithmetic lives in the C file, written from the definitions listed in
relax_oracle.h.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "relax_oracle.c")
_LIB = os.path.join(_HERE, "librelax_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain C99, -O2, OpenMP over outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared",
               "-fno-fast-math", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


class _Seqs(C.Structure):
    _fields_ = [("B", C.c_int32), ("q_lens", C.POINTER(C.c_int32)),
                ("kv_lens", C.POINTER(C.c_int32)), ("slots", C.POINTER(C.c_int32))]


class _Dims(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("kv_capacity", C.c_int32)]


class _QMat(C.Structure):
    _fields_ = [("q", C.c_void_p), ("s", C.c_void_p), ("m", C.c_int32), ("k", C.c_int32), ("group", C.c_int32)]


class _LayerWeights(C.Structure):
    _fields_ = [("wqkv", _QMat), ("wo", _QMat), ("wgu", _QMat), ("wdown", _QMat),
                ("norm_attn", C.c_void_p), ("norm_ffn", C.c_void_p)]


class _Taps(C.Structure):
    _fields_ = [("xn", C.c_void_p), ("qkv", C.c_void_p), ("attn", C.c_void_p),
                ("x1", C.c_void_p), ("act", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build(force=True)
        _lib = C.CDLL(_LIB)
        _lib.oracle_half_to_float.restype = C.c_float
        _lib.oracle_half_to_float.argtypes = [C.c_uint16]
        _lib.oracle_num_threads.restype = C.c_int32
        _lib.oracle_decoder_layer.restype = C.c_int32
        _lib.oracle_decoder_layer_f32.restype = C.c_int32
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def half_to_float(bits: int) -> float:
    return float(lib().oracle_half_to_float(C.c_uint16(bits)))


@dataclass
class Dims:
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    kv_capacity: int = 64

    def c(self) -> _Dims:
        return _Dims(self.hidden, self.n_heads, self.n_kv_heads, self.head_dim, self.ffn,
                     self.rms_eps, self.rope_base, self.kv_capacity)


class Seqs:
    """(B, q_lens, kv_lens, slots): kv_lens are lengths AFTER the append."""

    def __init__(self, q_lens: Sequence[int], kv_lens: Sequence[int],
                 slots: Optional[Sequence[int]] = None):
        self.q = np.asarray(q_lens, dtype=np.int32).copy()
        self.kv = np.asarray(kv_lens, dtype=np.int32).copy()
        self.sl = None if slots is None else np.asarray(slots, dtype=np.int32).copy()
        assert self.q.shape == self.kv.shape and self.q.ndim == 1

    def c(self) -> _Seqs:
        ip = C.POINTER(C.c_int32)
        return _Seqs(len(self.q), self.q.ctypes.data_as(ip), self.kv.ctypes.data_as(ip),
                     None if self.sl is None else self.sl.ctypes.data_as(ip))


def unpack_int4(qweight: np.ndarray, m: int, k: int) -> np.ndarray:
    qweight = _chk(qweight, np.uint32, (m, k // 8))
    out = np.empty((m, k), dtype=np.int8)
    lib().oracle_unpack_int4(_p(qweight), C.c_int32(m), C.c_int32(k), _p(out))
    return out


def dequantize(qweight: np.ndarray, scales: np.ndarray, m: int, k: int, group: int = 32) -> np.ndarray:
    qweight = _chk(qweight, np.uint32, (m, k // 8))
    scales = _chk(scales, np.uint16, (m, (k + group - 1) // group))
    out = np.empty((m, k), dtype=np.float32)
    if group == 32:
        lib().oracle_dequantize(_p(qweight), _p(scales), C.c_int32(m), C.c_int32(k), _p(out))
    else:
        lib().oracle_dequantize_g(_p(qweight), _p(scales), C.c_int32(m), C.c_int32(k), C.c_int32(group), _p(out))
    return out


def dequant_matmul(x: np.ndarray, qweight: np.ndarray, scales: np.ndarray, m: int, k: int, group: int = 32) -> np.ndarray:
    x = _chk(x, np.float32)
    n = x.shape[0]
    assert x.shape == (n, k)
    qweight = _chk(qweight, np.uint32, (m, k // 8))
    scales = _chk(scales, np.uint16, (m, (k + group - 1) // group))
    out = np.empty((n, m), dtype=np.float32)
    if group == 32:
        lib().oracle_dequant_matmul(_p(x), _p(qweight), _p(scales), C.c_int32(m), C.c_int32(k), _p(out), C.c_int32(n))
    else:
        lib().oracle_dequant_matmul_g(_p(x), _p(qweight), _p(scales), C.c_int32(m), C.c_int32(k), C.c_int32(group),
                                      _p(out), C.c_int32(n))
    return out


def half_matmul(x: np.ndarray, w_bits: np.ndarray) -> np.ndarray:
    x = _chk(x, np.float32)
    w_bits = _chk(w_bits, np.uint16)
    n, k = x.shape
    m = w_bits.shape[0]
    assert w_bits.shape == (m, k)
    out = np.empty((n, m), dtype=np.float32)
    lib().oracle_half_matmul(_p(x), _p(w_bits), C.c_int32(m), C.c_int32(k), _p(out), C.c_int32(n))
    return out


def rmsnorm(x: np.ndarray, w_bits: np.ndarray, eps: float) -> np.ndarray:
    x = _chk(x, np.float32)
    n, H = x.shape
    w_bits = _chk(w_bits, np.uint16, (H,))
    y = np.empty_like(x)
    lib().oracle_rmsnorm(_p(x), _p(w_bits), _p(y), C.c_int32(n), C.c_int32(H), C.c_float(eps))
    return y


def rope(v: np.ndarray, pos: int, base: float) -> np.ndarray:
    v = _chk(v, np.float32).copy()
    assert v.ndim == 1
    lib().oracle_rope(_p(v), C.c_int32(v.shape[0]), C.c_int32(pos), C.c_float(base))
    return v


def rope_append(qkv: np.ndarray, dims: Dims, kcache: np.ndarray, vcache: np.ndarray, seqs: Seqs) -> np.ndarray:
    """Returns the roped qkv; kcache / vcache (fp32, C-contiguous) are updated in place."""
    qkv = _chk(qkv, np.float32).copy()
    n = qkv.shape[0]
    assert qkv.shape[1] == (dims.n_heads + 2 * dims.n_kv_heads) * dims.head_dim
    _cache_ok(kcache, dims), _cache_ok(vcache, dims)
    d, s = dims.c(), seqs.c()
    lib().oracle_rope_append(_p(qkv), C.byref(d), _p(kcache), _p(vcache), C.byref(s), C.c_int32(n))
    return qkv


def _cache_ok(cache: np.ndarray, dims: Dims):
    assert cache.dtype == np.float32 and cache.flags["C_CONTIGUOUS"]
    assert cache.ndim == 4 and cache.shape[1:] == (dims.kv_capacity, dims.n_kv_heads, dims.head_dim), cache.shape


def attention(q: np.ndarray, kcache: np.ndarray, vcache: np.ndarray, dims: Dims, seqs: Seqs,
              want_probs: bool = False):
    q = _chk(q, np.float32)
    n = q.shape[0]
    q = q.reshape(n, dims.n_heads, dims.head_dim)
    _cache_ok(kcache, dims), _cache_ok(vcache, dims)
    out = np.empty_like(q)
    probs = np.full((n, dims.n_heads, dims.kv_capacity), np.nan, dtype=np.float32) if want_probs else None
    d, s = dims.c(), seqs.c()
    lib().oracle_attention(_p(q), _p(kcache), _p(vcache), C.byref(d), C.byref(s), _p(out),
                           C.c_int32(n), _p(probs))
    return (out, probs) if want_probs else out


def swiglu(gu: np.ndarray) -> np.ndarray:
    gu = _chk(gu, np.float32)
    n, F2 = gu.shape
    a = np.empty((n, F2 // 2), dtype=np.float32)
    lib().oracle_swiglu(_p(gu), _p(a), C.c_int32(n), C.c_int32(F2 // 2))
    return a


def argmax(logits: np.ndarray) -> np.ndarray:
    logits = _chk(logits, np.float32)
    rows, V = logits.shape
    ids = np.empty((rows,), dtype=np.int32)
    lib().oracle_argmax(_p(logits), C.c_int32(rows), C.c_int32(V), _p(ids))
    return ids


@dataclass
class QMat:
    q: np.ndarray  # uint32 [m, k/8]
    s: np.ndarray  # uint16 [m, ceil(k/group)]
    m: int
    k: int
    group: int = 32

    def c(self) -> _QMat:
        self.q = _chk(self.q, np.uint32, (self.m, self.k // 8))
        self.s = _chk(self.s, np.uint16, (self.m, (self.k + self.group - 1) // self.group))
        return _QMat(self.q.ctypes.data, self.s.ctypes.data, self.m, self.k, self.group)


@dataclass
class LayerWeights:
    wqkv: QMat
    wo: QMat
    wgu: QMat
    wdown: QMat
    norm_attn: np.ndarray  # uint16 [H]
    norm_ffn: np.ndarray   # uint16 [H]

    def c(self) -> _LayerWeights:
        self.norm_attn = _chk(self.norm_attn, np.uint16)
        self.norm_ffn = _chk(self.norm_ffn, np.uint16)
        return _LayerWeights(self.wqkv.c(), self.wo.c(), self.wgu.c(), self.wdown.c(),
                             self.norm_attn.ctypes.data, self.norm_ffn.ctypes.data)


def decoder_layer(dims: Dims, w: LayerWeights, x, kcache: np.ndarray, vcache: np.ndarray,
                  seqs: Seqs, taps: bool = False):
    """x: uint16 fp16 bit patterns [n,H] or float32 [n,H].  Caches updated in place.

    Returns out fp32 [n,H] (and a dict of intermediates when taps=True).
    Raises ValueError on an inconsistent descriptor."""
    x = np.ascontiguousarray(x)
    n, H = x.shape
    assert H == dims.hidden
    _cache_ok(kcache, dims), _cache_ok(vcache, dims)
    out = np.empty((n, H), dtype=np.float32)
    h, g, d, F = dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.ffn
    tp = None
    tapd = {}
    if taps:
        tapd = dict(xn=np.empty((n, H), np.float32), qkv=np.empty((n, (h + 2 * g) * d), np.float32),
                    attn=np.empty((n, h * d), np.float32), x1=np.empty((n, H), np.float32),
                    act=np.empty((n, F), np.float32))
        tp = _Taps(*(tapd[k].ctypes.data for k in ("xn", "qkv", "attn", "x1", "act")))
    dm, wc, sq = dims.c(), w.c(), seqs.c()
    if x.dtype == np.uint16:
        fn = lib().oracle_decoder_layer
    else:
        assert x.dtype == np.float32
        fn = lib().oracle_decoder_layer_f32
    rc = fn(C.byref(dm), C.byref(wc), _p(x), _p(kcache), _p(vcache), C.byref(sq), _p(out),
            C.c_int32(n), C.byref(tp) if tp is not None else None)
    if rc != 0:
        raise ValueError("oracle_decoder_layer: inconsistent descriptor")
    return (out, tapd) if taps else out


def model_step(dims: Dims, layers: Sequence[LayerWeights], embedding_bits: np.ndarray, norm_final_bits: np.ndarray,
               lm_head_bits: np.ndarray, ids: np.ndarray, kcaches: Sequence[np.ndarray], vcaches: Sequence[np.ndarray],
               seqs: Seqs):
    """One step of the layer stack (Relax, Sec. 5.1, end-to-end LLM; Llama-style wrapper):
    x = E[ids] (fp16 table, exact in fp32); x = layer_l(x) with the residual stream kept in fp32;
    y_b = RMSNorm(x[last row of sequence b]; w_final); logits[b] = y_b . W_lm^T (fp16 weights, fp32 sums);
    greedy id = lowest index among the maxima.  Caches (one fp32 pair per layer) are updated in place.

    Returns (logits fp32 [B, V], ids int32 [B])."""
    emb = np.ascontiguousarray(embedding_bits).view(np.float16)
    x = emb[np.asarray(ids, dtype=np.int64)].astype(np.float32)
    for l, w in enumerate(layers):
        x = decoder_layer(dims, w, x, kcaches[l], vcaches[l], seqs)
    last = np.cumsum(np.asarray(seqs.q, dtype=np.int64)) - 1
    y = rmsnorm(np.ascontiguousarray(x[last]), norm_final_bits, dims.rms_eps)
    logits = half_matmul(y, lm_head_bits)
    return logits, argmax(logits)
