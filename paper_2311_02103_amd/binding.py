"""ctypes binding of librelax_mi355.so: argument marshalling only.

Every function has the name and argument order of its C declaration in
include/relax_mi355.h (measurement and test aids: include/relax_mi355_bench.h) and returns the C status code.  Tensors are torch CUDA
tensors (PyTorch is used for device memory and streams, nothing else) or raw
integer device addresses; fp16 buffers may be torch.float16 or torch.uint16/int16.
There is no fallback: if the HIP library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Union

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librelax_mi355.so")

OK, ERR_NULL, ERR_SHAPE, ERR_CAPACITY, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = 0, -1, -2, -3, -4, -5, -6
STATUS_NAMES = {0: "RELAX_OK", -1: "RELAX_ERR_NULL", -2: "RELAX_ERR_SHAPE", -3: "RELAX_ERR_CAPACITY",
                -4: "RELAX_ERR_WORKSPACE", -5: "RELAX_ERR_UNSUPPORTED", -6: "RELAX_ERR_HIP"}


class RelaxError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__("%s returned %s" % (where, STATUS_NAMES.get(status, status)))
        self.status = status


def check(status: int, where: str = "relax call") -> None:
    if status != OK:
        raise RelaxError(status, where)


class LayerDims(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("group", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("kv_capacity", C.c_int32), ("kv_slots", C.c_int32)]


class QMatC(C.Structure):
    _fields_ = [("q", C.c_void_p), ("s", C.c_void_p), ("m", C.c_int32), ("k", C.c_int32), ("group", C.c_int32)]


class LayerWeightsC(C.Structure):
    _fields_ = [("wqkv", QMatC), ("wo", QMatC), ("wgu", QMatC), ("wdown", QMatC),
                ("norm_attn", C.c_void_p), ("norm_ffn", C.c_void_p)]


class LayerF16WeightsC(C.Structure):
    _fields_ = [("wqkv", C.c_void_p), ("wo", C.c_void_p), ("wgu", C.c_void_p), ("wdown", C.c_void_p),
                ("norm_attn", C.c_void_p), ("norm_ffn", C.c_void_p)]


class KVCacheC(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("rope", C.c_void_p)]


class SeqsC(C.Structure):
    _fields_ = [("B", C.c_int32), ("q_lens", C.POINTER(C.c_int32)), ("kv_lens", C.POINTER(C.c_int32)),
                ("slots", C.POINTER(C.c_int32)), ("device_table", C.c_void_p)]


class PlanEntryC(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("first_op", C.c_int32), ("last_op", C.c_int32), ("storage", C.c_int32), ("pinned", C.c_int32),
                ("offset", C.c_uint64), ("bytes", C.c_uint64), ("storage_bytes", C.c_uint64)]


class ModelC(C.Structure):
    _fields_ = [("dims", LayerDims), ("n_layers", C.c_int32), ("vocab", C.c_int32), ("layers", C.POINTER(LayerWeightsC)),
                ("embedding", C.c_void_p), ("norm_final", C.c_void_p), ("lm_head", C.c_void_p)]


_lib = None

_SIGNATURES = {
    "relax_build_id": (C.c_char_p, []),
    "relax_set_option": (C.c_int32, [C.c_char_p, C.c_int32]),
    "relax_profile_alt_gate_up": (None, [C.c_void_p, C.c_void_p]),
    "relax_workspace_init": (C.c_int32, [C.POINTER(LayerDims), C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_workspace_error": (C.c_int32, [C.POINTER(LayerDims), C.c_void_p, C.POINTER(C.c_int32)]),
    "relax_profile_step_events": (None, [C.c_void_p, C.c_void_p, C.c_int32]),
    "relax_workspace_bytes": (C.c_size_t, [C.POINTER(LayerDims), C.c_int32, C.c_int32, C.c_int32]),
    "relax_workspace_plan": (C.c_int32, [C.POINTER(LayerDims), C.c_int32, C.c_int32, C.c_int32, C.POINTER(PlanEntryC), C.c_int32,
                                         C.POINTER(C.c_int32), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "relax_workspace_plan_rule": (C.c_int32, [C.POINTER(LayerDims), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(PlanEntryC), C.c_int32,
                                              C.POINTER(C.c_int32), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "relax_rope_table_bytes": (C.c_size_t, [C.POINTER(LayerDims)]),
    "relax_rope_table_init": (C.c_int32, [C.POINTER(LayerDims), C.c_void_p, C.c_void_p]),
    "relax_matmul_workspace_bytes": (C.c_size_t, [C.POINTER(QMatC), C.c_int32]),
    "relax_dequant_matmul": (C.c_int32, [C.c_void_p, C.POINTER(QMatC), C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t,
                                         C.c_void_p]),
    "relax_half_matmul": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
    "relax_rmsnorm_rope": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                       C.POINTER(LayerDims), C.POINTER(KVCacheC), C.POINTER(SeqsC), C.c_void_p]),
    "relax_attention": (C.c_int32, [C.c_void_p, C.POINTER(KVCacheC), C.POINTER(SeqsC), C.POINTER(LayerDims), C.c_void_p,
                                    C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_attention_static_max_bytes": (C.c_size_t, []),
    "relax_attention_static": (C.c_int32, [C.c_void_p, C.POINTER(KVCacheC), C.POINTER(SeqsC), C.POINTER(LayerDims), C.c_void_p,
                                           C.c_int32, C.c_void_p]),
    "relax_decoder_layer": (C.c_int32, [C.POINTER(LayerDims), C.POINTER(LayerWeightsC), C.c_void_p, C.POINTER(KVCacheC),
                                        C.POINTER(SeqsC), C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_layer_q3_workspace_bytes": (C.c_size_t, [C.POINTER(LayerDims), C.c_int32, C.c_int32, C.c_int32]),
    "relax_decoder_layer_q3": (C.c_int32, [C.POINTER(LayerDims), C.POINTER(LayerWeightsC), C.c_void_p, C.POINTER(KVCacheC),
                                           C.POINTER(SeqsC), C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_layer_f16_workspace_bytes": (C.c_size_t, [C.POINTER(LayerDims), C.c_int32, C.c_int32, C.c_int32]),
    "relax_decoder_layer_f16": (C.c_int32, [C.POINTER(LayerDims), C.POINTER(LayerF16WeightsC), C.c_void_p, C.POINTER(KVCacheC),
                                            C.POINTER(SeqsC), C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_model_workspace_bytes": (C.c_size_t, [C.POINTER(ModelC), C.c_int32, C.c_int32, C.c_int32]),
    "relax_model_step": (C.c_int32, [C.POINTER(ModelC), C.c_void_p, C.POINTER(KVCacheC), C.POINTER(SeqsC), C.c_void_p,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
    "relax_probe_stream_read": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "relax_probe_mfma": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.c_void_p]),
    "relax_unpack_int4": (C.c_int32, [C.POINTER(QMatC), C.c_void_p, C.c_void_p]),
    "relax_dequantize": (C.c_int32, [C.POINTER(QMatC), C.c_void_p, C.c_void_p]),
    "relax_unpack_q3": (C.c_int32, [C.POINTER(QMatC), C.c_void_p, C.c_void_p]),
    "relax_dequant_matmul_q3": (C.c_int32, [C.c_void_p, C.POINTER(QMatC), C.c_void_p, C.c_int32, C.c_void_p]),
    "relax_repack_q3": (C.c_int32, [C.POINTER(QMatC), C.c_void_p, C.c_void_p]),
    "relax_unpack_q3_native": (C.c_int32, [C.POINTER(QMatC), C.c_void_p, C.c_void_p]),
    "relax_dequant_matmul_q3_native": (C.c_int32, [C.c_void_p, C.POINTER(QMatC), C.c_void_p, C.c_int32, C.c_void_p]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """Loads the HIP library; raises (never falls back) when it has not been built."""
    global _lib
    if _lib is None:
        try:                       # torch ships its own HIP runtime: it must be in the process first so that this library binds
            import torch  # noqa: F401  to the same one (a second runtime loaded beside it reports "no device" at the first launch)
        except ImportError:
            pass
        if not os.path.exists(LIB_PATH):
            raise ImportError("librelax_mi355.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or python paper_2311_02103_amd/build.py) first")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


Ptr = Union[None, int, "torch.Tensor"]  # noqa: F821


def _ptr(t: Ptr) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream or None
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _ref(obj):
    return None if obj is None else C.byref(obj)


@dataclass
class QMat:
    """A quantised matrix on the device: q int32/uint32 [m,k/8], s fp16 [m,ceil(k/group)]."""
    q: Ptr
    s: Ptr
    m: int
    k: int
    group: int = 32

    def c(self) -> QMatC:
        return QMatC(_ptr(self.q), _ptr(self.s), self.m, self.k, self.group)


@dataclass
class LayerWeights:
    wqkv: QMat
    wo: QMat
    wgu: QMat
    wdown: QMat
    norm_attn: Ptr
    norm_ffn: Ptr

    def c(self) -> LayerWeightsC:
        return LayerWeightsC(self.wqkv.c(), self.wo.c(), self.wgu.c(), self.wdown.c(), _ptr(self.norm_attn),
                             _ptr(self.norm_ffn))


@dataclass
class KVCache:
    k: Ptr
    v: Ptr
    rope: Ptr

    def c(self) -> KVCacheC:
        return KVCacheC(_ptr(self.k), _ptr(self.v), _ptr(self.rope))


class Seqs:
    """Host-side ragged descriptor; kv_lens are lengths AFTER this call's rows are appended.  device_table: optional
    device int32 [4][B] (q_start, q_len, kv_len, slot) that the kernels read instead; kv_lens are then upper bounds."""

    def __init__(self, q_lens: Sequence[int], kv_lens: Sequence[int], slots: Optional[Sequence[int]] = None, device_table: Ptr = None):
        arr = lambda v: (C.c_int32 * len(v))(*[int(e) for e in v])
        self.B = len(q_lens)
        self._q, self._kv = arr(q_lens), arr(kv_lens)
        self._sl = None if slots is None else arr(slots)
        self._table = device_table

    def c(self) -> SeqsC:
        ip = C.POINTER(C.c_int32)
        return SeqsC(self.B, C.cast(self._q, ip), C.cast(self._kv, ip), None if self._sl is None else C.cast(self._sl, ip),
                     _ptr(self._table))


def make_dims(hidden, n_heads, n_kv_heads, head_dim, ffn, kv_capacity, kv_slots=1, rms_eps=1e-5, rope_base=10000.0,
              group=32) -> LayerDims:
    return LayerDims(hidden, n_heads, n_kv_heads, head_dim, ffn, group, rms_eps, rope_base, kv_capacity, kv_slots)


def relax_build_id() -> str:
    return lib().relax_build_id().decode()


def relax_workspace_bytes(dims: Optional[LayerDims], n_max: int, L_max: int, B_max: int) -> int:
    return int(lib().relax_workspace_bytes(_ref(dims), n_max, L_max, B_max))


def relax_workspace_plan(dims: Optional[LayerDims], n: int, L: int, B: int, capacity: int = 32, rule: Optional[int] = None):
    """(status, entries, planned_bytes, unplanned_bytes); entries are dicts of the C struct's fields.  rule: None calls
    relax_workspace_plan, an integer calls relax_workspace_plan_rule with it (0: provably fits, 1: equal expressions)."""
    arr = (PlanEntryC * capacity)()
    count, planned, unplanned = C.c_int32(0), C.c_size_t(0), C.c_size_t(0)
    if rule is None:
        rc = lib().relax_workspace_plan(_ref(dims), n, L, B, arr, capacity, C.byref(count), C.byref(planned), C.byref(unplanned))
    else:
        rc = lib().relax_workspace_plan_rule(_ref(dims), n, L, B, rule, arr, capacity, C.byref(count), C.byref(planned), C.byref(unplanned))
    entries = []
    if rc == 0:
        for e in arr[:count.value]:
            entries.append({"name": e.name.decode(), "first_op": e.first_op, "last_op": e.last_op, "storage": e.storage, "pinned": e.pinned,
                            "offset": e.offset, "bytes": e.bytes, "storage_bytes": e.storage_bytes})
    return rc, entries, planned.value, unplanned.value


def relax_rope_table_bytes(dims: Optional[LayerDims]) -> int:
    return int(lib().relax_rope_table_bytes(_ref(dims)))


def relax_rope_table_init(dims: Optional[LayerDims], table: Ptr, stream=None) -> int:
    return lib().relax_rope_table_init(_ref(dims), _ptr(table), _stream(stream))


def relax_matmul_workspace_bytes(w: Optional[QMat], n_max: int) -> int:
    wc = None if w is None else w.c()
    return int(lib().relax_matmul_workspace_bytes(_ref(wc), n_max))


def relax_dequant_matmul(x: Ptr, w: Optional[QMat], out: Ptr, n: int, ws: Ptr = None, ws_bytes: int = 0, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_dequant_matmul(_ptr(x), _ref(wc), _ptr(out), n, _ptr(ws), ws_bytes, _stream(stream))


def relax_rmsnorm_rope(x: Ptr, w: Ptr, y: Ptr, n: int, H: int, eps: float, qkv: Ptr = None,
                       dims: Optional[LayerDims] = None, cache: Optional[KVCache] = None, seqs: Optional[Seqs] = None,
                       stream=None) -> int:
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_rmsnorm_rope(_ptr(x), _ptr(w), _ptr(y), n, H, eps, _ptr(qkv), _ref(dims), _ref(cc), _ref(sc),
                                    _stream(stream))


def relax_half_matmul(x: Ptr, w: Ptr, out: Ptr, n: int, m: int, k: int, stream=None) -> int:
    return lib().relax_half_matmul(_ptr(x), _ptr(w), _ptr(out), n, m, k, _stream(stream))


def relax_attention(q: Ptr, cache: Optional[KVCache], seqs: Optional[Seqs], dims: Optional[LayerDims], out: Ptr, n: int,
                    ws: Ptr, ws_bytes: int, stream=None) -> int:
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_attention(_ptr(q), _ref(cc), _ref(sc), _ref(dims), _ptr(out), n, _ptr(ws), ws_bytes, _stream(stream))


def relax_attention_static_max_bytes() -> int:
    return int(lib().relax_attention_static_max_bytes())


def relax_attention_static(q: Ptr, cache: Optional[KVCache], seqs: Optional[Seqs], dims: Optional[LayerDims], out: Ptr, n: int,
                           stream=None) -> int:
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_attention_static(_ptr(q), _ref(cc), _ref(sc), _ref(dims), _ptr(out), n, _stream(stream))


def relax_decoder_layer(dims: Optional[LayerDims], weights: Optional[LayerWeights], x: Ptr, cache: Optional[KVCache],
                        seqs: Optional[Seqs], out: Ptr, n: int, ws: Ptr, ws_bytes: int, stream=None) -> int:
    wc = None if weights is None else weights.c()
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_decoder_layer(_ref(dims), _ref(wc), _ptr(x), _ref(cc), _ref(sc), _ptr(out), n, _ptr(ws), ws_bytes,
                                     _stream(stream))


def relax_layer_q3_workspace_bytes(dims: Optional[LayerDims], n_max: int, L_max: int, B_max: int) -> int:
    return int(lib().relax_layer_q3_workspace_bytes(_ref(dims), n_max, L_max, B_max))


def relax_decoder_layer_q3(dims: Optional[LayerDims], weights: Optional[LayerWeights], x: Ptr, cache: Optional[KVCache],
                           seqs: Optional[Seqs], out: Ptr, n: int, ws: Ptr, ws_bytes: int, stream=None) -> int:
    wc = None if weights is None else weights.c()
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_decoder_layer_q3(_ref(dims), _ref(wc), _ptr(x), _ref(cc), _ref(sc), _ptr(out), n, _ptr(ws), ws_bytes,
                                        _stream(stream))


def relax_layer_f16_workspace_bytes(dims: Optional[LayerDims], n_max: int, L_max: int, B_max: int) -> int:
    return int(lib().relax_layer_f16_workspace_bytes(_ref(dims), n_max, L_max, B_max))


def relax_decoder_layer_f16(dims: Optional[LayerDims], weights, x: Ptr, cache: Optional[KVCache], seqs: Optional[Seqs], out: Ptr,
                            n: int, ws: Ptr, ws_bytes: int, stream=None) -> int:
    """weights: sequence of six device pointers (wqkv, wo, wgu, wdown, norm_attn, norm_ffn) or None."""
    wc = None if weights is None else LayerF16WeightsC(*[_ptr(w) for w in weights])
    cc = None if cache is None else cache.c()
    sc = None if seqs is None else seqs.c()
    return lib().relax_decoder_layer_f16(_ref(dims), _ref(wc), _ptr(x), _ref(cc), _ref(sc), _ptr(out), n, _ptr(ws), ws_bytes,
                                         _stream(stream))


class Model:
    """Host-side image of relax_model: keeps the C arrays (layer weight structs) alive."""

    def __init__(self, dims: LayerDims, layers: Sequence[LayerWeights], vocab: int, embedding: Ptr, norm_final: Ptr, lm_head: Ptr):
        self.dims, self.vocab, self.n_layers = dims, vocab, len(layers)
        self._layers = (LayerWeightsC * max(1, len(layers)))(*[lw.c() for lw in layers])
        self._keep = (layers, embedding, norm_final, lm_head)
        self._c = ModelC(dims, len(layers), vocab, C.cast(self._layers, C.POINTER(LayerWeightsC)) if layers else None,
                         _ptr(embedding), _ptr(norm_final), _ptr(lm_head))

    def c(self) -> ModelC:
        return self._c


def relax_model_workspace_bytes(model: Optional[Model], n_max: int, L_max: int, B_max: int) -> int:
    return int(lib().relax_model_workspace_bytes(None if model is None else C.byref(model.c()), n_max, L_max, B_max))


def relax_model_step(model: Optional[Model], ids: Ptr, caches: Optional[Sequence[KVCache]], seqs: Optional[Seqs], logits: Ptr,
                     next_ids: Ptr, n: int, ws: Ptr, ws_bytes: int, stream=None) -> int:
    sc = None if seqs is None else seqs.c()
    carr = None
    if caches is not None:
        carr = (KVCacheC * max(1, len(caches)))(*[c.c() for c in caches])
    return lib().relax_model_step(None if model is None else C.byref(model.c()), _ptr(ids),
                                  None if carr is None else C.cast(carr, C.POINTER(KVCacheC)), _ref(sc), _ptr(logits),
                                  _ptr(next_ids), n, _ptr(ws), ws_bytes, _stream(stream))


def relax_probe_stream_read(buf: Ptr, nbytes: int, sink: Ptr, stream=None) -> int:
    return lib().relax_probe_stream_read(_ptr(buf), nbytes, _ptr(sink), _stream(stream))


def relax_probe_mfma(sink: Ptr, iters: int, random_data: bool, stream=None):
    """Returns (status, floating-point operations of the launch)."""
    flops = C.c_int64(0)
    rc = lib().relax_probe_mfma(_ptr(sink), iters, 1 if random_data else 0, C.byref(flops), _stream(stream))
    return rc, flops.value


def relax_unpack_int4(w: Optional[QMat], out: Ptr, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_unpack_int4(_ref(wc), _ptr(out), _stream(stream))


def relax_dequantize(w: Optional[QMat], out: Ptr, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_dequantize(_ref(wc), _ptr(out), _stream(stream))


def relax_unpack_q3(w: Optional[QMat], out: Ptr, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_unpack_q3(_ref(wc), _ptr(out), _stream(stream))


def relax_dequant_matmul_q3(x: Ptr, w: Optional[QMat], out: Ptr, n: int, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_dequant_matmul_q3(_ptr(x), _ref(wc), _ptr(out), n, _stream(stream))


def relax_repack_q3(canonical: Optional[QMat], native_q: Ptr, stream=None) -> int:
    wc = None if canonical is None else canonical.c()
    return lib().relax_repack_q3(_ref(wc), _ptr(native_q), _stream(stream))


def relax_unpack_q3_native(w: Optional[QMat], out: Ptr, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_unpack_q3_native(_ref(wc), _ptr(out), _stream(stream))


def relax_dequant_matmul_q3_native(x: Ptr, w: Optional[QMat], out: Ptr, n: int, stream=None) -> int:
    wc = None if w is None else w.c()
    return lib().relax_dequant_matmul_q3_native(_ptr(x), _ref(wc), _ptr(out), n, _stream(stream))


def relax_profile_step_events(start: Optional[int], stop: Optional[int], step: int) -> None:
    """start / stop: raw hipEvent_t handles (e.g. torch.cuda.Event(enable_timing=True).cuda_event after a record)."""
    lib().relax_profile_step_events(start, stop, step)


def relax_set_option(name: str, value: int) -> int:
    return lib().relax_set_option(name.encode(), value)


def relax_workspace_init(dims: Optional[LayerDims], ws: Ptr, ws_bytes: int, stream=None) -> int:
    return lib().relax_workspace_init(_ref(dims), _ptr(ws), ws_bytes, _stream(stream))


def relax_workspace_error(dims: Optional[LayerDims], ws: Ptr) -> int:
    """Returns word 0 of the workspace's flag line (0 = fine; bit 1: a token id was out of range); raises on a call error."""
    flag = C.c_int32(0)
    check(lib().relax_workspace_error(_ref(dims), _ptr(ws), C.byref(flag)), "relax_workspace_error")
    return flag.value


def relax_profile_alt_gate_up(q_alt: Ptr, s_alt: Ptr) -> None:
    lib().relax_profile_alt_gate_up(_ptr(q_alt), _ptr(s_alt))
