"""Device-side bookkeeping around the C ABI: torch tensors that own the weights, the KV cache,
the rotary table and the workspace of one layer.  Allocation and host->device copies only."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as rx


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint16 (fp16 bits) -> torch.float16, uint32 -> int32 (same bits), others as is."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.float16)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(device)
    return torch.from_numpy(a).to(device)


def f16_bits(t: torch.Tensor) -> np.ndarray:
    """torch.float16 tensor -> numpy uint16 bit patterns on the host."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceLayer:
    """One decoder layer resident on the GPU, sized by upper bounds (n_max, L_max = kv_capacity, B_max)."""

    def __init__(self, host_weights: Dict[str, np.ndarray], *, hidden: int, n_heads: int, n_kv_heads: int, head_dim: int,
                 ffn: int, kv_capacity: int, kv_slots: int = 1, n_max: int = 1, B_max: Optional[int] = None,
                 rms_eps: float = 1e-5, rope_base: float = 10000.0, device="cuda", share_from: "DeviceLayer" = None, group: int = 32):
        self.device = device
        self.dims = rx.make_dims(hidden, n_heads, n_kv_heads, head_dim, ffn, kv_capacity, kv_slots, rms_eps, rope_base, group)
        mats = {"wqkv": ((n_heads + 2 * n_kv_heads) * head_dim, hidden), "wo": (hidden, n_heads * head_dim),
                "wgu": (2 * ffn, hidden), "wdown": (hidden, ffn)}
        self.t = {k: to_device(v, device) for k, v in host_weights.items()}
        self.weights = rx.LayerWeights(*(rx.QMat(self.t[n + ".q"], self.t[n + ".s"], *mats[n], group) for n in mats),
                                       self.t["norm_attn"], self.t["norm_ffn"])
        self.n_max, self.B_max = n_max, (B_max if B_max is not None else max(kv_slots, 1))
        if share_from is not None:          # layers of one model share cache geometry, rope table and workspace
            self.rope, self.ws, self.ws_bytes = share_from.rope, share_from.ws, share_from.ws_bytes
        else:
            self.rope = torch.empty(rx.relax_rope_table_bytes(self.dims) // 4, dtype=torch.float32, device=device)
            rx.check(rx.relax_rope_table_init(self.dims, self.rope), "relax_rope_table_init")
            self.ws_bytes = rx.relax_workspace_bytes(self.dims, n_max, kv_capacity, self.B_max)
            self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
            rx.check(rx.relax_workspace_init(self.dims, self.ws, self.ws_bytes), "relax_workspace_init")
        shape = (kv_slots, kv_capacity, n_kv_heads, head_dim)
        self.k = torch.zeros(shape, dtype=torch.float16, device=device)
        self.v = torch.zeros(shape, dtype=torch.float16, device=device)
        self.cache = rx.KVCache(self.k, self.v, self.rope)

    def load_cache(self, k_bits: np.ndarray, v_bits: np.ndarray) -> None:
        self.k.copy_(to_device(k_bits, self.device).view(self.k.shape))
        self.v.copy_(to_device(v_bits, self.device).view(self.v.shape))

    def forward(self, x: torch.Tensor, q_lens: Sequence[int], kv_lens: Sequence[int], slots=None,
                out: Optional[torch.Tensor] = None, device_table: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        seqs = rx.Seqs(q_lens, kv_lens, slots, device_table)
        rx.check(rx.relax_decoder_layer(self.dims, self.weights, x, self.cache, seqs, out, n, self.ws, self.ws_bytes, stream),
                 "relax_decoder_layer")
        return out

    def prepare(self, x: torch.Tensor, q_lens: Sequence[int], kv_lens: Sequence[int], slots=None,
                out: Optional[torch.Tensor] = None, stream=None):
        """Marshal one relax_decoder_layer call once; the returned closure only crosses the C boundary.
        The symbolic values (n, every L_b) are still plain arguments of that C call."""
        import ctypes as C
        n = x.shape[0]
        out = torch.empty_like(x) if out is None else out
        seqs = rx.Seqs(q_lens, kv_lens, slots)
        keep = (seqs, self.weights.c(), self.cache.c(), seqs.c(), x, out)
        fn = rx.lib().relax_decoder_layer
        args = (C.byref(self.dims), C.byref(keep[1]), x.data_ptr(), C.byref(keep[2]), C.byref(keep[3]), out.data_ptr(), n,
                self.ws.data_ptr(), self.ws_bytes)

        def call(stream_handle=None):
            rc = fn(*args, stream_handle if stream_handle is not None else rx._stream(stream))
            if rc != 0:
                raise rx.RelaxError(rc, "relax_decoder_layer")
            return out

        call.keep = keep
        return call


class DeviceModel:
    """A stack of decoder layers with embedding, final norm and fp16 LM head resident on the GPU.

    layer_weights: one host dict per layer (as DeviceLayer takes); a dict may appear several times in the list
    (weight sharing between layers keeps big synthetic models small on the host) -- its device copy is shared too,
    each layer still has its own KV cache."""

    def __init__(self, layer_weights: Sequence[Dict[str, np.ndarray]], embedding_bits: np.ndarray, norm_final_bits: np.ndarray,
                 lm_head_bits: np.ndarray, *, hidden: int, n_heads: int, n_kv_heads: int, head_dim: int, ffn: int,
                 kv_capacity: int, kv_slots: int = 1, n_max: int = 1, B_max: Optional[int] = None, rms_eps: float = 1e-5,
                 rope_base: float = 10000.0, device="cuda", group: int = 32):
        self.device = device
        self.dims = rx.make_dims(hidden, n_heads, n_kv_heads, head_dim, ffn, kv_capacity, kv_slots, rms_eps, rope_base, group)
        self.vocab = int(embedding_bits.shape[0])
        mats = {"wqkv": ((n_heads + 2 * n_kv_heads) * head_dim, hidden), "wo": (hidden, n_heads * head_dim),
                "wgu": (2 * ffn, hidden), "wdown": (hidden, ffn)}
        uploaded = {}
        self.layers = []
        for hw in layer_weights:
            if id(hw) not in uploaded:
                t = {k: to_device(v, device) for k, v in hw.items()}
                uploaded[id(hw)] = (t, rx.LayerWeights(*(rx.QMat(t[n + ".q"], t[n + ".s"], *mats[n], group) for n in mats),
                                                       t["norm_attn"], t["norm_ffn"]))
            self.layers.append(uploaded[id(hw)][1])
        self._tensors = uploaded
        self.embedding = to_device(embedding_bits, device)
        self.norm_final = to_device(norm_final_bits, device)
        self.lm_head = to_device(lm_head_bits, device)
        self.model = rx.Model(self.dims, self.layers, self.vocab, self.embedding, self.norm_final, self.lm_head)
        self.n_max, self.B_max = n_max, (B_max if B_max is not None else max(kv_slots, 1))
        self.rope = torch.empty(rx.relax_rope_table_bytes(self.dims) // 4, dtype=torch.float32, device=device)
        rx.check(rx.relax_rope_table_init(self.dims, self.rope), "relax_rope_table_init")
        self.ws_bytes = rx.relax_model_workspace_bytes(self.model, n_max, kv_capacity, self.B_max)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        rx.check(rx.relax_workspace_init(self.dims, self.ws, self.ws_bytes), "relax_workspace_init")
        shape = (kv_slots, kv_capacity, n_kv_heads, head_dim)
        self.k = [torch.zeros(shape, dtype=torch.float16, device=device) for _ in self.layers]
        self.v = [torch.zeros(shape, dtype=torch.float16, device=device) for _ in self.layers]
        self.caches = [rx.KVCache(k, v, self.rope) for k, v in zip(self.k, self.v)]

    def step(self, ids: torch.Tensor, q_lens: Sequence[int], kv_lens: Sequence[int], slots=None,
             logits: Optional[torch.Tensor] = None, next_ids: Optional[torch.Tensor] = None, stream=None,
             device_table: Optional[torch.Tensor] = None):
        """ids: int32 [n] on the device.  Returns (logits fp16 [B,V], next_ids int32 [B]).  With device_table (int32 [4][B] on
        the device: q_start, q_len, kv_len, slot) the kernels read positions there and kv_lens are upper bounds."""
        B = len(q_lens)
        if logits is None:
            logits = torch.empty((B, self.vocab), dtype=torch.float16, device=self.device)
        if next_ids is None:
            next_ids = torch.empty((B,), dtype=torch.int32, device=self.device)
        rx.check(rx.relax_model_step(self.model, ids, self.caches, rx.Seqs(q_lens, kv_lens, slots, device_table), logits, next_ids,
                                     int(ids.shape[0]), self.ws, self.ws_bytes, stream), "relax_model_step")
        return logits, next_ids


class DeviceLayerQ3:
    """One decoder layer on 3-bit weights resident on the GPU: the canonical matrices are uploaded, repacked once into the
    GPU-native layout (relax_repack_q3) and dropped; cache, rotary table and workspace as in DeviceLayer."""

    def __init__(self, host_weights: Dict[str, np.ndarray], *, hidden: int, n_heads: int, n_kv_heads: int, head_dim: int,
                 ffn: int, kv_capacity: int, kv_slots: int = 1, n_max: int = 1, B_max: Optional[int] = None,
                 rms_eps: float = 1e-5, rope_base: float = 10000.0, device="cuda"):
        self.device = device
        self.dims = rx.make_dims(hidden, n_heads, n_kv_heads, head_dim, ffn, kv_capacity, kv_slots, rms_eps, rope_base, 32)
        mats = {"wqkv": ((n_heads + 2 * n_kv_heads) * head_dim, hidden), "wo": (hidden, n_heads * head_dim),
                "wgu": (2 * ffn, hidden), "wdown": (hidden, ffn)}
        self.t = {}
        qm = []
        for name, (m, k) in mats.items():
            canon, sc = to_device(host_weights[name + ".q"], device), to_device(host_weights[name + ".s"], device)
            native = torch.empty_like(canon)
            rx.check(rx.relax_repack_q3(rx.QMat(canon, sc, m, k, 32), native), "relax_repack_q3")
            torch.cuda.synchronize()
            self.t[name + ".q"], self.t[name + ".s"] = native, sc
            qm.append(rx.QMat(native, sc, m, k, 32))
        self.t["norm_attn"], self.t["norm_ffn"] = to_device(host_weights["norm_attn"], device), to_device(host_weights["norm_ffn"], device)
        self.weights = rx.LayerWeights(*qm, self.t["norm_attn"], self.t["norm_ffn"])
        self.n_max, self.B_max = n_max, (B_max if B_max is not None else max(kv_slots, 1))
        self.rope = torch.empty(rx.relax_rope_table_bytes(self.dims) // 4, dtype=torch.float32, device=device)
        rx.check(rx.relax_rope_table_init(self.dims, self.rope), "relax_rope_table_init")
        self.ws_bytes = rx.relax_layer_q3_workspace_bytes(self.dims, n_max, kv_capacity, self.B_max)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        shape = (kv_slots, kv_capacity, n_kv_heads, head_dim)
        self.k = torch.zeros(shape, dtype=torch.float16, device=device)
        self.v = torch.zeros(shape, dtype=torch.float16, device=device)
        self.cache = rx.KVCache(self.k, self.v, self.rope)

    def load_cache(self, k_bits: np.ndarray, v_bits: np.ndarray) -> None:
        self.k.copy_(to_device(k_bits, self.device).view(self.k.shape))
        self.v.copy_(to_device(v_bits, self.device).view(self.v.shape))

    def forward(self, x: torch.Tensor, q_lens: Sequence[int], kv_lens: Sequence[int], slots=None,
                out: Optional[torch.Tensor] = None, device_table: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        seqs = rx.Seqs(q_lens, kv_lens, slots, device_table)
        rx.check(rx.relax_decoder_layer_q3(self.dims, self.weights, x, self.cache, seqs, out, n, self.ws, self.ws_bytes, stream),
                 "relax_decoder_layer_q3")
        return out


class DeviceLayerF16:
    """One decoder layer on plain fp16 weights resident on the GPU.  host_weights: 'wqkv', 'wo', 'wgu', 'wdown' as fp16 bit
    patterns [m,k] and the two norm vectors."""

    def __init__(self, host_weights: Dict[str, np.ndarray], *, hidden: int, n_heads: int, n_kv_heads: int, head_dim: int,
                 ffn: int, kv_capacity: int, kv_slots: int = 1, n_max: int = 1, B_max: Optional[int] = None,
                 rms_eps: float = 1e-5, rope_base: float = 10000.0, device="cuda"):
        self.device = device
        self.dims = rx.make_dims(hidden, n_heads, n_kv_heads, head_dim, ffn, kv_capacity, kv_slots, rms_eps, rope_base, 32)
        names = ("wqkv", "wo", "wgu", "wdown", "norm_attn", "norm_ffn")
        self.t = {k: to_device(host_weights[k], device) for k in names}
        self.weights = [self.t[k] for k in names]
        self.n_max, self.B_max = n_max, (B_max if B_max is not None else max(kv_slots, 1))
        self.rope = torch.empty(rx.relax_rope_table_bytes(self.dims) // 4, dtype=torch.float32, device=device)
        rx.check(rx.relax_rope_table_init(self.dims, self.rope), "relax_rope_table_init")
        self.ws_bytes = rx.relax_layer_f16_workspace_bytes(self.dims, n_max, kv_capacity, self.B_max)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        shape = (kv_slots, kv_capacity, n_kv_heads, head_dim)
        self.k = torch.zeros(shape, dtype=torch.float16, device=device)
        self.v = torch.zeros(shape, dtype=torch.float16, device=device)
        self.cache = rx.KVCache(self.k, self.v, self.rope)

    def load_cache(self, k_bits: np.ndarray, v_bits: np.ndarray) -> None:
        self.k.copy_(to_device(k_bits, self.device).view(self.k.shape))
        self.v.copy_(to_device(v_bits, self.device).view(self.v.shape))

    def forward(self, x: torch.Tensor, q_lens: Sequence[int], kv_lens: Sequence[int], slots=None,
                out: Optional[torch.Tensor] = None, device_table: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        seqs = rx.Seqs(q_lens, kv_lens, slots, device_table)
        rx.check(rx.relax_decoder_layer_f16(self.dims, self.weights, x, self.cache, seqs, out, n, self.ws, self.ws_bytes, stream),
                 "relax_decoder_layer_f16")
        return out
