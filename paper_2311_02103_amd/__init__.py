"""MI355X (gfx950) implementation of the dynamic-shape int4 Llama-style decoder layer
(the hot path behind the LLM results of Relax, arXiv 2311.02103).

`binding` mirrors the C ABI of include/relax_mi355.h one to one; `runtime` holds the few
torch-side conveniences (device buffers for weights / cache / workspace).  Nothing here
computes: every step of the layer runs in the HIP kernels of csrc/.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    KVCache, LayerDims, LayerWeights, QMat, RelaxError, Seqs, check, make_dims,
    relax_attention, relax_build_id, relax_decoder_layer, relax_dequant_matmul, relax_dequantize,
    relax_rmsnorm_rope, relax_rope_table_bytes, relax_rope_table_init, relax_set_option, relax_unpack_int4, relax_workspace_bytes, relax_workspace_error,
    relax_workspace_init,
)
