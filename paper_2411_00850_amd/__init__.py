"""MI355X-native GWQ linear layer: thin Python binding over the C-ABI library libgwq.so.

All arithmetic of the path runs in the HIP kernels behind `gwq_pack` and `gwq_linear`; this
package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (GwqError, PackedLayer, layout, pack, quality, score, linear, linear_workspace, linear_scratch, linear_index, prepare_linear, linear_static, linear_bf16, STATIC_SCRATCH_BYTES, linear_plan, probe_stream, probe_mfma, linear_gate_up, prepare_linear_gate_up,
                      linear_batch, prepare_linear_batch, tuning_set,
                      version, library_path, lib)

__all__ = ["GwqError", "PackedLayer", "layout", "pack", "quality", "score", "linear", "linear_workspace", "linear_scratch", "linear_index", "prepare_linear", "linear_static", "linear_bf16", "STATIC_SCRATCH_BYTES", "linear_plan", "probe_stream", "probe_mfma", "linear_gate_up", "prepare_linear_gate_up", "linear_batch", "prepare_linear_batch", "tuning_set", "version",
           "library_path", "lib"]
