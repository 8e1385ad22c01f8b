"""MI355X-native chunkwise-parallel mLSTM kernels (Tiled Flash Linear Attention).

Thin binding over the C ABI of lib/libtfla_mlstm.so (see include/tfla_mlstm.h): argument
marshalling only, every step of the computation runs in the HIP kernels.  PyTorch is used
for device memory and streams.  There is no CPU or eager fallback: if the library has not
been built (python -m paper_2503_14376_amd.build) importing the binding fails loudly.
"""
from .binding import (BF16, EXP, F32, NORM_LAYER, NORM_RMS, SIG, TflaError, check, layer_workspace_bytes, lib_path,
                      load_library, mlstm_bwd, mlstm_fwd, mlstm_fwd_static, static_scratch_bytes, mlstm_layer_bwd, mlstm_layer_fwd, mlstm_layer_step, mlstm_step, profile_enable,
                      profile_read, status_string, tile_width, transfer_gain, workspace_bytes)

__all__ = ["EXP", "SIG", "F32", "BF16", "TflaError", "check", "lib_path", "load_library", "mlstm_fwd", "mlstm_fwd_static", "static_scratch_bytes",
           "mlstm_bwd", "mlstm_step", "mlstm_layer_fwd", "mlstm_layer_bwd", "mlstm_layer_step", "transfer_gain", "layer_workspace_bytes",
           "NORM_RMS", "NORM_LAYER", "profile_enable", "profile_read", "status_string", "tile_width", "workspace_bytes"]
