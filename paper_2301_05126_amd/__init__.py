"""libbnn for MI355X: binarized-network layers (conv / FC over bit-packed +-1 operands, integer
sign thresholds, max-pool) behind a C ABI, with a thin ctypes binding.  The dense layers
expand the packed bits to FP4 +-1.0 in registers and multiply on the matrix cores with exact
FP32 accumulators; batch <= 8 FC layers use xor + popcount on the vector ALU.

Every step of the path runs in the HIP kernels of libbnn.so; this package only marshals
arguments.  There is no CPU fallback: importing the package raises if the shared library has
not been built (python -m paper_2301_05126_amd.build).
"""
from . import api  # noqa: F401
from . import runtime  # noqa: F401
from .api import (  # noqa: F401
    BnnError, Epilogue, LayerDesc, LayerTiming, Model,
    bnn_pack_bits, bnn_conv_first_int8, bnn_conv_binary, bnn_fc_binary,
    bnn_threshold_sign_maxpool, bnn_model_create, bnn_run_model, bnn_run_model_noalloc, bnn_model_destroy,
    bnn_model_workspace_bytes, bnn_status_string, bnn_last_hip_error, bnn_version,
    bnn_map_layers, bnn_fold_batchnorm,
    RUN_TIMED, RUN_GRAPH, RUN_STREAM, LAYER_CONV_FIRST_INT8, LAYER_CONV_BINARY, LAYER_FC_BINARY,
)
