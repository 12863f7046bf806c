"""Helpers for the GPU parity tests: device buffers via torch, model descriptors."""
import numpy as np
import torch

import paper_2301_05126_amd as P
from paper_2301_05126_amd.runtime import DeviceModel, pack_on_device  # noqa: F401

DEV = "cuda:0"
KINDS = {"conv_first_int8": P.LAYER_CONV_FIRST_INT8, "conv_binary": P.LAYER_CONV_BINARY,
         "fc_binary": P.LAYER_FC_BINARY}


def require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("GPU tests need a GPU (they never fall back to the CPU)")


def dev(a):
    """numpy -> device tensor (uint32 is carried as int32 bits)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(DEV)


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def empty_i32(*shape):
    return torch.empty(shape, dtype=torch.int32, device=DEV)


def fill_i32(shape, value):
    return torch.full(shape, value, dtype=torch.int32, device=DEV)


def pack_on_gpu(a_pm1):
    """+-1 int8 [rows, k] (numpy) -> packed device tensor via bnn_pack_bits."""
    return pack_on_device(a_pm1, DEV)
