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


_hooks = None


def hooks():
    """The test-hook library tests/hooks/libbnn_test_hooks.so (ctypes handle)."""
    global _hooks
    import ctypes as C
    import os
    from paper_2301_05126_amd import api
    if _hooks is None:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hooks", "libbnn_test_hooks.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run __graft_entry__.build() (or tests/hooks/build.py)")
        _hooks = C.CDLL(path)
        _hooks.bnn_test_conv_binary_tiles.argtypes = api._lib.bnn_conv_binary.argtypes
        _hooks.bnn_test_conv_binary_tiles.restype = C.c_int
        _hooks.bnn_test_conv_binary_kernel_choice.argtypes = [C.c_int] * 6
        _hooks.bnn_test_conv_binary_kernel_choice.restype = C.c_int
    return _hooks


def conv_binary_tiles(inp, n, h, w, c_in, wt, c_out, thr=None, flip=None, pool=1, pool_first=0,
                      preact_out=None, packed_out=None):
    """bnn_conv_binary's arguments, run on the persistent tile kernels whatever the shape
    (through the test-hook library; marshalling only)."""
    from paper_2301_05126_amd import api
    api._check(hooks().bnn_test_conv_binary_tiles(
        api._ptr(inp), n, h, w, c_in, api._ptr(wt), c_out, api._ep(thr, flip, pool, pool_first),
        api._ptr(preact_out), api._ptr(packed_out), api._stream(None)), "bnn_test_conv_binary_tiles")


KERNEL_SMALL, TILE_256x128, TILE_128x128_STREAMED, TILE_128x128, TILE_64x64 = 10, 3, 2, 1, 0


def conv_kernel_choice(n, h, w, c_in, c_out, tiles_only=False):
    """Which kernel a binary convolution of this shape runs on (host-side query, no GPU work)."""
    return hooks().bnn_test_conv_binary_kernel_choice(n, h, w, c_in, c_out, 1 if tiles_only else 0)
