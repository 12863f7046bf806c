"""Helpers for the GPU parity tests: device buffers via torch, model descriptors."""
import numpy as np
import torch

import paper_2301_05126_amd as P

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
    """+-1 int8 [rows, k] (numpy) -> packed device tensor [rows, ceil(k/32)] via bnn_pack_bits."""
    rows, k = a_pm1.shape
    src = dev(a_pm1)
    dst = fill_i32((rows, (k + 31) // 32), -1)
    P.bnn_pack_bits(src, rows, k, dst)
    return dst


class DeviceModel:
    """Weights / thresholds of a workloads model on the device + a bnn_model handle."""

    def __init__(self, layers, batch, in_shape, first_pad_value=-1, taps=False):
        self.layers = layers
        self.batch = batch
        self.keep = []
        self.preact_taps, self.packed_taps = [], []
        descs = []
        ih, iw, ic = in_shape
        for L in layers:
            if L.kind == "conv_first_int8":
                wdev = dev(L.weights)
            else:
                w2 = L.weights.reshape(L.c_out, -1) if L.kind == "fc_binary" else L.weights
                if L.kind == "conv_binary":
                    # [c_out][3][3][c_in] -> pack each tap's channels separately
                    rows = w2.reshape(L.c_out * 9, L.c_in)
                    wdev = pack_on_gpu(rows)
                else:
                    wdev = pack_on_gpu(w2)
            thr = dev(L.thr) if L.step else None
            flip = dev(L.flip) if L.step else None
            self.keep += [wdev, thr, flip]
            ptap = ktap = None
            if taps:
                hpre, wpre = L.h_out * L.pool, L.w_out * L.pool
                ptap = fill_i32((batch, hpre, wpre, L.c_out), -7)
                if L.step:
                    ktap = fill_i32((batch, L.h_out, L.w_out, (L.c_out + 31) // 32), -1)
            self.preact_taps.append(ptap)
            self.packed_taps.append(ktap)
            descs.append(P.LayerDesc(KINDS[L.kind], L.c_in, L.c_out, L.kh, L.kw, L.pad, first_pad_value,
                                     1 if L.step else 0, L.pool, wdev.data_ptr(),
                                     thr.data_ptr() if thr is not None else None,
                                     flip.data_ptr() if flip is not None else None,
                                     ptap.data_ptr() if ptap is not None else None,
                                     ktap.data_ptr() if ktap is not None else None))
        self.model = P.bnn_model_create(descs, batch, ih, iw, ic)
        self.ws_bytes = P.bnn_model_workspace_bytes(self.model)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=DEV)
        self.logits = fill_i32((batch, layers[-1].c_out), -9)

    def run(self, images_dev, mode=P.RUN_STREAM, host_fn=None):
        return P.bnn_run_model(self.model, images_dev, self.logits, self.ws, self.ws_bytes, mode,
                               host_fn=host_fn)
