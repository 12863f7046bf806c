"""Device-side set-up of a model for bnn_run_model: uploads tensors with torch, packs the
+-1 weights with bnn_pack_bits and fills the bnn_layer_desc array.  Marshalling only --
all arithmetic happens in libbnn's kernels."""
import numpy as np
import torch

from . import api as P

KINDS = {"conv_first_int8": P.LAYER_CONV_FIRST_INT8, "conv_binary": P.LAYER_CONV_BINARY,
         "fc_binary": P.LAYER_FC_BINARY}


def to_device(a, device="cuda:0"):
    """numpy array -> device tensor (uint32 carried as int32 bits)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(device)


def pack_on_device(a_pm1, device="cuda:0"):
    """+-1 int8 numpy [rows, k] -> packed device tensor [rows, ceil(k/32)] (bnn_pack_bits)."""
    rows, k = a_pm1.shape
    src = to_device(a_pm1, device)
    dst = torch.full((rows, (k + 31) // 32), -1, dtype=torch.int32, device=device)
    P.bnn_pack_bits(src, rows, k, dst)
    return dst


class DeviceModel:
    """A list of layer records (kind, c_in, c_out, kh, kw, pad, step, pool, h_out, w_out,
    weights, thr, flip as numpy) placed on the device, plus the bnn_model handle, its
    workspace and logits buffer.  With taps=True every layer also gets buffers that
    receive its int32 pre-activations and packed activations."""

    def __init__(self, layers, batch, in_shape, first_pad_value=-1, taps=False, device="cuda:0",
                 pool_first=False):
        if not torch.cuda.is_available():
            raise RuntimeError("libbnn needs a GPU; there is no CPU path")
        self.layers, self.batch, self.device = layers, batch, device
        self.keep, self.preact_taps, self.packed_taps = [], [], []
        descs = []
        ih, iw, ic = in_shape
        for L in layers:
            if L.kind == "conv_first_int8":
                wdev = to_device(L.weights, device)
            elif L.kind == "conv_binary":
                # [c_out][3][3][c_in]: each tap's channels are packed on their own
                wdev = pack_on_device(L.weights.reshape(L.c_out * 9, L.c_in), device)
            else:
                wdev = pack_on_device(L.weights.reshape(L.c_out, -1), device)
            thr = to_device(L.thr, device) if L.step else None
            flip = to_device(L.flip, device) if L.step else None
            self.keep += [wdev, thr, flip]
            ptap = ktap = None
            if taps:
                ptap = torch.full((batch, L.h_out * L.pool, L.w_out * L.pool, L.c_out), -7,
                                  dtype=torch.int32, device=device)
                if L.step:
                    ktap = torch.full((batch, L.h_out, L.w_out, (L.c_out + 31) // 32), -1,
                                      dtype=torch.int32, device=device)
            self.preact_taps.append(ptap)
            self.packed_taps.append(ktap)
            descs.append(P.LayerDesc(
                KINDS[L.kind], L.c_in, L.c_out, L.kh, L.kw, L.pad, first_pad_value,
                1 if L.step else 0, L.pool, 1 if pool_first else 0, wdev.data_ptr(),
                thr.data_ptr() if thr is not None else None,
                flip.data_ptr() if flip is not None else None,
                ptap.data_ptr() if ptap is not None else None,
                ktap.data_ptr() if ktap is not None else None))
        self.model = P.bnn_model_create(descs, batch, ih, iw, ic)
        self.ws_bytes = P.bnn_model_workspace_bytes(self.model)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        self.logits = torch.full((batch, layers[-1].c_out), -9, dtype=torch.int32, device=device)

    def run(self, images_dev, mode=P.RUN_STREAM, host_fn=None):
        return P.bnn_run_model(self.model, images_dev, self.logits, self.ws, self.ws_bytes, mode,
                               host_fn=host_fn)
