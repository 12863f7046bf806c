"""ctypes binding of libbnn.so -- argument marshalling only.

Functions carry the names of the C entry points declared in include/bnn.h and take
torch tensors (device memory) or raw integer addresses.  Nothing is computed here.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbnn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2301_05126_amd.build` "
        "(there is no fallback path)")

_lib = C.CDLL(LIB_PATH)

RUN_TIMED, RUN_GRAPH, RUN_STREAM = 0, 1, 2
LAYER_CONV_FIRST_INT8, LAYER_CONV_BINARY, LAYER_FC_BINARY = 0, 1, 2


class Epilogue(C.Structure):
    _fields_ = [("thr", C.c_void_p), ("flip", C.c_void_p), ("pool", C.c_int), ("pool_first", C.c_int)]


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int), ("c_in", C.c_int), ("c_out", C.c_int),
                ("kh", C.c_int), ("kw", C.c_int), ("pad", C.c_int), ("pad_value", C.c_int),
                ("has_step", C.c_int), ("pool", C.c_int), ("pool_first", C.c_int),
                ("weights_dev", C.c_void_p), ("thr_dev", C.c_void_p), ("flip_dev", C.c_void_p),
                ("preact_tap_dev", C.c_void_p), ("packed_tap_dev", C.c_void_p)]


class LayerTiming(C.Structure):
    _fields_ = [("gpu_us", C.c_double), ("host_us", C.c_double),
                ("macs", C.c_int64), ("bytes_algorithmic", C.c_int64)]


HOST_LAYER_FN = C.CFUNCTYPE(None, C.c_int, C.c_void_p)

_vp, _i, _i64 = C.c_void_p, C.c_int, C.c_int64
_lib.bnn_status_string.restype = C.c_char_p
_lib.bnn_status_string.argtypes = [_i]
_lib.bnn_last_hip_error.restype = _i
_lib.bnn_version.restype = C.c_char_p
_lib.bnn_pack_bits.argtypes = [_vp, _i64, _i64, _vp, _vp]
_lib.bnn_conv_first_int8.argtypes = [_vp, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i,
                                     C.POINTER(Epilogue), _vp, _vp, _vp]
_lib.bnn_conv_binary.argtypes = [_vp, _i, _i, _i, _i, _vp, _i, C.POINTER(Epilogue), _vp, _vp, _vp]
_lib.bnn_fc_binary.argtypes = [_vp, _i64, _i64, _vp, _i64, C.POINTER(Epilogue), _vp, _vp, _vp]
_lib.bnn_threshold_sign_maxpool.argtypes = [_vp, _i, _i, _i, _i, _vp, _vp, _i, _i, _vp, _vp]
_lib.bnn_model_create.argtypes = [C.POINTER(LayerDesc), _i, _i, _i, _i, _i, C.POINTER(_vp)]
_lib.bnn_model_workspace_bytes.argtypes = [_vp]
_lib.bnn_model_workspace_bytes.restype = C.c_size_t
_lib.bnn_model_num_layers.argtypes = [_vp]
_lib.bnn_model_num_classes.argtypes = [_vp]
_lib.bnn_run_model.argtypes = [_vp, _vp, _vp, _vp, C.c_size_t, _i, C.POINTER(LayerTiming),
                               HOST_LAYER_FN, _vp, _vp]
_lib.bnn_run_model_noalloc.argtypes = [_vp, _vp, _vp, _vp]
_lib.bnn_run_model_noalloc.restype = _i
NOALLOC_SCRATCH_BYTES = 16 << 20
_lib.bnn_model_destroy.argtypes = [_vp]
_lib.bnn_model_destroy.restype = None
_dp = C.POINTER(C.c_double)
_lib.bnn_map_layers.argtypes = [_dp, _dp, _i, _i, _i, C.POINTER(_i), C.POINTER(_i), _dp]
_lib.bnn_fold_batchnorm.argtypes = [_dp, _dp, _dp, _dp, C.c_double, _i, C.POINTER(C.c_int32),
                                    C.POINTER(C.c_uint8)]
for _n in ("bnn_map_layers", "bnn_fold_batchnorm"):
    getattr(_lib, _n).restype = _i
for _n in ("bnn_pack_bits", "bnn_conv_first_int8", "bnn_conv_binary", "bnn_fc_binary",
           "bnn_threshold_sign_maxpool", "bnn_model_create", "bnn_run_model",
           "bnn_model_num_layers", "bnn_model_num_classes"):
    getattr(_lib, _n).restype = _i


class BnnError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        name = _lib.bnn_status_string(self.status).decode()
        extra = f" (hipError {_lib.bnn_last_hip_error()})" if name == "BNN_ERR_HIP" else ""
        super().__init__(f"{where}: {name}{extra}")


def bnn_status_string(s):
    return _lib.bnn_status_string(int(s)).decode()


def bnn_last_hip_error():
    return _lib.bnn_last_hip_error()


def bnn_version():
    return _lib.bnn_version().decode()


def _ptr(x):
    """Device address of a torch tensor, or a raw int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


_torch = None


def _stream(stream):
    if stream is None:
        global _torch
        if _torch is None:
            import torch
            _torch = torch
        return _torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(st, where):
    if st != 0:
        raise BnnError(st, where)


def _ep(thr, flip, pool, pool_first=0):
    if thr is None:
        return None
    return C.byref(Epilogue(_ptr(thr), _ptr(flip), int(pool), int(pool_first)))


def bnn_pack_bits(src, rows, k, dst, stream=None):
    _check(_lib.bnn_pack_bits(_ptr(src), rows, k, _ptr(dst), _stream(stream)), "bnn_pack_bits")


def bnn_conv_first_int8(inp, n, h, w, c_in, wt, c_out, kh, kw, pad, pad_value,
                        thr=None, flip=None, pool=1, pool_first=0, preact_out=None, packed_out=None,
                        stream=None):
    _check(_lib.bnn_conv_first_int8(_ptr(inp), n, h, w, c_in, _ptr(wt), c_out, kh, kw, pad, pad_value,
                                    _ep(thr, flip, pool, pool_first), _ptr(preact_out), _ptr(packed_out),
                                    _stream(stream)), "bnn_conv_first_int8")


def bnn_conv_binary(inp, n, h, w, c_in, wt, c_out, thr=None, flip=None, pool=1, pool_first=0,
                    preact_out=None, packed_out=None, stream=None):
    _check(_lib.bnn_conv_binary(_ptr(inp), n, h, w, c_in, _ptr(wt), c_out, _ep(thr, flip, pool, pool_first),
                                _ptr(preact_out), _ptr(packed_out), _stream(stream)), "bnn_conv_binary")


def bnn_fc_binary(a, m, k, b, n, thr=None, flip=None, c_out=None, packed_out=None, stream=None):
    _check(_lib.bnn_fc_binary(_ptr(a), m, k, _ptr(b), n, _ep(thr, flip, 1), _ptr(c_out),
                              _ptr(packed_out), _stream(stream)), "bnn_fc_binary")


def bnn_threshold_sign_maxpool(preact, n, h, w, c, thr, flip, pool, packed_out, pool_first=0, stream=None):
    _check(_lib.bnn_threshold_sign_maxpool(_ptr(preact), n, h, w, c, _ptr(thr), _ptr(flip), pool,
                                           int(pool_first), _ptr(packed_out), _stream(stream)),
           "bnn_threshold_sign_maxpool")


class Model:
    """Owner of a bnn_model handle (host object only)."""

    def __init__(self, handle, n_layers):
        self.handle = handle
        self.n_layers = n_layers

    def __del__(self):
        try:
            bnn_model_destroy(self)
        except Exception:
            pass


def bnn_model_create(descs, batch, in_h, in_w, in_c):
    arr = (LayerDesc * len(descs))(*descs)
    out = C.c_void_p()
    _check(_lib.bnn_model_create(arr, len(descs), batch, in_h, in_w, in_c, C.byref(out)),
           "bnn_model_create")
    return Model(out.value, len(descs))


def bnn_model_workspace_bytes(model):
    return int(_lib.bnn_model_workspace_bytes(model.handle))


_NO_HOST_FN = HOST_LAYER_FN(0)


def bnn_run_model(model, input_dev, logits_dev, workspace_dev, workspace_bytes, mode=RUN_STREAM,
                  host_fn=None, stream=None):
    """Returns the list of LayerTiming in TIMED mode, else None."""
    timings = (LayerTiming * model.n_layers)() if mode == RUN_TIMED else None
    cb = HOST_LAYER_FN(lambda layer, ctx: host_fn(layer)) if host_fn else _NO_HOST_FN
    _check(_lib.bnn_run_model(model.handle, _ptr(input_dev), _ptr(logits_dev), _ptr(workspace_dev),
                              workspace_bytes, mode, timings, cb, None, _stream(stream)),
           "bnn_run_model")
    return list(timings) if timings is not None else None


def bnn_run_model_noalloc(model, input_dev, logits_dev, stream=None):
    _check(_lib.bnn_run_model_noalloc(model.handle, _ptr(input_dev), _ptr(logits_dev), _stream(stream)),
           "bnn_run_model_noalloc")


def bnn_model_destroy(model):
    if model is not None and model.handle:
        _lib.bnn_model_destroy(model.handle)
        model.handle = None


def bnn_map_layers(cpu_us, gpu_us):
    """cpu_us, gpu_us: nested lists / arrays [n_batch][n_layers][n_impl] (host).
    Returns (best_batch_index, mapping list, total_us)."""
    import numpy as np
    c = np.ascontiguousarray(cpu_us, dtype=np.float64)
    g = np.ascontiguousarray(gpu_us, dtype=np.float64)
    if c.shape != g.shape or c.ndim != 3:
        raise ValueError("bnn_map_layers: tables must have the same [batch][layer][impl] shape")
    nb, nl, ni = c.shape
    best = C.c_int()
    mapping = (C.c_int * nl)()
    total = C.c_double()
    _check(_lib.bnn_map_layers(c.ctypes.data_as(_dp), g.ctypes.data_as(_dp), nb, nl, ni, C.byref(best),
                               mapping, C.byref(total)), "bnn_map_layers")
    return best.value, list(mapping), total.value


def bnn_fold_batchnorm(gamma, beta, mean, var, eps):
    """Host arrays in, (thr int32 array, flip uint8 array) out."""
    import numpy as np
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (gamma, beta, mean, var)]
    n = arrs[0].shape[0]
    thr = np.empty(n, dtype=np.int32)
    flip = np.empty(n, dtype=np.uint8)
    _check(_lib.bnn_fold_batchnorm(*[a.ctypes.data_as(_dp) for a in arrs], float(eps), n,
                                   thr.ctypes.data_as(C.POINTER(C.c_int32)),
                                   flip.ctypes.data_as(C.POINTER(C.c_uint8))), "bnn_fold_batchnorm")
    return thr, flip
