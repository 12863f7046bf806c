"""CPU oracle for the binarized-network layers -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over `bnn_oracle.c`, which states each layer of the HEP-BNN
paper's Sec. II-A (binarized neuron, 3x3 convolution, 2x2 max-pool, step, fully
connected, flatten) as plain loops over unpacked +-1 / int8 values with int32 sums.
Nothing here packs bits or uses xor/popcount, and nothing here is imported by the GPU
library or its Python binding.  Allowed callers: tests, the smoke check, and the
benchmark's CPU-baseline leg.

Pins (tests/test_oracle_pins.py): the popcount identity of the neuron formula evaluated
on independently packed Python integers, brute force over all inputs of tiny layers,
closed forms for constant inputs at interior / edge / corner pixels, exact numpy int64
products, threshold ties, and OR-equals-max pooling.  Conventions that the paper does
not fix (pad value -1, strict '>', flip flag, step-then-pool order, (h, w, c) flatten
order) are pinned only by those closed forms once chosen: parity unpinned by the paper
for those choices.
"""
import ctypes as C
import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        i8p, i32p, u8p = C.POINTER(C.c_int8), C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
        L.ref_conv2d.argtypes = [i8p, C.c_int, C.c_int, C.c_int, C.c_int, i8p, C.c_int,
                                 C.c_int, C.c_int, C.c_int, C.c_int, i32p]
        L.ref_conv2d.restype = C.c_int
        L.ref_fc.argtypes = [i8p, C.c_int64, C.c_int64, i8p, C.c_int64, i32p]
        L.ref_fc.restype = C.c_int
        L.ref_dot.argtypes = [i8p, i8p, C.c_int64]
        L.ref_dot.restype = C.c_int32
        L.ref_step.argtypes = [i32p, C.c_int64, C.c_int, i32p, u8p, i8p]
        L.ref_step.restype = C.c_int
        L.ref_maxpool2_i32.argtypes = [i32p, C.c_int, C.c_int, C.c_int, C.c_int, i32p]
        L.ref_maxpool2_i32.restype = C.c_int
        L.ref_maxpool2_i8.argtypes = [i8p, C.c_int, C.c_int, C.c_int, C.c_int, i8p]
        L.ref_maxpool2_i8.restype = C.c_int
        L.ref_max_threads.restype = C.c_int
        L.ref_set_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle: bad shape in {what}")


def max_threads() -> int:
    return lib().ref_max_threads()


def set_threads(t: int) -> None:
    lib().ref_set_threads(int(t))


def conv2d(x, wt, pad, pad_value):
    """x int8 [n,h,w,c_in]; wt int8 +-1 [c_out,kh,kw,c_in] -> int32 [n,ho,wo,c_out]."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    wt = np.ascontiguousarray(wt, dtype=np.int8)
    n, h, w, ci = x.shape
    co, kh, kw, ci2 = wt.shape
    if ci != ci2:
        raise ValueError("oracle: channel mismatch")
    ho, wo = h + 2 * pad - kh + 1, w + 2 * pad - kw + 1
    out = np.empty((n, max(ho, 0), max(wo, 0), co), dtype=np.int32)
    _chk(lib().ref_conv2d(_p(x, C.c_int8), n, h, w, ci, _p(wt, C.c_int8), co, kh, kw, pad,
                          int(pad_value), _p(out, C.c_int32)), "conv2d")
    return out


def fc(a, wt):
    """a int8 [m,k]; wt int8 +-1 [n,k] -> int32 [m,n]."""
    a = np.ascontiguousarray(a, dtype=np.int8)
    wt = np.ascontiguousarray(wt, dtype=np.int8)
    m, k = a.shape
    n, k2 = wt.shape
    if k != k2:
        raise ValueError("oracle: K mismatch")
    out = np.empty((m, n), dtype=np.int32)
    _chk(lib().ref_fc(_p(a, C.c_int8), m, k, _p(wt, C.c_int8), n, _p(out, C.c_int32)), "fc")
    return out


def dot(a_row, b_row) -> int:
    a_row = np.ascontiguousarray(a_row, dtype=np.int8)
    b_row = np.ascontiguousarray(b_row, dtype=np.int8)
    assert a_row.shape == b_row.shape and a_row.ndim == 1
    return int(lib().ref_dot(_p(a_row, C.c_int8), _p(b_row, C.c_int8), a_row.shape[0]))


def step(x, thr, flip=None):
    """x int32 [..., c] -> int8 +-1 of the same shape: +1 iff (x > thr[c]) xor flip[c]."""
    x = np.ascontiguousarray(x, dtype=np.int32)
    thr = np.ascontiguousarray(thr, dtype=np.int32)
    c = x.shape[-1]
    if thr.shape != (c,):
        raise ValueError("oracle: thr shape")
    fp = None
    if flip is not None:
        flip = np.ascontiguousarray(flip, dtype=np.uint8)
        if flip.shape != (c,):
            raise ValueError("oracle: flip shape")
        fp = _p(flip, C.c_uint8)
    out = np.empty(x.shape, dtype=np.int8)
    rows = x.size // c if c else 0
    _chk(lib().ref_step(_p(x, C.c_int32), rows, c, _p(thr, C.c_int32), fp, _p(out, C.c_int8)),
         "step")
    return out


def maxpool2(x):
    """2x2 stride-2 max over [n,h,w,c]; int32 or int8 input, same dtype out."""
    n, h, w, c = x.shape
    if x.dtype == np.int8:
        x = np.ascontiguousarray(x)
        out = np.empty((n, h // 2, w // 2, c), dtype=np.int8)
        _chk(lib().ref_maxpool2_i8(_p(x, C.c_int8), n, h, w, c, _p(out, C.c_int8)), "maxpool2")
    else:
        x = np.ascontiguousarray(x, dtype=np.int32)
        out = np.empty((n, h // 2, w // 2, c), dtype=np.int32)
        _chk(lib().ref_maxpool2_i32(_p(x, C.c_int32), n, h, w, c, _p(out, C.c_int32)),
             "maxpool2")
    return out


def run_layer(L, act, first_pad_value=-1, pool_first=False):
    """One model layer: conv/FC -> [step -> [pool]].  Returns (preact int32, act_out).

    `act` is int8: NHWC pixels for the first layer, +-1 NHWC (or [n,k]) afterwards.
    act_out is +-1 int8 (NHWC or [n,c]) for hidden layers and None for the logits layer.
    Order is step then pool (the benchmark configurations' order) unless pool_first, which
    pools the integer pre-activations and then steps (the order of the paper's Tab. I / II).
    """
    if L.kind == "fc_binary":
        a = act.reshape(act.shape[0], -1)          # flatten: (h, w, c), c fastest
        pre = fc(a, L.weights)
        pre4 = pre.reshape(pre.shape[0], 1, 1, -1)
    elif L.kind == "conv_binary":
        pre4 = conv2d(act, L.weights, 1, -1)
        pre = pre4
    else:
        pre4 = conv2d(act, L.weights, L.pad, first_pad_value)
        pre = pre4
    if not L.step:
        return pre, None
    if L.pool == 2 and pool_first:
        s = step(maxpool2(pre4), L.thr, L.flip)
    else:
        s = step(pre4, L.thr, L.flip)
        if L.pool == 2:
            s = maxpool2(s)
    return pre, s


def run_model(layers, images, first_pad_value=-1, pool_first=False):
    """Whole model.  Returns (logits int32 [n, classes], per-layer list of (preact, act))."""
    act = np.ascontiguousarray(images, dtype=np.int8)
    trace = []
    pre = None
    for L in layers:
        pre, nxt = run_layer(L, act, first_pad_value, pool_first)
        trace.append((pre, nxt))
        if nxt is not None:
            act = nxt
    logits = pre.reshape(pre.shape[0], -1)
    return logits, trace
