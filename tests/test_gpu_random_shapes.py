"""Parity on seeded random shapes: many small layers with arbitrary (ragged, odd, degenerate)
dimensions through every layer entry point, and random small models through bnn_run_model,
each against the oracle element by element.  The fixed shape lists of the other files aim at
known tile boundaries; these draws look for the ones nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import DeviceModel, dev, fill_i32, host_u32, require_gpu
from tests.helpers import pack_pm1

pytestmark = pytest.mark.gpu

FC, FIRST, CONV = W.configs.KIND_FC_BIN, W.configs.KIND_CONV_FIRST, W.configs.KIND_CONV_BIN


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()
    yield
    torch.cuda.synchronize()


def pm1(rng, shape):
    return (2 * rng.integers(0, 2, size=shape, dtype=np.int8) - 1).astype(np.int8)


def thresholds(rng, want, co, k):
    """Thresholds around the sums that occur, half of them equal to an actual sum (ties)."""
    thr = rng.integers(-(k // 4) - 1, k // 4 + 2, size=co).astype(np.int32)
    flat = want.reshape(-1, co)
    rows = rng.integers(0, flat.shape[0], size=co)
    tie = rng.integers(0, 2, size=co).astype(bool)
    thr[tie] = flat[rows, np.arange(co)][tie]
    return thr, rng.integers(0, 2, size=co).astype(np.uint8)


@pytest.mark.parametrize("seed", range(48))
def test_random_first_layers(seed):
    rng = np.random.default_rng(9000 + seed)
    kh, kw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    ci = int(rng.integers(1, 7 if seed % 4 else 20))
    pad = int(rng.integers(0, 4))
    h = int(rng.integers(max(1, kh - 2 * pad), 13))
    w = int(rng.integers(max(1, kw - 2 * pad), 13))
    n = int(rng.integers(1, 7)) if seed % 3 else int(rng.integers(30, 400))
    co = int(rng.integers(1, 100))
    padv = int(rng.integers(-128, 128))
    ho, wo = h + 2 * pad - kh + 1, w + 2 * pad - kw + 1
    print("random first", n, h, w, ci, co, kh, kw, pad, padv, flush=True)
    x = rng.integers(-128, 128, size=(n, h, w, ci), dtype=np.int8)
    wt = pm1(rng, (co, kh, kw, ci))
    want = oracle.conv2d(x, wt, pad, padv)
    xd, wd = dev(x), dev(wt)
    raw = fill_i32((n, ho, wo, co), 4242)
    P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, preact_out=raw)
    np.testing.assert_array_equal(raw.cpu().numpy(), want)
    thr, flip = thresholds(rng, want, co, kh * kw * ci * 64)
    s = oracle.step(want, thr, flip)
    packed = fill_i32((n, ho, wo, (co + 31) // 32), -1)
    P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, thr=dev(thr), flip=dev(flip), packed_out=packed)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(s))
    if ho % 2 == 0 and wo % 2 == 0:
        for pool_first, ref in ((0, oracle.maxpool2(s)), (1, oracle.step(oracle.maxpool2(want), thr, flip))):
            pk = fill_i32((n, ho // 2, wo // 2, (co + 31) // 32), -1)
            P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, thr=dev(thr), flip=dev(flip),
                                  pool=2, pool_first=pool_first, packed_out=pk)
            np.testing.assert_array_equal(host_u32(pk), pack_pm1(ref), err_msg=f"pool_first {pool_first}")


@pytest.mark.parametrize("seed", range(40))
def test_random_binary_convs(seed):
    rng = np.random.default_rng(9100 + seed)
    ci = int(rng.choice([64, 128, 256, 512])) if seed % 2 else int(rng.integers(1, 300))
    co = int(rng.integers(1, 140))
    h, w = int(rng.integers(1, 12)), int(rng.integers(1, 12))
    n = int(rng.integers(1, 5)) if seed % 5 else int(rng.integers(20, 120))
    print("random conv", n, h, w, ci, co, flush=True)
    x, wt = pm1(rng, (n, h, w, ci)), pm1(rng, (co, 3, 3, ci))
    want = oracle.conv2d(x, wt, 1, -1)
    cw = (ci + 31) // 32
    xd = dev(pack_pm1(x))
    wd = dev(pack_pm1(wt.reshape(co * 9, ci)).reshape(co, 3, 3, cw))
    raw = fill_i32((n, h, w, co), 4242)
    P.bnn_conv_binary(xd, n, h, w, ci, wd, co, preact_out=raw)
    np.testing.assert_array_equal(raw.cpu().numpy(), want)
    thr, flip = thresholds(rng, want, co, 9 * ci)
    s = oracle.step(want, thr, flip)
    packed = fill_i32((n, h, w, (co + 31) // 32), -1)
    P.bnn_conv_binary(xd, n, h, w, ci, wd, co, thr=dev(thr), flip=dev(flip), packed_out=packed)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(s))
    if h % 2 == 0 and w % 2 == 0:
        for pool_first, ref in ((0, oracle.maxpool2(s)), (1, oracle.step(oracle.maxpool2(want), thr, flip))):
            pk = fill_i32((n, h // 2, w // 2, (co + 31) // 32), -1)
            P.bnn_conv_binary(xd, n, h, w, ci, wd, co, thr=dev(thr), flip=dev(flip), pool=2, pool_first=pool_first,
                              packed_out=pk)
            np.testing.assert_array_equal(host_u32(pk), pack_pm1(ref), err_msg=f"pool_first {pool_first}")


@pytest.mark.parametrize("seed", range(40))
def test_random_fc(seed):
    rng = np.random.default_rng(9200 + seed)
    m = int(rng.integers(1, 9)) if seed % 3 == 0 else int(rng.integers(9, 300))
    n, k = int(rng.integers(1, 400)), int(rng.integers(1, 3000))
    print("random fc", m, n, k, flush=True)
    a, b = pm1(rng, (m, k)), pm1(rng, (n, k))
    want = oracle.fc(a, b)
    ad, bd = dev(pack_pm1(a)), dev(pack_pm1(b))
    c = fill_i32((m, n), 4242)
    thr, flip = thresholds(rng, want, n, k)
    packed = fill_i32((m, (n + 31) // 32), -1)
    P.bnn_fc_binary(ad, m, k, bd, n, thr=dev(thr), flip=dev(flip), c_out=c, packed_out=packed)
    np.testing.assert_array_equal(c.cpu().numpy(), want)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(oracle.step(want, thr, flip)))


@pytest.mark.parametrize("seed", range(24))
def test_random_models(seed):
    """first layer (3x3 or 1x1) -> up to two binary convs -> one to three FC layers, random widths and
    batch (1 .. 40): logits and every layer's outputs in STREAM mode, logits in TIMED and GRAPH mode."""
    rng = np.random.default_rng(9300 + seed)
    batch = int(rng.integers(1, 9)) if seed % 2 else int(rng.integers(9, 41))
    layers = []
    if seed % 3 == 0:                                   # all-FC model on a flat int8 vector
        in_shape = (1, 1, int(rng.integers(1, 8)) * 16)
        c = int(rng.integers(1, 300))
        layers.append(W.Layer(FIRST, in_shape[2], c, 1, 1, 0))
    else:
        hw = int(rng.choice([4, 8, 12]))
        in_shape = (hw, hw, int(rng.integers(1, 4)))
        c = int(rng.choice([32, 64, 96, 128]))
        pool = int(rng.choice([1, 2]))
        layers.append(W.Layer(FIRST, in_shape[2], c, 3, 3, 1, pool=pool))
        hw //= pool
        for _ in range(int(rng.integers(0, 3))):
            c2 = int(rng.choice([32, 64, 128]))
            pool = int(rng.choice([1, 2])) if hw % 2 == 0 and hw >= 4 else 1
            layers.append(W.Layer(CONV, c, c2, 3, 3, 1, pool=pool))
            c, hw = c2, hw // pool
        c = hw * hw * c
    for _ in range(int(rng.integers(0, 3))):
        c2 = int(rng.integers(1, 1200))
        layers.append(W.Layer(FC, c, c2))
        c = c2
    layers.append(W.Layer(FC, c, int(rng.integers(1, 40)), step=False))
    print("random model batch", batch, in_shape, [(L.kind, L.c_in, L.c_out, L.pool) for L in layers], flush=True)
    cid = 400 + seed
    layers = W.build_model(layers, *in_shape, cid)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    logits, trace = oracle.run_model(layers, imgs)
    dm = DeviceModel(layers, batch, in_shape, taps=True)
    xd = dev(imgs)
    for mode in (P.RUN_STREAM, P.RUN_TIMED, P.RUN_GRAPH, P.RUN_GRAPH):
        dm.logits.fill_(77)
        dm.run(xd, mode)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits, err_msg=f"mode {mode}")
        if mode == P.RUN_STREAM:
            for li, (pre, act) in enumerate(trace):
                np.testing.assert_array_equal(dm.preact_taps[li].cpu().numpy().reshape(pre.shape), pre,
                                              err_msg=f"layer {li} pre-activations")
                if act is not None:
                    want = pack_pm1(act)
                    np.testing.assert_array_equal(host_u32(dm.packed_taps[li]).reshape(want.shape), want,
                                                  err_msg=f"layer {li} bits")
