"""GPU parity: every entry point of libbnn, called through the C ABI, against the CPU
oracle on the same seeded inputs.  All comparisons are bit-exact (integer path)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import (DEV, DeviceModel, conv_binary_tiles, dev, empty_i32, fill_i32, host_u32,
                            pack_on_gpu, require_gpu)
from tests.helpers import pack_pm1

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()
    yield
    torch.cuda.synchronize()


def rng_of(seed):
    return np.random.default_rng(seed)


def pm1(rng, shape):
    return (2 * rng.integers(0, 2, size=shape, dtype=np.int8) - 1).astype(np.int8)


# ------------------------------------------------------------------------ pack_bits
@pytest.mark.parametrize("rows,k", [(1, 1), (3, 32), (5, 64), (7, 70), (2, 33), (130, 1152),
                                    (4, 8192), (1000, 96), (257, 1000), (0, 64)])
def test_pack_bits(rows, k):
    print("pack_bits", rows, k, flush=True)
    a = pm1(rng_of(rows * 131 + k), (rows, k))
    got = host_u32(pack_on_gpu(a)) if rows else np.zeros((0, (k + 31) // 32), np.uint32)
    if rows == 0:
        P.bnn_pack_bits(dev(np.zeros(16, np.int8)), 0, k, empty_i32(4))
    np.testing.assert_array_equal(got, pack_pm1(a))


def test_pack_bits_general_int8_values():
    # an element is +1 iff it is > 0: zeros and -128 give bit 0
    rng = rng_of(5)
    for k in (64, 50):
        a = rng.integers(-128, 128, size=(33, k), dtype=np.int8)
        a[0, :8] = [0, 1, -1, 127, -128, 0, 2, -2]
        np.testing.assert_array_equal(host_u32(pack_on_gpu(a)), pack_pm1(a))


# --------------------------------------------------------------- threshold/sign/pool
@pytest.mark.parametrize("n,h,w,c", [(2, 4, 6, 8), (1, 2, 2, 3), (3, 6, 6, 40), (2, 8, 8, 64),
                                     (1, 28, 28, 64), (2, 4, 4, 33), (1, 16, 16, 256), (5, 2, 2, 130)])
@pytest.mark.parametrize("pool", [1, 2])
@pytest.mark.parametrize("use_flip", [False, True])
def test_threshold_sign_maxpool(n, h, w, c, pool, use_flip):
    print("step", n, h, w, c, pool, use_flip, flush=True)
    rng = rng_of(n * 7 + h * 11 + c * 13 + pool)
    x = rng.integers(-40, 41, size=(n, h, w, c)).astype(np.int32)
    thr = rng.integers(-10, 11, size=c).astype(np.int32)
    x[0, 0, 0, :] = thr                      # exact ties
    x[0, h - 1, w - 1, :] = thr + 1
    flip = rng.integers(0, 2, size=c).astype(np.uint8) if use_flip else None
    out = fill_i32((n, h // pool, w // pool, (c + 31) // 32), -1)
    P.bnn_threshold_sign_maxpool(dev(x), n, h, w, c, dev(thr), dev(flip) if use_flip else None, pool, out)
    s = oracle.step(x, thr, flip)
    if pool == 2:
        s = oracle.maxpool2(s)
    np.testing.assert_array_equal(host_u32(out), pack_pm1(s))
    if pool == 2:
        # the paper's order: pool the integers, then step
        out2 = fill_i32((n, h // 2, w // 2, (c + 31) // 32), -1)
        P.bnn_threshold_sign_maxpool(dev(x), n, h, w, c, dev(thr), dev(flip) if use_flip else None, 2, out2,
                                     pool_first=1)
        np.testing.assert_array_equal(host_u32(out2), pack_pm1(oracle.step(oracle.maxpool2(x), thr, flip)))


# ------------------------------------------------------------------------- fc_binary
FC_SHAPES = [(1, 8, 32), (1, 33, 70), (3, 100, 96), (8, 40, 3136), (9, 130, 64), (64, 512, 512),
             (64, 10, 512), (200, 300, 1000), (129, 257, 4100), (256, 2048, 3136), (1, 1024, 8192),
             (130, 128, 128), (300, 10, 1024),
             # small problems with K beyond one round of the K-split kernel (more than 32 units of 256 bits)
             (40, 70, 20000), (33, 64, 16896), (256, 1024, 8192),
             # many whole tiles of the largest block shapes, 1 to 5 K chunks
             (2048, 1536, 512), (2048, 1536, 1536), (1920, 1664, 1024), (4096, 3072, 1024), (4096, 3072, 2560)]


@pytest.mark.parametrize("m,n,k", FC_SHAPES)
def test_fc_binary_raw_and_fused(m, n, k):
    print("fc", m, n, k, flush=True)
    rng = rng_of(m * 3 + n * 5 + k)
    a, b = pm1(rng, (m, k)), pm1(rng, (n, k))
    want = oracle.fc(a, b)
    ad, bd = dev(pack_pm1(a)), dev(pack_pm1(b))
    c = fill_i32((m, n), 123456)
    P.bnn_fc_binary(ad, m, k, bd, n, c_out=c)
    np.testing.assert_array_equal(c.cpu().numpy(), want)
    # fused epilogue, with ties planted: thresholds taken from actual outputs of row 0
    thr = rng.integers(-(k // 8), k // 8 + 1, size=n).astype(np.int32)
    thr[: n // 2] = want[0, : n // 2]
    flip = rng.integers(0, 2, size=n).astype(np.uint8)
    c2 = fill_i32((m, n), 123456)
    packed = fill_i32((m, (n + 31) // 32), -1)
    P.bnn_fc_binary(ad, m, k, bd, n, thr=dev(thr), flip=dev(flip), c_out=c2, packed_out=packed)
    np.testing.assert_array_equal(c2.cpu().numpy(), want)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(oracle.step(want, thr, flip)))
    # packed only, no flips
    packed2 = fill_i32((m, (n + 31) // 32), -1)
    P.bnn_fc_binary(ad, m, k, bd, n, thr=dev(thr), packed_out=packed2)
    np.testing.assert_array_equal(host_u32(packed2), pack_pm1(oracle.step(want, thr, None)))


def test_fc_binary_with_gpu_packed_operands_and_empty_batch():
    rng = rng_of(77)
    a, b = pm1(rng, (70, 777)), pm1(rng, (90, 777))
    c = fill_i32((70, 90), 5)
    P.bnn_fc_binary(pack_on_gpu(a), 70, 777, pack_on_gpu(b), 90, c_out=c)
    np.testing.assert_array_equal(c.cpu().numpy(), oracle.fc(a, b))
    P.bnn_fc_binary(pack_on_gpu(a), 0, 777, pack_on_gpu(b), 90, c_out=c)     # m == 0: no-op
    np.testing.assert_array_equal(c.cpu().numpy(), oracle.fc(a, b))


# ----------------------------------------------------------------------- conv_binary
CONV_SHAPES = [(1, 4, 4, 32, 8, 1), (2, 8, 8, 64, 64, 2), (3, 14, 14, 64, 64, 2), (2, 16, 16, 128, 256, 1),
               (1, 32, 32, 128, 128, 2), (2, 8, 8, 256, 512, 1), (5, 8, 8, 512, 512, 2), (1, 5, 7, 32, 40, 1),
               (2, 3, 3, 96, 130, 1), (1, 1, 1, 32, 32, 1), (3, 2, 2, 64, 16, 2), (2, 6, 6, 40, 24, 1),
               (3, 4, 4, 512, 512, 2), (1, 20, 36, 128, 64, 2), (17, 4, 4, 128, 128, 1),
               (2, 4, 4, 1024, 64, 2), (1, 6, 6, 608, 96, 1), (40, 8, 8, 256, 256, 2), (2, 2, 6, 32, 300, 1),
               (600, 2, 2, 64, 64, 2), (9, 16, 16, 64, 128, 2),
               # ragged pixel tiles and channel tiles with C_in a multiple of 64 (small-problem kernel)
               (1, 5, 7, 64, 40, 1), (2, 6, 10, 128, 96, 2), (1, 3, 9, 256, 33, 1), (3, 2, 18, 64, 70, 2),
               # exactly at and just past the small-problem kernel's limit of 1024 tiles
               (128, 8, 8, 64, 128, 2), (129, 8, 8, 64, 128, 1)]


def extreme_thresholds(thr, room, k):
    """Overwrite up to `room` trailing thresholds with values at and beyond the range of a sum."""
    big = [np.iinfo(np.int32).max, np.iinfo(np.int32).min, k, -k, k - 1, -k - 1, k + 1, -k + 1]
    for q, v in enumerate(big[:room]):
        thr[len(thr) - 1 - q] = v


def conv_weights_packed(wt):
    co, _, _, ci = wt.shape
    return pack_pm1(wt.reshape(co * 9, ci)).reshape(co, 3, 3, (ci + 31) // 32)


@pytest.mark.parametrize("path", ["auto", "tiles"])
@pytest.mark.parametrize("n,h,w,ci,co,pool", CONV_SHAPES)
def test_conv_binary_raw_and_fused(n, h, w, ci, co, pool, path):
    # "auto": bnn_conv_binary as the library dispatches it; "tiles": the persistent tile kernels
    # also for shapes that the library would send to its small-problem kernel (test hook)
    conv = P.bnn_conv_binary if path == "auto" else conv_binary_tiles
    print("conv", path, n, h, w, ci, co, pool, flush=True)
    rng = rng_of(n + h * 3 + w * 5 + ci * 7 + co * 11)
    x, wt = pm1(rng, (n, h, w, ci)), pm1(rng, (co, 3, 3, ci))
    want = oracle.conv2d(x, wt, 1, -1)
    xd, wd = dev(pack_pm1(x)), dev(conv_weights_packed(wt))
    raw = fill_i32((n, h, w, co), 99999)
    conv(xd, n, h, w, ci, wd, co, preact_out=raw)
    np.testing.assert_array_equal(raw.cpu().numpy(), want)
    k = 9 * ci
    thr = rng.integers(-(k // 8), k // 8 + 1, size=co).astype(np.int32)
    thr[: co // 2] = want[0, 0, 0, : co // 2]         # ties at one pixel
    extreme_thresholds(thr, co - co // 2, k)
    flip = rng.integers(0, 2, size=co).astype(np.uint8)
    s = oracle.step(want, thr, flip)
    if pool == 2:
        s = oracle.maxpool2(s)
    raw2 = fill_i32((n, h, w, co), 99999)
    packed = fill_i32((n, h // pool, w // pool, (co + 31) // 32), -1)
    conv(xd, n, h, w, ci, wd, co, thr=dev(thr), flip=dev(flip), pool=pool, preact_out=raw2, packed_out=packed)
    np.testing.assert_array_equal(raw2.cpu().numpy(), want)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(s))
    packed2 = fill_i32((n, h // pool, w // pool, (co + 31) // 32), -1)
    conv(xd, n, h, w, ci, wd, co, thr=dev(thr), flip=dev(flip), pool=pool, packed_out=packed2)
    np.testing.assert_array_equal(host_u32(packed2), pack_pm1(s))
    if pool == 2:
        packed3 = fill_i32((n, h // 2, w // 2, (co + 31) // 32), -1)
        conv(xd, n, h, w, ci, wd, co, thr=dev(thr), flip=dev(flip), pool=2, pool_first=1, packed_out=packed3)
        np.testing.assert_array_equal(host_u32(packed3),
                                      pack_pm1(oracle.step(oracle.maxpool2(want), thr, flip)))


def test_conv_binary_rejects_too_many_channels():
    x = fill_i32((1, 4, 4, 40), 0)
    w = fill_i32((32, 3, 3, 40), 0)
    out = fill_i32((1, 4, 4, 32), 0)
    with pytest.raises(P.BnnError) as e:
        P.bnn_conv_binary(x, 1, 4, 4, 1280, w, 32, preact_out=out)
    assert e.value.status == 4      # BNN_ERR_UNSUPPORTED


def test_conv_binary_closed_form_borders():
    # all-(+1) input and weights: 9C interior, 3C on an edge, -C at a corner (padding is -1)
    n, h, w, c, co = 1, 6, 5, 64, 32
    x = np.ones((n, h, w, c), np.int8)
    wt = np.ones((co, 3, 3, c), np.int8)
    raw = empty_i32(n, h, w, co)
    P.bnn_conv_binary(dev(pack_pm1(x)), n, h, w, c, dev(conv_weights_packed(wt)), co, preact_out=raw)
    r = raw.cpu().numpy()
    assert r[0, 2, 2, 0] == 9 * c and r[0, 0, 2, 0] == 3 * c and r[0, 0, 0, 0] == -c
    assert r[0, h - 1, w - 1, co - 1] == -c


# ------------------------------------------------------------------- conv_first_int8
FIRST_SHAPES = [(2, 28, 28, 1, 64, 3, 3, 1, -1, 2), (2, 32, 32, 3, 128, 3, 3, 1, -1, 1),
                (64, 1, 1, 784, 512, 1, 1, 0, -1, 1), (3, 8, 8, 3, 32, 3, 3, 1, 0, 2),
                (1, 5, 7, 2, 40, 3, 3, 1, 7, 1), (2, 6, 6, 3, 33, 5, 3, 2, -1, 2),
                (1, 4, 4, 4, 8, 1, 1, 0, -1, 1), (300, 2, 2, 5, 70, 3, 3, 1, -1, 2),
                # one K step (two kernel rows), two channel groups; four full kernel rows with a ragged
                # second channel tile; kernel rows wider than 16 bytes with a patch beyond 1 KB
                (2, 9, 9, 2, 96, 2, 2, 0, -1, 1), (1, 16, 16, 4, 130, 4, 4, 1, -1, 1),
                (2, 12, 12, 8, 64, 3, 3, 1, 3, 2),
                # padding wider than a signed byte (tile-relative coordinates down to -200 / -130)
                (1, 300, 4, 1, 8, 3, 3, 200, -1, 2), (1, 6, 6, 2, 16, 3, 3, 130, 3, 1),
                # 1x1 layer with exactly one 16-byte slice per row (K = 16), last row included
                (3, 1, 1, 16, 40, 1, 1, 0, -1, 1), (70, 1, 1, 16, 64, 1, 1, 0, -1, 1),
                (5, 1, 1, 48, 33, 1, 1, 0, -1, 1),
                # 3x3 over small power-of-two-wide images (whole images in LDS): one and two channel
                # groups per block, several images per tile with a ragged last group, several tiles and
                # several work units per block, image groups of 4 / 8 KB (16 KB: the general kernel), every pad value
                (5, 32, 32, 3, 128, 3, 3, 1, -1, 1), (70, 32, 32, 3, 128, 3, 3, 1, 7, 2),
                (9, 16, 16, 4, 64, 3, 3, 1, 0, 2), (33, 8, 8, 1, 40, 3, 3, 1, -1, 1),
                (3, 64, 32, 3, 96, 3, 3, 1, 3, 1), (2, 128, 128, 1, 32, 3, 3, 1, -1, 2),
                (300, 4, 4, 2, 16, 3, 3, 1, -1, 2), (1100, 32, 32, 3, 128, 3, 3, 1, -1, 1),
                (1300, 16, 16, 3, 64, 3, 3, 1, -128, 2),
                # weight tensor of 33 * 27 = 891 bytes (not a whole number of dwords), ragged channel tile
                (6, 8, 8, 3, 33, 3, 3, 1, 5, 1),
                # up to 6144 tiles of 32 pixels x 32 channels the one-wave kernel runs (most shapes above with
                # few images); its own edges: padding wider than the image, 4x4 kernel with 16-byte rows, 1x1
                # with pooling, input and weight tensors that are not whole numbers of dwords, one pixel
                (1, 2, 2, 1, 8, 3, 3, 20, -1, 1), (2, 4, 4, 16, 40, 1, 1, 0, -1, 2),
                (3, 5, 5, 1, 20, 3, 3, 1, -5, 1), (1, 1, 1, 3, 5, 1, 1, 0, -1, 1),
                (8, 32, 32, 3, 128, 3, 3, 1, -1, 1), (8, 28, 28, 1, 64, 3, 3, 1, -1, 2),
                (1, 3, 90, 2, 70, 2, 7, 3, 9, 2), (48, 32, 32, 3, 128, 3, 3, 1, -1, 1),
                # the same layers with enough images (more than 6144 such tiles) for the staged kernels
                (130, 28, 28, 1, 64, 3, 3, 1, -1, 2), (3100, 8, 8, 3, 32, 3, 3, 1, 0, 2),
                (2900, 5, 7, 2, 40, 3, 3, 1, 7, 1), (16500, 2, 2, 5, 70, 3, 3, 1, -1, 2),
                (1100, 9, 9, 2, 96, 2, 2, 0, -1, 1), (180, 16, 16, 4, 130, 4, 4, 1, -1, 1),
                (400, 16, 16, 4, 64, 3, 3, 1, 0, 2), (1600, 8, 8, 1, 40, 3, 3, 1, -1, 1),
                (34, 64, 32, 3, 96, 3, 3, 1, 3, 1), (12400, 4, 4, 2, 16, 3, 3, 1, -1, 2),
                (1600, 8, 8, 3, 33, 3, 3, 1, 5, 1), (50, 32, 32, 3, 128, 3, 3, 1, -1, 1),
                (3, 6, 6, 2, 16, 3, 3, 130, 3, 1), (9, 128, 128, 1, 32, 3, 3, 1, -1, 2),
                # 1x1 layers: below 192 blocks of 64 x 64 the K-split kernel runs (the shapes further up, and
                # K over two rounds of eight steps per wave, ragged rows and channels); above, the plain one
                (70, 1, 1, 1072, 96, 1, 1, 0, -1, 1), (33, 1, 1, 784, 100, 1, 1, 0, -1, 1),
                (12300, 1, 1, 16, 40, 1, 1, 0, -1, 1), (12300, 1, 1, 48, 33, 1, 1, 0, -1, 1),
                (2000, 1, 1, 784, 512, 1, 1, 0, -1, 1)]


@pytest.mark.parametrize("n,h,w,ci,co,kh,kw,pad,padv,pool", FIRST_SHAPES)
def test_conv_first_int8(n, h, w, ci, co, kh, kw, pad, padv, pool):
    print("first", n, h, w, ci, co, kh, kw, pad, padv, pool, flush=True)
    rng = rng_of(n + h * 3 + ci * 7 + co * 11 + kh)
    x = rng.integers(-127, 128, size=(n, h, w, ci), dtype=np.int8)
    x[0, 0, 0, 0] = -128
    wt = pm1(rng, (co, kh, kw, ci))
    want = oracle.conv2d(x, wt, pad, padv)
    ho, wo = want.shape[1], want.shape[2]
    xd, wd = dev(x), dev(wt)
    raw = fill_i32((n, ho, wo, co), 99999)
    P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, preact_out=raw)
    np.testing.assert_array_equal(raw.cpu().numpy(), want)
    k = kh * kw * ci
    thr = rng.integers(-(k // 8), k // 8 + 1, size=co).astype(np.int32)
    thr[: co // 2] = want[0, 0, 0, : co // 2]
    extreme_thresholds(thr, co - co // 2, 128 * k)
    flip = rng.integers(0, 2, size=co).astype(np.uint8)
    s = oracle.step(want, thr, flip)
    if pool == 2:
        s = oracle.maxpool2(s)
    raw2 = fill_i32((n, ho, wo, co), 99999)
    packed = fill_i32((n, ho // pool, wo // pool, (co + 31) // 32), -1)
    P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, thr=dev(thr), flip=dev(flip),
                          pool=pool, preact_out=raw2, packed_out=packed)
    np.testing.assert_array_equal(raw2.cpu().numpy(), want)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(s))
    if pool == 2:
        packed3 = fill_i32((n, ho // 2, wo // 2, (co + 31) // 32), -1)
        P.bnn_conv_first_int8(xd, n, h, w, ci, wd, co, kh, kw, pad, padv, thr=dev(thr), flip=dev(flip),
                              pool=2, pool_first=1, packed_out=packed3)
        np.testing.assert_array_equal(host_u32(packed3),
                                      pack_pm1(oracle.step(oracle.maxpool2(want), thr, flip)))


# ------------------------------------------------------------------------- run_model
def check_model(name, batch, modes):
    cid, layers, in_shape = W.model_by_name(name)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    logits, trace = oracle.run_model(layers, imgs)
    dm = DeviceModel(layers, batch, in_shape, taps=True)
    xd = dev(imgs)
    for mode in modes:
        print("model", name, batch, "mode", mode, flush=True)
        dm.logits.fill_(-9)
        t = dm.run(xd, mode)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits)
        if mode == P.RUN_TIMED:
            assert len(t) == len(layers)
            assert all(x.gpu_us > 0 for x in t)
            assert sum(x.macs for x in t) == batch * (W.model_binary_macs(layers) + W.model_int8_macs(layers))
        if mode != P.RUN_GRAPH:
            for li, (pre, act) in enumerate(trace):
                got_pre = dm.preact_taps[li].cpu().numpy().reshape(pre.shape)
                np.testing.assert_array_equal(got_pre, pre, err_msg=f"layer {li} pre-activations")
                if act is not None:
                    want = pack_pm1(act)
                    got = host_u32(dm.packed_taps[li]).reshape(want.shape)
                    np.testing.assert_array_equal(got, want, err_msg=f"layer {li} packed activations")
    return dm, xd, logits


@pytest.mark.parametrize("name,batch", [("mlp", 64), ("small_cnn", 1), ("small_cnn", 5), ("small_cnn", 256),
                                        ("vgg_small", 1), ("vgg_small", 3), ("vgg_small", 32),
                                        # batch 64: the first layer takes two channel groups per block
                                        ("vgg_small", 64)])
def test_run_model_layer_by_layer(name, batch):
    check_model(name, batch, [P.RUN_TIMED, P.RUN_STREAM])


@pytest.mark.parametrize("name,batch", [("small_cnn", 1), ("vgg_small", 1), ("vgg_small", 4)])
def test_run_model_graph_replays(name, batch):
    dm, xd, logits = check_model(name, batch, [P.RUN_STREAM, P.RUN_GRAPH])
    # replay several times with eager work and synchronisations in between
    for it in range(4):
        dm.logits.fill_(-9)
        junk = torch.arange(1000, device=DEV).sum().item()
        assert junk == 499500
        dm.run(xd, P.RUN_GRAPH)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits, err_msg=f"replay {it}")


@pytest.mark.parametrize("name,batch", [("small_cnn", 6), ("vgg_small", 3)])
def test_run_model_paper_layer_order(name, batch):
    # C -> MP -> S as in the paper's model tables: pool the integers, then step
    cid, layers, in_shape = W.model_by_name(name)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    logits, trace = oracle.run_model(layers, imgs, pool_first=True)
    logits_sp, _ = oracle.run_model(layers, imgs)
    assert not np.array_equal(logits, logits_sp)          # the two orders differ on flipped channels
    dm = DeviceModel(layers, batch, in_shape, taps=True, pool_first=True)
    dm.run(dev(imgs), P.RUN_STREAM)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits)
    for li, (pre, act) in enumerate(trace):
        if act is not None:
            want = pack_pm1(act)
            np.testing.assert_array_equal(host_u32(dm.packed_taps[li]).reshape(want.shape), want)


def test_run_model_golden_logits():
    import os
    for name in ("mlp", "small_cnn", "vgg_small"):
        path = os.path.join(os.path.dirname(__file__), "golden", f"{name}_logits.txt")
        want = np.loadtxt(path, dtype=np.int64, comments="#", ndmin=2)
        cid, layers, in_shape = W.model_by_name(name)
        imgs = W.draw_images(W.rng_for(cid, 0, 0), want.shape[0], *in_shape)
        dm = DeviceModel(layers, want.shape[0], in_shape)
        dm.run(dev(imgs), P.RUN_STREAM)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), want)


def test_run_model_host_callback_and_table():
    cid, layers, in_shape = W.model_by_name("small_cnn")
    imgs = W.draw_images(W.rng_for(cid, 0, 0), 8, *in_shape)
    dm = DeviceModel(layers, 8, in_shape)
    state = {"act": imgs, "calls": []}

    def host(layer):
        pre, nxt = oracle.run_layer(layers[layer], state["act"])
        state["calls"].append(layer)
        if nxt is not None:
            state["act"] = nxt
        else:
            state["logits"] = pre

    t = dm.run(dev(imgs), P.RUN_TIMED, host_fn=host)
    assert state["calls"] == [0, 1, 2, 3]
    assert all(x.host_us > 0 and x.gpu_us > 0 and x.bytes_algorithmic > 0 for x in t)
    np.testing.assert_array_equal(dm.logits.cpu().numpy(), state["logits"].reshape(8, 10))
