"""Pins for the CPU oracle: everything here checks oracle/ against something that is not
the oracle -- the paper's neuron identity evaluated on Python integers, brute force,
closed forms, exact numpy int64 products, and invariants.  CPU only."""
import itertools

import numpy as np
import pytest

import oracle
from tests.helpers import pack_pm1

RNG = np.random.default_rng(12345)


def pm1(shape, rng=RNG):
    return (2 * rng.integers(0, 2, size=shape, dtype=np.int8) - 1).astype(np.int8)


# ----------------------------------------------------------------------------- neuron
def _to_pyint(row):
    """+-1 vector -> Python int with bit t = 1 iff row[t] == +1 (independent packing)."""
    v = 0
    for t, x in enumerate(row):
        if x > 0:
            v |= 1 << t
    return v


@pytest.mark.parametrize("k", [1, 2, 31, 32, 33, 64, 100, 577, 1152])
def test_dot_equals_paper_popcount_identity(k):
    # Sec. II-A neuron formula: dot = 2*popcount(xnor(W, I)) - #bits.
    a, w = pm1((5, k)), pm1((7, k))
    got = oracle.fc(a, w)
    mask = (1 << k) - 1
    for r in range(5):
        ai = _to_pyint(a[r])
        for o in range(7):
            wi = _to_pyint(w[o])
            xnor = ~(ai ^ wi) & mask
            assert got[r, o] == 2 * bin(xnor).count("1") - k
            assert oracle.dot(a[r], w[o]) == got[r, o]


@pytest.mark.parametrize("k", [1, 3, 8, 11])
def test_fc_brute_force_all_inputs(k):
    # every one of the 2^k input vectors against a few weight rows; expected value is
    # (#positions that agree) - (#positions that disagree), counted in plain Python.
    rows = np.array(list(itertools.product([-1, 1], repeat=k)), dtype=np.int8)
    w = pm1((4, k))
    got = oracle.fc(rows, w)
    for r in range(rows.shape[0]):
        for o in range(4):
            agree = sum(1 for t in range(k) if rows[r, t] == w[o, t])
            assert got[r, o] == agree - (k - agree)


def test_fc_matches_numpy_int64_nonsquare():
    # m != n != k so a transposed operand or swapped index cannot pass.
    a, w = pm1((13, 71)), pm1((29, 71))
    want = a.astype(np.int64) @ w.astype(np.int64).T
    np.testing.assert_array_equal(oracle.fc(a, w), want)
    # int8 (non +-1) activations, as used by the first layer of the MLP
    a8 = RNG.integers(-127, 128, size=(9, 784), dtype=np.int8)
    w8 = pm1((17, 784))
    np.testing.assert_array_equal(oracle.fc(a8, w8), a8.astype(np.int64) @ w8.astype(np.int64).T)


def test_fc_invariants():
    k = 96
    a, w = pm1((6, k)), pm1((10, k))
    x = oracle.fc(a, w)
    assert np.all((x - k) % 2 == 0)              # x == K (mod 2)
    assert np.all(np.abs(x) <= k)
    np.testing.assert_array_equal(oracle.fc(a, -w), -x)       # negate weights
    np.testing.assert_array_equal(oracle.fc(-a, -w), x)       # negate both
    np.testing.assert_array_equal(oracle.fc(a, a), a.astype(np.int64) @ a.astype(np.int64).T)
    assert np.all(np.diag(oracle.fc(a, a)) == k)              # self dot = K


# ------------------------------------------------------------------------------- conv
def _np_conv(x, wt, pad, pad_value):
    """Independent formulation: explicit padding + sliding windows + einsum in int64."""
    n, h, w, c = x.shape
    co, kh, kw, _ = wt.shape
    xp = np.pad(x.astype(np.int64), ((0, 0), (pad, pad), (pad, pad), (0, 0)),
                constant_values=pad_value)
    win = np.lib.stride_tricks.sliding_window_view(xp, (kh, kw), axis=(1, 2))  # n,ho,wo,c,kh,kw
    return np.einsum("nyxcij,oijc->nyxo", win, wt.astype(np.int64))


@pytest.mark.parametrize("h,w,c,co", [(5, 7, 3, 4), (1, 1, 2, 3), (2, 2, 5, 2), (8, 3, 33, 5)])
@pytest.mark.parametrize("pad_value", [-1, 0, 7])
def test_conv3x3_matches_numpy(h, w, c, co, pad_value):
    x = pm1((2, h, w, c))
    wt = pm1((co, 3, 3, c))
    np.testing.assert_array_equal(oracle.conv2d(x, wt, 1, pad_value), _np_conv(x, wt, 1, pad_value))


def test_conv_generic_kernel_shapes_and_int8_input():
    x = RNG.integers(-127, 128, size=(3, 6, 5, 3), dtype=np.int8)
    for kh, kw, pad in [(1, 1, 0), (3, 3, 1), (3, 1, 1), (1, 3, 0), (5, 3, 2)]:
        wt = pm1((6, kh, kw, 3))
        got = oracle.conv2d(x, wt, pad, -1)
        want = _np_conv(x, wt, pad, -1)
        assert got.shape == want.shape
        np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("c", [1, 3, 64])
def test_conv_closed_form_constant_inputs(c):
    # all-(+1) input and weights with -1 padding: x = C*(2t - 9), t = taps inside the image
    h, w = 6, 5
    ones = np.ones((1, h, w, c), np.int8)
    wt = np.ones((2, 3, 3, c), np.int8)
    x = oracle.conv2d(ones, wt, 1, -1)
    for y in range(h):
        for xx in range(w):
            ty = 3 - (y == 0) - (y == h - 1)
            tx = 3 - (xx == 0) - (xx == w - 1)
            t = ty * tx
            assert np.all(x[0, y, xx] == c * (2 * t - 9)), (y, xx)
    assert x[0, 2, 2, 0] == 9 * c and x[0, 0, 2, 0] == 3 * c and x[0, 0, 0, 0] == -c
    # all-(-1) input: padding is indistinguishable from data
    x = oracle.conv2d(-ones, wt, 1, -1)
    assert np.all(x == -9 * c)
    # constant int8 image v, +1 weights, pad p: v*t*C + p*(9-t)*C
    v, p = 37, -1
    x = oracle.conv2d((v * ones).astype(np.int8), wt, 1, p)
    assert x[0, 2, 2, 0] == v * 9 * c
    assert x[0, 0, 2, 0] == v * 6 * c + p * 3 * c
    assert x[0, 0, 0, 0] == v * 4 * c + p * 5 * c
    x0 = oracle.conv2d((v * ones).astype(np.int8), wt, 1, 0)
    assert x0[0, 0, 0, 0] == v * 4 * c


def test_conv_tap_orientation():
    # a single +1 weight tap at (i, j) (others -1) on an impulse image tells apart
    # correlation from flipped convolution and a swapped (kh, kw) index.
    h = w = 5
    img = np.zeros((1, h, w, 1), np.int8)
    img[0, 2, 3, 0] = 10
    for i in range(3):
        for j in range(3):
            wt = np.zeros((1, 3, 3, 1), np.int8)
            wt[0, i, j, 0] = 1
            x = oracle.conv2d(img, wt, 1, 0)
            # out[y, x] = in[y+i-1, x+j-1] -> the impulse shows up at (2-i+1, 3-j+1)
            yy, xx = 2 - i + 1, 3 - j + 1
            want = np.zeros((h, w), np.int64)
            if 0 <= yy < h and 0 <= xx < w:
                want[yy, xx] = 10
            np.testing.assert_array_equal(x[0, :, :, 0], want)


def test_conv_linearity_int8():
    a = RNG.integers(-60, 61, size=(2, 7, 7, 3), dtype=np.int8)
    b = RNG.integers(-60, 61, size=(2, 7, 7, 3), dtype=np.int8)
    wt = pm1((8, 3, 3, 3))
    s = oracle.conv2d((a + b).astype(np.int8), wt, 1, 0)
    np.testing.assert_array_equal(s, oracle.conv2d(a, wt, 1, 0) + oracle.conv2d(b, wt, 1, 0))


def test_1x1_conv_equals_fc():
    x = RNG.integers(-127, 128, size=(6, 1, 1, 784), dtype=np.int8)
    wt = pm1((32, 784))
    got = oracle.conv2d(x, wt.reshape(32, 1, 1, 784), 0, -1)
    np.testing.assert_array_equal(got.reshape(6, 32), oracle.fc(x.reshape(6, 784), wt))


# ------------------------------------------------------------------------------- step
def test_step_ties_and_flip():
    thr = np.array([5, -3, 0, 7], np.int32)
    x = np.array([[5, -3, 0, 7],       # exactly at T
                  [6, -2, 1, 8],       # one above
                  [4, -4, -1, 6]], np.int32)
    f0 = np.zeros(4, np.uint8)
    f1 = np.ones(4, np.uint8)
    np.testing.assert_array_equal(oracle.step(x, thr, f0),
                                  [[-1] * 4, [1] * 4, [-1] * 4])
    np.testing.assert_array_equal(oracle.step(x, thr, f1),
                                  [[1] * 4, [-1] * 4, [1] * 4])
    np.testing.assert_array_equal(oracle.step(x, thr, None), oracle.step(x, thr, f0))
    mixed = np.array([0, 1, 0, 1], np.uint8)
    np.testing.assert_array_equal(oracle.step(x, thr, mixed)[0], [-1, 1, -1, 1])


def test_step_saturation_monotone_complement():
    k = 64
    x = oracle.fc(pm1((50, k)), pm1((8, k)))
    flip = np.array([0, 1, 0, 1, 1, 0, 0, 1], np.uint8)
    hi = np.full(8, k, np.int32)            # T >= K  -> (x > T) never true -> bit = flip
    lo = np.full(8, -k - 1, np.int32)       # T < -K  -> always true       -> bit = !flip
    want_hi = np.where(flip == 1, 1, -1)
    np.testing.assert_array_equal(oracle.step(x, hi, flip), np.broadcast_to(want_hi, x.shape))
    np.testing.assert_array_equal(oracle.step(x, lo, flip), np.broadcast_to(-want_hi, x.shape))
    # flip == complement
    thr = RNG.integers(-8, 9, size=8).astype(np.int32)
    np.testing.assert_array_equal(oracle.step(x, thr, flip),
                                  oracle.step(x, thr, None) * np.where(flip == 1, -1, 1))
    # monotone in T (flip = 0): raising T can only turn +1 into -1
    s_lo = oracle.step(x, thr, None)
    s_hi = oracle.step(x, thr + 3, None)
    assert np.all(s_hi <= s_lo)
    # direct definition
    np.testing.assert_array_equal(s_lo, np.where(x > thr, 1, -1))


# ------------------------------------------------------------------------------- pool
def test_pool_or_equals_max_on_pm1_all_windows():
    for bits in itertools.product([0, 1], repeat=4):
        win = np.array(bits, np.int8).reshape(1, 2, 2, 1) * 2 - 1
        got = oracle.maxpool2(win.astype(np.int8))
        assert got.shape == (1, 1, 1, 1)
        assert got[0, 0, 0, 0] == (1 if any(bits) else -1)


def test_pool_matches_numpy_and_rejects_odd():
    x = RNG.integers(-1000, 1000, size=(2, 6, 4, 5)).astype(np.int32)
    want = x.reshape(2, 3, 2, 2, 2, 5).max(axis=(2, 4))
    np.testing.assert_array_equal(oracle.maxpool2(x), want)
    x8 = pm1((2, 6, 4, 5))
    np.testing.assert_array_equal(oracle.maxpool2(x8), x8.reshape(2, 3, 2, 2, 2, 5).max(axis=(2, 4)))
    with pytest.raises(ValueError):
        oracle.maxpool2(np.zeros((1, 3, 4, 1), np.int32))
    # window placement: only (2y..2y+1, 2x..2x+1) contribute
    z = np.zeros((1, 4, 4, 1), np.int32)
    z[0, 1, 2, 0] = 9
    p = oracle.maxpool2(z)
    assert p[0, 0, 1, 0] == 9 and p.sum() == 9


def test_step_pool_order():
    # flip = 0: step(pool(x)) == pool(step(x)) because max is monotone.
    # flip = 1: pooling first turns the bit pool into an AND (min) of the stepped bits.
    x = RNG.integers(-20, 21, size=(3, 4, 6, 8)).astype(np.int32)
    thr = RNG.integers(-5, 6, size=8).astype(np.int32)
    f0, f1 = np.zeros(8, np.uint8), np.ones(8, np.uint8)
    np.testing.assert_array_equal(oracle.step(oracle.maxpool2(x), thr, f0),
                                  oracle.maxpool2(oracle.step(x, thr, f0)))
    s1 = oracle.step(x, thr, f1)
    and_pool = s1.reshape(3, 2, 2, 3, 2, 8).min(axis=(2, 4))
    np.testing.assert_array_equal(oracle.step(oracle.maxpool2(x), thr, f1), and_pool)


# ------------------------------------------------------------------------------ model
def test_flatten_order_is_hwc():
    import workloads as W
    h, w, c, n_out = 2, 3, 4, 5
    L = W.Layer("fc_binary", h * w * c, n_out, step=False)
    L.weights = pm1((n_out, h * w * c))
    act = pm1((1, h, w, c))
    pre, nxt = oracle.run_layer(L, act)
    assert nxt is None
    for (y, x, ch) in [(0, 0, 0), (1, 2, 3), (0, 1, 2), (1, 0, 1)]:
        act2 = act.copy()
        act2[0, y, x, ch] *= -1
        pre2, _ = oracle.run_layer(L, act2)
        idx = (y * w + x) * c + ch
        np.testing.assert_array_equal(pre2 - pre, (-2 * act[0, y, x, ch] * L.weights[:, idx])[None, :])


def test_model_shapes_and_batch_invariance():
    import workloads as W
    cid, layers, (ih, iw, ic) = W.model_by_name("small_cnn")
    imgs = W.draw_images(W.rng_for(cid, 0, 0), 6, ih, iw, ic)
    logits, trace = oracle.run_model(layers, imgs)
    assert logits.shape == (6, 10) and logits.dtype == np.int32
    assert trace[0][0].shape == (6, 28, 28, 64) and trace[0][1].shape == (6, 14, 14, 64)
    assert trace[1][0].shape == (6, 14, 14, 64) and trace[1][1].shape == (6, 7, 7, 64)
    assert trace[2][0].shape == (6, 2048) and trace[3][0].shape == (6, 10)
    # image i gives the same logits alone, and at another position in the batch
    for i in (0, 3, 5):
        li, _ = oracle.run_model(layers, imgs[i:i + 1])
        np.testing.assert_array_equal(li[0], logits[i])
    perm = np.array([4, 2, 5, 0, 1, 3])
    lp, _ = oracle.run_model(layers, imgs[perm])
    np.testing.assert_array_equal(lp, logits[perm])
    # logits of a +-1 layer of fan-in 2048 have the parity of 2048 and are bounded by it
    assert np.all(logits % 2 == 0) and np.all(np.abs(logits) <= 2048)


def test_model_layer_chain_matches_manual_composition():
    import workloads as W
    cid, layers, (ih, iw, ic) = W.model_by_name("mlp")
    imgs = W.draw_images(W.rng_for(cid, 0, 0), 5, ih, iw, ic)
    logits, trace = oracle.run_model(layers, imgs)
    a = imgs.reshape(5, 784).astype(np.int64)
    x1 = a @ layers[0].weights.reshape(512, 784).astype(np.int64).T
    s1 = np.where((x1 > layers[0].thr) ^ (layers[0].flip == 1), 1, -1)
    x2 = s1 @ layers[1].weights.astype(np.int64).T
    s2 = np.where((x2 > layers[1].thr) ^ (layers[1].flip == 1), 1, -1)
    x3 = s2 @ layers[2].weights.astype(np.int64).T
    np.testing.assert_array_equal(trace[0][0].reshape(5, 512), x1)
    np.testing.assert_array_equal(trace[1][0], x2)
    np.testing.assert_array_equal(logits, x3)


def _np_step(x, thr, flip):
    return np.where((x > thr.astype(np.int64)) ^ (flip == 1), 1, -1).astype(np.int64)


def _np_pool(x):
    n, h, w, c = x.shape
    return x.reshape(n, h // 2, 2, w // 2, 2, c).max(axis=(2, 4))


@pytest.mark.parametrize("pool_first", [False, True])
@pytest.mark.parametrize("first_pad_value", [-1, 5])
def test_small_cnn_matches_numpy_composition(pool_first, first_pad_value):
    # The Python composition in oracle.run_layer / run_model (which layer gets which pad value,
    # step and pool in which order, flatten, no step on the logits layer) against a chain written
    # out here with numpy only: explicit padding + einsum, np.where, reshape-max.
    import workloads as W
    cid, layers, (ih, iw, ic) = W.model_by_name("small_cnn")
    imgs = W.draw_images(W.rng_for(cid, 0, 0), 2, ih, iw, ic)
    logits, trace = oracle.run_model(layers, imgs, first_pad_value=first_pad_value, pool_first=pool_first)

    def hidden(x, L):
        if pool_first:
            return _np_step(_np_pool(x), L.thr, L.flip)
        return _np_pool(_np_step(x, L.thr, L.flip))

    c1, c2, f1, f2 = layers
    x1 = _np_conv(imgs, c1.weights, 1, first_pad_value)            # int8 pixels, pad value as given
    a1 = hidden(x1, c1)
    x2 = _np_conv(a1, c2.weights, 1, -1)                           # binary layer: padding is -1
    a2 = hidden(x2, c2)
    x3 = a2.reshape(2, 7 * 7 * 64) @ f1.weights.astype(np.int64).T   # flatten (h, w, c), c fastest
    a3 = _np_step(x3, f1.thr, f1.flip)
    x4 = a3 @ f2.weights.astype(np.int64).T                        # logits: no step
    np.testing.assert_array_equal(trace[0][0], x1)
    np.testing.assert_array_equal(trace[0][1], a1)
    np.testing.assert_array_equal(trace[1][0], x2)
    np.testing.assert_array_equal(trace[1][1], a2)
    np.testing.assert_array_equal(trace[2][0], x3)
    np.testing.assert_array_equal(trace[2][1].reshape(2, 2048), a3)
    np.testing.assert_array_equal(logits, x4)
    assert trace[3][1] is None
    # the planted alternatives really differ on this input, so the equalities above pin them
    assert not np.array_equal(_np_conv(a1, c2.weights, 1, 0), x2)              # pad 0 instead of -1
    assert not np.array_equal(_np_step(_np_pool(x1), c1.thr, c1.flip),
                              _np_pool(_np_step(x1, c1.thr, c1.flip)))         # the two pool orders


def test_conv_chain_with_and_without_pool_matches_numpy():
    # a VGG-like fragment (binary conv without pool -> binary conv with pool -> FC) through
    # oracle.run_layer, per layer, in both pool orders
    import workloads as W
    rng = np.random.default_rng(2024)
    la = W.Layer("conv_binary", 6, 40, 3, 3, 1, pool=1)
    lb = W.Layer("conv_binary", 40, 8, 3, 3, 1, pool=2)
    lc = W.Layer("fc_binary", 3 * 2 * 8, 5, step=False)
    for L, k in ((la, 54), (lb, 360)):
        L.weights = pm1((L.c_out, 3, 3, L.c_in), rng)
        L.thr = rng.integers(-k // 8, k // 8 + 1, size=L.c_out).astype(np.int32)
        L.flip = rng.integers(0, 2, size=L.c_out).astype(np.uint8)
    lc.weights = pm1((5, 48), rng)
    act = pm1((3, 6, 4, 6), rng)
    for pool_first in (False, True):
        pre_a, out_a = oracle.run_layer(la, act, pool_first=pool_first)
        xa = _np_conv(act, la.weights, 1, -1)
        sa = _np_step(xa, la.thr, la.flip)
        np.testing.assert_array_equal(pre_a, xa)
        np.testing.assert_array_equal(out_a, sa)                   # no pool: order flag is irrelevant
        pre_b, out_b = oracle.run_layer(lb, out_a, pool_first=pool_first)
        xb = _np_conv(sa, lb.weights, 1, -1)
        sb = _np_step(_np_pool(xb), lb.thr, lb.flip) if pool_first else _np_pool(_np_step(xb, lb.thr, lb.flip))
        np.testing.assert_array_equal(pre_b, xb)
        np.testing.assert_array_equal(out_b, sb)
        pre_c, out_c = oracle.run_layer(lc, out_b, pool_first=pool_first)
        np.testing.assert_array_equal(pre_c, sb.reshape(3, 48) @ lc.weights.astype(np.int64).T)
        assert out_c is None


def test_helper_packer_roundtrip():
    from tests.helpers import unpack_words
    a = pm1((3, 5, 70))
    p = pack_pm1(a)
    assert p.shape == (3, 5, 3) and p.dtype == np.uint32
    np.testing.assert_array_equal(unpack_words(p, 70), a)
    assert (int(p[0, 0, 0]) & 1) == (1 if a[0, 0, 0] > 0 else 0)
    assert np.all(p[..., 2] >> 6 == 0)      # tail bits are zero


@pytest.mark.parametrize("name", ["mlp", "small_cnn", "vgg_small"])
def test_golden_logits_regression(name):
    # stored values were written by tests/golden/make_golden.py from the oracle alone
    import os
    import workloads as W
    path = os.path.join(os.path.dirname(__file__), "golden", f"{name}_logits.txt")
    want = np.loadtxt(path, dtype=np.int64, comments="#", ndmin=2)
    cid, layers, (ih, iw, ic) = W.model_by_name(name)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), want.shape[0], ih, iw, ic)
    logits, _ = oracle.run_model(layers, imgs)
    np.testing.assert_array_equal(logits, want)
