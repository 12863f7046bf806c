"""GPU parity at the benchmark configurations' full sizes, in the launch shapes bench.py
times.  Where the full oracle is affordable it is used in full; above that the product is
checked with an exact Freivalds-style identity over every entry (C r == A (B r) for random
+-1 vectors r, evaluated in float64 where every intermediate is an integer below 2^53) plus
full oracle rows / columns and sampled entries."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import DeviceModel, dev, fill_i32, host_u32, pack_on_gpu, require_gpu
from tests.helpers import pack_pm1, unpack_words

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()
    yield
    torch.cuda.synchronize()


def gemm_on_gpu(a, b):
    m, k = a.shape
    n = b.shape[0]
    ad, bd = pack_on_gpu(a), pack_on_gpu(b)
    c = fill_i32((m, n), 7)
    P.bnn_fc_binary(ad, m, k, bd, n, c_out=c)
    torch.cuda.synchronize()
    return c.cpu().numpy()


def test_gemm_4096_full_oracle():
    m = n = k = 4096
    a = W.draw_bits_pm1(W.rng_for(3, 1, 0), m, k)
    b = W.draw_bits_pm1(W.rng_for(3, 1, 1), n, k)
    print("gemm 4096^3 full oracle", flush=True)
    np.testing.assert_array_equal(gemm_on_gpu(a, b), oracle.fc(a, b))


def test_gemv_m1_8192_full_oracle():
    a = W.draw_bits_pm1(W.rng_for(3, 4, 0), 1, 8192)
    b = W.draw_bits_pm1(W.rng_for(3, 4, 1), 8192, 8192)
    print("gemv 1x8192x8192 full oracle", flush=True)
    np.testing.assert_array_equal(gemm_on_gpu(a, b), oracle.fc(a, b))


def freivalds_check(a, b, c, n_vec=32, seed=99):
    """Exact: (C r) == A (B r) for n_vec random +-1 vectors, blockwise in float64."""
    m, k = a.shape
    n = b.shape[0]
    rng = np.random.default_rng(seed)
    r = (2.0 * rng.integers(0, 2, size=(n, n_vec)) - 1.0)
    br = np.zeros((k, n_vec))
    blk = 1024
    for j0 in range(0, n, blk):                      # B^T r accumulated over row blocks of B
        bb = b[j0:j0 + blk].astype(np.float64)
        br += bb.T @ r[j0:j0 + blk]
    for i0 in range(0, m, blk):
        lhs = c[i0:i0 + blk].astype(np.float64) @ r
        rhs = a[i0:i0 + blk].astype(np.float64) @ br
        if not np.array_equal(lhs, rhs):
            bad = np.argwhere(lhs != rhs)[0]
            raise AssertionError(f"Freivalds mismatch in row {i0 + bad[0]}, vector {bad[1]}")


@pytest.mark.timeout(600)
@pytest.mark.parametrize("size,layer", [(8192, 2), (16384, 3)])
def test_gemm_large_freivalds_rows_cols_samples(size, layer):
    m = n = k = size
    print(f"gemm {size}^3: drawing operands", flush=True)
    a = W.draw_bits_pm1(W.rng_for(3, layer, 0), m, k)
    b = W.draw_bits_pm1(W.rng_for(3, layer, 1), n, k)
    print("  GPU product", flush=True)
    c = gemm_on_gpu(a, b)
    print("  Freivalds over all entries", flush=True)
    freivalds_check(a, b, c)
    print("  64 full rows and 64 full columns from the oracle", flush=True)
    rng = np.random.default_rng(size)
    rows = np.sort(rng.choice(m, 64, replace=False))
    cols = np.sort(rng.choice(n, 64, replace=False))
    rows[0], rows[-1], cols[0], cols[-1] = 0, m - 1, 0, n - 1
    np.testing.assert_array_equal(c[rows], oracle.fc(a[rows], b))
    np.testing.assert_array_equal(c[:, cols], oracle.fc(a, b[cols]))
    print("  2^20 sampled entries (1024 random rows x 1024 random columns)", flush=True)
    ri = rng.choice(m, 1024, replace=False)
    ci = rng.choice(n, 1024, replace=False)
    np.testing.assert_array_equal(c[np.ix_(ri, ci)], oracle.fc(a[ri], b[ci]))
    for _ in range(256):                             # and single dots at unstructured positions
        i, j = int(rng.integers(m)), int(rng.integers(n))
        assert c[i, j] == oracle.dot(a[i], b[j])


@pytest.mark.timeout(300)
def test_vgg_small_batch256_all_logits():
    cid, layers, in_shape = W.model_by_name("vgg_small")
    imgs = W.draw_images(W.rng_for(cid, 0, 0), 256, *in_shape)
    print("vgg_small b256: oracle", flush=True)
    logits, _ = oracle.run_model(layers, imgs)
    dm = DeviceModel(layers, 256, in_shape)
    xd = dev(imgs)
    for mode in (P.RUN_STREAM, P.RUN_GRAPH):
        dm.logits.fill_(-9)
        dm.run(xd, mode)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits)


@pytest.mark.timeout(600)
def test_vgg_small_batch4096_sampled_images():
    # images are independent: the logits of image i in the big batch equal those of a batch
    # holding only the sampled images (256 of them, spread over the batch, both ends included)
    cid, layers, in_shape = W.model_by_name("vgg_small")
    batch = 4096
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    dm = DeviceModel(layers, batch, in_shape)
    print("vgg_small b4096: GPU", flush=True)
    dm.run(dev(imgs), P.RUN_STREAM)
    torch.cuda.synchronize()
    got = dm.logits.cpu().numpy()
    rng = np.random.default_rng(4096)
    idx = np.unique(np.concatenate([[0, 1, 255, 256, 4095], rng.choice(batch, 251, replace=False)]))
    print("vgg_small b4096: oracle on", len(idx), "images", flush=True)
    want, _ = oracle.run_model(layers, imgs[idx])
    np.testing.assert_array_equal(got[idx], want)
    assert np.all(got % 2 == 0) and np.all(np.abs(got) <= 1024)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("hw,c", W.CONV_SWEEP_SHAPES)
def test_conv_sweep_batch1024(hw, c):
    """The per-layer sweep at its full batch.  The whole output is compared with the oracle where
    that costs at most 155 G MAC (six shapes); the three largest layers are compared on 64 images
    spread over the batch (first, last and every 16th in between)."""
    n = 1024
    cw = c // 32
    rng = W.rng_for(4, hw, c % 1000)
    xw = rng.integers(0, 2**32, size=(n, hw, hw, cw), dtype=np.uint32)
    wt = W.draw_pm1(rng, (c, 3, 3, c))
    thr = W.draw_threshold(rng, c, 9 * c)
    flip = W.draw_flip(rng, c)
    wd = dev(pack_pm1(wt.reshape(c * 9, c)).reshape(c, 3, 3, cw))
    out = fill_i32((n, hw, hw, cw), -1)
    P.bnn_conv_binary(dev(xw), n, hw, hw, c, wd, c, thr=dev(thr), flip=dev(flip), pool=1, packed_out=out)
    torch.cuda.synchronize()
    got = host_u32(out)
    macs = n * hw * hw * c * 9 * c
    full = macs <= 155e9
    idx = np.arange(n) if full else np.unique(np.concatenate([np.arange(0, n, 16), [1, n - 1]]))
    print(f"conv sweep {hw}x{hw} C{c} batch {n}: oracle on {len(idx)} images", flush=True)
    x_s = unpack_words(xw[idx], c)
    want = pack_pm1(oracle.step(oracle.conv2d(x_s, wt, 1, -1), thr, flip))
    np.testing.assert_array_equal(got[idx], want)
    # the other images: bits look random, none of the fill value survives
    assert not np.any(np.all(got.reshape(n, -1) == 0xFFFFFFFF, axis=1))


@pytest.mark.timeout(300)
@pytest.mark.parametrize("n,hw,ci,co,pool", [(8192, 4, 1024, 128, 2), (2048, 8, 512, 256, 1), (2050, 8, 512, 128, 2),
                                             (4096, 4, 1024, 128, 1), (1030, 8, 512, 128, 2), (3001, 5, 512, 256, 1),
                                             (2100, 7, 1024, 128, 1), (1024, 8, 512, 192, 2), (1500, 6, 608, 160, 1)])
def test_conv_wide_layers_streamed_weights_sampled_images(n, hw, ci, co, pool):
    """C_in >= 512 at a batch that selects the largest block tile (weight chunks streamed through two
    LDS buffers): sampled images against the oracle, first / last / ragged-tail images included."""
    cw = (ci + 31) // 32
    rng = W.rng_for(4, hw + 50, ci % 1000 + co)
    print(f"conv wide {hw}x{hw} {ci}->{co} batch {n} pool {pool}", flush=True)
    xw = rng.integers(0, 2**32, size=(n, hw, hw, cw), dtype=np.uint32)
    if ci % 32:
        xw[..., -1] &= np.uint32((1 << (ci % 32)) - 1)       # tail bits of the last word are zero
    wt = W.draw_pm1(rng, (co, 3, 3, ci))
    thr = W.draw_threshold(rng, co, 9 * ci)
    flip = W.draw_flip(rng, co)
    wd = dev(pack_pm1(wt.reshape(co * 9, ci)).reshape(co, 3, 3, cw))
    out = fill_i32((n, hw // pool, hw // pool, (co + 31) // 32), -1)
    P.bnn_conv_binary(dev(xw), n, hw, hw, ci, wd, co, thr=dev(thr), flip=dev(flip), pool=pool, packed_out=out)
    torch.cuda.synchronize()
    got = host_u32(out)
    idx = np.array([0, 1, 15, 16, n // 2 + 3, n - 17, n - 2, n - 1])
    x_s = unpack_words(xw[idx], ci)
    s = oracle.step(oracle.conv2d(x_s, wt, 1, -1), thr, flip)
    if pool == 2:
        s = oracle.maxpool2(s)
    np.testing.assert_array_equal(got[idx], pack_pm1(s))
    assert not np.any(np.all(got.reshape(n, -1) == 0xFFFFFFFF, axis=1))
