"""GPU parity of the convolution kernels that the benchmark actually times: shapes large enough
that bnn_conv_binary itself selects the 256 x 128 block tile (asserted through the host-side
kernel-choice query), compared with the FULL oracle for every image: raw int32 sums, step,
step + pool and pool + step (the paper's order), with ties and out-of-range thresholds planted."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_05126_amd as P
from tests.gpu_util import (TILE_256x128, conv_kernel_choice, dev, fill_i32, host_u32, require_gpu)
from tests.helpers import pack_pm1, unpack_words
from tests.test_gpu_parity import extreme_thresholds

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()
    yield
    torch.cuda.synchronize()


# (n, h = w, c_in, c_out): one shape per channel-word width of the big tile (2, 4, 8, 16 and 32
# words per pixel); the 8 x 8 shapes have four images per pixel tile and a ragged last tile
BIG_TILE_SHAPES = [(512, 14, 64, 64), (131, 32, 128, 128), (512, 16, 256, 256), (1026, 8, 512, 512),
                   (2050, 8, 1024, 128), (300, 16, 128, 256)]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n,hw,ci,co", BIG_TILE_SHAPES)
def test_big_tile_full_oracle_all_epilogues(n, hw, ci, co):
    assert conv_kernel_choice(n, hw, hw, ci, co) == TILE_256x128
    print(f"big tile {n}x{hw}x{hw} {ci}->{co}: drawing", flush=True)
    rng = np.random.default_rng(n * 7 + hw * 3 + ci + co)
    cw = ci // 32
    xw = rng.integers(0, 2**32, size=(n, hw, hw, cw), dtype=np.uint32)
    wt = (2 * rng.integers(0, 2, size=(co, 3, 3, ci), dtype=np.int8) - 1).astype(np.int8)
    print("  oracle", flush=True)
    want = oracle.conv2d(unpack_words(xw, ci), wt, 1, -1)
    xd = dev(xw)
    wd = dev(pack_pm1(wt.reshape(co * 9, ci)).reshape(co, 3, 3, cw))
    print("  GPU raw", flush=True)
    raw = fill_i32((n, hw, hw, co), 99999)
    P.bnn_conv_binary(xd, n, hw, hw, ci, wd, co, preact_out=raw)
    np.testing.assert_array_equal(raw.cpu().numpy(), want)
    del raw
    k = 9 * ci
    thr = rng.integers(-(k // 8), k // 8 + 1, size=co).astype(np.int32)
    thr[: co // 2] = want[n - 1, hw - 1, 0, : co // 2]          # ties at a pixel of the last image
    extreme_thresholds(thr, 8, k)
    flip = rng.integers(0, 2, size=co).astype(np.uint8)
    td, fd = dev(thr), dev(flip)
    s = oracle.step(want, thr, flip)
    print("  GPU step (+ raw)", flush=True)
    raw2 = fill_i32((n, hw, hw, co), 99999)
    packed = fill_i32((n, hw, hw, co // 32), -1)
    P.bnn_conv_binary(xd, n, hw, hw, ci, wd, co, thr=td, flip=fd, pool=1, preact_out=raw2, packed_out=packed)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(s))
    np.testing.assert_array_equal(raw2.cpu().numpy(), want)
    del raw2
    print("  GPU step, no flips", flush=True)
    packed = fill_i32((n, hw, hw, co // 32), -1)
    P.bnn_conv_binary(xd, n, hw, hw, ci, wd, co, thr=td, pool=1, packed_out=packed)
    np.testing.assert_array_equal(host_u32(packed), pack_pm1(oracle.step(want, thr, None)))
    print("  GPU step + pool", flush=True)
    pooled = fill_i32((n, hw // 2, hw // 2, co // 32), -1)
    P.bnn_conv_binary(xd, n, hw, hw, ci, wd, co, thr=td, flip=fd, pool=2, packed_out=pooled)
    np.testing.assert_array_equal(host_u32(pooled), pack_pm1(oracle.maxpool2(s)))
    print("  GPU pool + step", flush=True)
    pooled = fill_i32((n, hw // 2, hw // 2, co // 32), -1)
    P.bnn_conv_binary(xd, n, hw, hw, ci, wd, co, thr=td, flip=fd, pool=2, pool_first=1, packed_out=pooled)
    np.testing.assert_array_equal(host_u32(pooled), pack_pm1(oracle.step(oracle.maxpool2(want), thr, flip)))
