"""Small-batch models whose last two layers are fully connected: outside TIMED mode the last
layer (no step) runs inside the launch of the layer before it (the batch <= 8 kernel or the
32 x 32 tile kernel), as integer atomic additions into logits that the first layer's launch has
zeroed.  Logits and every layer's outputs against the
oracle, for widths that are not whole words, for the largest (batch x classes) that takes this
path and the first that does not, on repeated runs over logits holding garbage, as graph replays
and through the entry point that allocates nothing; TIMED mode (separate launches) must agree."""
import numpy as np
import pytest
import torch

import oracle
import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import DeviceModel, dev, host_u32, require_gpu
from tests.helpers import pack_pm1

pytestmark = pytest.mark.gpu

FC, FIRST = W.configs.KIND_FC_BIN, W.configs.KIND_CONV_FIRST


def fc_model(widths, in_c, cid):
    """first layer (1x1 over in_c int8 features) -> FC ... -> FC without step."""
    layers = [W.Layer(FIRST, in_c, widths[0], 1, 1, 0)]
    for a, b in zip(widths[:-2], widths[1:-1]):
        layers.append(W.Layer(FC, a, b))
    layers.append(W.Layer(FC, widths[-2], widths[-1], step=False))
    return W.build_model(layers, 1, 1, in_c, cid), (1, 1, in_c)


def check(layers, in_shape, batch, cid, what):
    print("fc tail:", what, "batch", batch, flush=True)
    imgs = W.draw_images(W.rng_for(cid, 0, batch), batch, *in_shape)
    logits, trace = oracle.run_model(layers, imgs)
    dm = DeviceModel(layers, batch, in_shape, taps=True)
    xd = dev(imgs)
    runs = [("stream", lambda: dm.run(xd, P.RUN_STREAM)), ("stream again", lambda: dm.run(xd, P.RUN_STREAM)),
            ("timed", lambda: dm.run(xd, P.RUN_TIMED)), ("graph", lambda: dm.run(xd, P.RUN_GRAPH)),
            ("graph replay", lambda: dm.run(xd, P.RUN_GRAPH)),
            ("noalloc", lambda: P.bnn_run_model_noalloc(dm.model, xd, dm.logits))]
    for i, (mode, fn) in enumerate(runs):
        dm.logits.fill_(1234567 * (i + 1))          # whatever the logits held must not matter
        fn()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dm.logits.cpu().numpy(), logits, err_msg=f"{what}: logits, {mode}")
        if not mode.startswith("graph"):
            for li, (pre, act) in enumerate(trace):
                got_pre = dm.preact_taps[li].cpu().numpy().reshape(pre.shape)
                np.testing.assert_array_equal(got_pre, pre, err_msg=f"{what}: layer {li} pre-activations, {mode}")
                if act is not None:
                    want = pack_pm1(act)
                    got = host_u32(dm.packed_taps[li]).reshape(want.shape)
                    np.testing.assert_array_equal(got, want, err_msg=f"{what}: layer {li} bits, {mode}")


@pytest.mark.parametrize("widths,in_c,batch", [
    ((64, 64, 10), 16, 1),            # one word per row, one block
    ((100, 70, 33), 48, 3),           # hidden widths and class count that are not whole words
    ((96, 1000, 64), 32, 8),          # 8 x 64 = 512 (row, class) pairs: the most one block takes
    ((96, 1000, 65), 32, 8),          # 520 pairs: separate launches
    ((96, 1000, 65), 32, 7),          # 455 pairs
    ((512, 2050, 2), 784, 5),         # last word of the hidden layer holds two bits
    ((128, 4097, 1), 64, 8),          # a single logit; hidden width one bit over a word multiple
    ((64, 8192, 10), 16, 2),          # the widest hidden layer that takes this path
    ((64, 8224, 10), 16, 2),          # one word wider: separate launches
    ((256, 33, 10), 128, 2),          # hidden layer of two words, the second with one bit
    ((64, 96, 40, 10), 16, 4),        # two hidden FC layers before the last
    # more than 8 rows: the 32 x 32 tile kernel
    ((96, 1000, 16), 32, 40),         # 16 classes: the most it takes; two row blocks, the second ragged
    ((96, 1000, 17), 32, 40),         # 17 classes: separate launches
    ((100, 70, 9), 48, 33),           # ragged everywhere, one row in the second row block
    ((512, 994, 2), 784, 100),        # last word of the hidden layer holds two bits
    ((96, 1024, 10), 32, 70),         # the widest hidden layer that takes this path at more than 8 rows
    ((96, 1056, 10), 32, 70),         # one word wider: separate launches
    ((64, 33, 1), 16, 9),             # a single logit
    ((64, 96, 40, 10), 16, 300),      # ten row blocks
])
def test_fc_tail_shapes(widths, in_c, batch):
    require_gpu()
    layers, in_shape = fc_model(list(widths), in_c, 50 + len(widths))
    check(layers, in_shape, batch, 50 + len(widths), f"first {in_c}->" + "->".join(map(str, widths)))


@pytest.mark.parametrize("name", ["mlp", "small_cnn", "vgg_small"])
@pytest.mark.parametrize("batch", [1, 2, 8, 9])
def test_fc_tail_benchmark_models(name, batch):
    require_gpu()
    cid, layers, in_shape = W.model_by_name(name)
    check(layers, in_shape, batch, cid, name)


@pytest.mark.parametrize("kh,pad,hw,c_in", [(5, 2, 8, 5),      # general first-layer kernel
                                            (3, 1, 6, 3),      # patch kernel (width not a power of two)
                                            (3, 1, 8, 3)])     # whole-image kernel
def test_fc_tail_after_each_first_layer_kernel(kh, pad, hw, c_in):
    """The logits are zeroed by whichever first-layer kernel the shape selects."""
    require_gpu()
    cid = 70 + kh + hw
    layers = W.build_model([W.Layer(FIRST, c_in, 32, kh, kh, pad), W.Layer(FC, hw * hw * 32, 100),
                            W.Layer(FC, 100, 10, step=False)], hw, hw, c_in, cid)
    check(layers, (hw, hw, c_in), 3, cid, f"conv {kh}x{kh} on {hw}x{hw}x{c_in} -> 100 -> 10")


@pytest.mark.parametrize("name,batch", [("mlp", 64), ("mlp", 300), ("small_cnn", 40), ("vgg_small", 20)])
def test_fc_tail_benchmark_models_larger_batches(name, batch):
    require_gpu()
    cid, layers, in_shape = W.model_by_name(name)
    check(layers, in_shape, batch, cid, name)


def test_two_layer_model_has_no_tail_to_fold():
    require_gpu()
    layers, in_shape = fc_model([64, 10], 16, 61)
    check(layers, in_shape, 4, 61, "first 16->64->10")
