"""Run-to-run bit identity: every benchmark configuration three times on the same inputs; all
outputs (logits, packed activations, GEMM products) must be identical bit for bit."""
import numpy as np
import pytest
import torch

import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import DeviceModel, dev, fill_i32, require_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()
    yield
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,batch", [("mlp", 64), ("small_cnn", 1), ("small_cnn", 256), ("vgg_small", 1),
                                        ("vgg_small", 256), ("vgg_small", 4096)])
def test_models_three_runs_identical(name, batch):
    print("determinism", name, batch, flush=True)
    cid, layers, in_shape = W.model_by_name(name)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    dm = DeviceModel(layers, batch, in_shape)
    xd = dev(imgs)
    runs = []
    for mode in (P.RUN_STREAM, P.RUN_GRAPH, P.RUN_STREAM):
        dm.logits.fill_(-9)
        dm.ws.fill_(0x5a)
        dm.run(xd, mode)
        torch.cuda.synchronize()
        runs.append(dm.logits.clone())
    assert torch.equal(runs[0], runs[1]) and torch.equal(runs[0], runs[2])
    assert not bool((runs[0] == -9).all())


@pytest.mark.parametrize("m,n,k", W.GEMM_SWEEP_SHAPES[:3] + W.GEMM_SWEEP_SHAPES[4:])
def test_gemm_three_runs_identical(m, n, k):
    print("determinism gemm", m, n, k, flush=True)
    g = torch.Generator(device="cuda").manual_seed(m + n + k)
    a = torch.randint(-2**31, 2**31 - 1, (m, k // 32), dtype=torch.int32, device="cuda", generator=g)
    b = torch.randint(-2**31, 2**31 - 1, (n, k // 32), dtype=torch.int32, device="cuda", generator=g)
    outs = []
    for _ in range(3):
        c = fill_i32((m, n), 7)
        P.bnn_fc_binary(a, m, k, b, n, c_out=c)
        torch.cuda.synchronize()
        outs.append(c)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("hw,c", [(8, 512), (16, 256), (32, 128)])
def test_conv_sweep_three_runs_identical(hw, c):
    print("determinism conv", hw, c, flush=True)
    n, cw = 1024, c // 32
    g = torch.Generator(device="cuda").manual_seed(hw * c)
    x = torch.randint(-2**31, 2**31 - 1, (n, hw, hw, cw), dtype=torch.int32, device="cuda", generator=g)
    wt = torch.randint(-2**31, 2**31 - 1, (c, 3, 3, cw), dtype=torch.int32, device="cuda", generator=g)
    thr = torch.randint(-c, c, (c,), dtype=torch.int32, device="cuda", generator=g)
    outs = []
    for _ in range(3):
        o = fill_i32((n, hw, hw, cw), -1)
        P.bnn_conv_binary(x, n, hw, hw, c, wt, c, thr=thr, pool=1, packed_out=o)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("name,batch", [("small_cnn", 5), ("vgg_small", 32), ("vgg_small", 256)])
def test_two_model_objects_on_two_streams_at_once(name, batch):
    """Independent batches issued alternately on two streams (each model object owns its workspace
    and logits) overlap on the device; both must give what one stream alone gives, every time."""
    import oracle
    print("two streams", name, batch, flush=True)
    cid, layers, in_shape = W.model_by_name(name)
    imgs_a = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    imgs_b = W.draw_images(W.rng_for(cid, 0, 1), batch, *in_shape)
    want = [oracle.run_model(layers, im)[0] for im in (imgs_a, imgs_b)]
    dms = [DeviceModel(layers, batch, in_shape) for _ in range(2)]
    xs = [dev(imgs_a), dev(imgs_b)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(6):
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                dms[i].logits.fill_(-9)
                dms[i].run(xs[i], P.RUN_STREAM)
        torch.cuda.synchronize()
        for i in range(2):
            np.testing.assert_array_equal(dms[i].logits.cpu().numpy(), want[i], err_msg=f"stream {i}, repeat {rep}")
