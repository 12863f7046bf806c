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
