"""bnn_run_model_noalloc (the entry point for callers that cannot allocate: its activation
buffers live in a fixed device array inside the library) against bnn_run_model on the same
model and input, through the C ABI: logits and every layer's packed activations bit for bit, on
two calls in a row, the second with a smaller model and batch, then the first again (the array
keeps earlier contents; no result may depend on them)."""
import numpy as np
import pytest
import torch

import paper_2301_05126_amd as P
import workloads as W
from tests.gpu_util import DeviceModel, dev, require_gpu

pytestmark = pytest.mark.gpu


def run_both(name, batch):
    cid, layers, in_shape = W.model_by_name(name)
    imgs = W.draw_images(W.rng_for(cid, 0, 0), batch, *in_shape)
    dm = DeviceModel(layers, batch, in_shape, taps=True)
    assert dm.ws_bytes <= P.api.NOALLOC_SCRATCH_BYTES
    xd = dev(imgs)
    dm.logits.fill_(-9)
    dm.run(xd, P.RUN_STREAM)
    torch.cuda.synchronize()
    want_logits = dm.logits.clone()
    want_taps = [t.clone() if t is not None else None for t in dm.packed_taps]
    want_pre = [t.clone() if t is not None else None for t in dm.preact_taps]
    assert not bool((want_logits == -9).all())
    return dm, xd, want_logits, want_taps, want_pre


def check_noalloc(dm, xd, want_logits, want_taps, want_pre, what):
    print("noalloc", what, flush=True)
    dm.logits.fill_(-9)
    for t in dm.packed_taps + dm.preact_taps:
        if t is not None:
            t.fill_(-1)
    P.bnn_run_model_noalloc(dm.model, xd, dm.logits)
    torch.cuda.synchronize()
    assert torch.equal(dm.logits, want_logits), what + ": logits"
    for li, (got, want) in enumerate(zip(dm.packed_taps, want_taps)):
        if want is not None:
            assert torch.equal(got, want), f"{what}: packed activations of layer {li}"
    for li, (got, want) in enumerate(zip(dm.preact_taps, want_pre)):
        if want is not None:
            assert torch.equal(got, want), f"{what}: pre-activations of layer {li}"


def test_noalloc_matches_run_model_on_two_calls_in_a_row():
    require_gpu()
    big = run_both("vgg_small", 64)
    small = run_both("small_cnn", 5)
    check_noalloc(*big, "vgg_small batch 64")
    check_noalloc(*small, "small_cnn batch 5 (smaller, right after)")
    check_noalloc(*big, "vgg_small batch 64 again")
    check_noalloc(*run_both("vgg_small", 512), "vgg_small batch 512 (the largest that fits)")
    check_noalloc(*run_both("mlp", 64), "mlp batch 64")


def test_noalloc_refuses_models_beyond_its_array():
    require_gpu()
    cid, layers, in_shape = W.model_by_name("vgg_small")
    dm = DeviceModel(layers, 513, in_shape)
    assert dm.ws_bytes > P.api.NOALLOC_SCRATCH_BYTES
    x = torch.zeros((513,) + tuple(in_shape), dtype=torch.int8, device="cuda")
    with pytest.raises(P.BnnError) as e:
        P.bnn_run_model_noalloc(dm.model, x, dm.logits)
    assert e.value.status == 5      # BNN_ERR_WORKSPACE
