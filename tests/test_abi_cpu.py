"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before touching HIP."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    so = os.path.join(ROOT, "paper_2301_05126_amd", "libbnn.so")
    if not os.path.exists(so):
        from paper_2301_05126_amd.build import build
        build()
    import paper_2301_05126_amd as P
    return P


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(bnn_[a-z0-9_]+)\s*\(", text)
    return sorted(set(n for n in names if n != "bnn_host_layer_fn"))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"bnn_pack_bits", "bnn_conv_first_int8", "bnn_conv_binary", "bnn_fc_binary",
            "bnn_threshold_sign_maxpool", "bnn_run_model", "bnn_model_create",
            "bnn_model_destroy", "bnn_model_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib.api._lib, n), n


def test_status_strings(lib):
    want = ["BNN_OK", "BNN_ERR_NULL", "BNN_ERR_SHAPE", "BNN_ERR_ALIGN", "BNN_ERR_UNSUPPORTED",
            "BNN_ERR_WORKSPACE", "BNN_ERR_HIP"]
    assert [lib.bnn_status_string(i) for i in range(7)] == want
    assert lib.bnn_version()


OK, NULL, SHAPE, ALIGN, UNSUP, WS = 0, 1, 2, 3, 4, 5
P16 = 0x1000          # fake, aligned "device" address; never dereferenced by validation
P8 = 0x1008           # misaligned


def test_pack_bits_validation(lib):
    f = lib.api._lib.bnn_pack_bits
    assert f(None, 1, 32, P16, None) == NULL
    assert f(P16, 1, 32, None, None) == NULL
    assert f(P16, -1, 32, P16, None) == SHAPE
    assert f(P16, 1, 0, P16, None) == SHAPE
    assert f(P8, 1, 32, P16, None) == ALIGN
    assert f(P16, 1, 32, P8, None) == ALIGN


def test_fc_validation(lib):
    f = lib.api._lib.bnn_fc_binary
    ep = lib.Epilogue(P16, None, 1, 0)
    assert f(None, 4, 64, P16, 8, None, P16, None, None) == NULL
    assert f(P16, 4, 64, None, 8, None, P16, None, None) == NULL
    assert f(P16, 4, 64, P16, 8, None, None, None, None) == NULL          # raw output required
    assert f(P16, 4, 64, P16, 8, C.byref(ep), None, None, None) == NULL   # packed output required
    assert f(P16, 4, 0, P16, 8, None, P16, None, None) == SHAPE
    assert f(P16, -4, 64, P16, 8, None, P16, None, None) == SHAPE
    assert f(P16, 4, 64, P16, 0, None, P16, None, None) == SHAPE
    assert f(P8, 4, 64, P16, 8, None, P16, None, None) == ALIGN
    assert f(P16, 4, 64, P16, 8, None, P8, None, None) == ALIGN
    bad_pool = lib.Epilogue(P16, None, 2, 0)
    assert f(P16, 4, 64, P16, 8, C.byref(bad_pool), None, P16, None) == SHAPE
    no_thr = lib.Epilogue(None, None, 1, 0)
    assert f(P16, 4, 64, P16, 8, C.byref(no_thr), None, P16, None) == NULL
    # more than 8 rows run with FP32 accumulators: K beyond their exact range is refused
    assert f(P16, 9, (1 << 24) - 2047, P16, 8, None, P16, None, None) == UNSUP
    assert f(P16, 9, (1 << 30) + 1, P16, 8, None, P16, None, None) == SHAPE


def test_conv_validation(lib):
    f = lib.api._lib.bnn_conv_binary
    assert f(None, 1, 8, 8, 32, P16, 32, None, P16, None, None) == NULL
    assert f(P16, 1, 0, 8, 32, P16, 32, None, P16, None, None) == SHAPE
    assert f(P16, 1, 8, 8, 32, P16, 0, None, P16, None, None) == SHAPE
    assert f(P16, 1, 8, 8, 32, P8, 32, None, P16, None, None) == ALIGN
    pool = lib.Epilogue(P16, None, 2, 0)
    assert f(P16, 1, 7, 8, 32, P16, 32, C.byref(pool), None, P16, None) == SHAPE   # odd height
    pool3 = lib.Epilogue(P16, None, 3, 0)
    assert f(P16, 1, 8, 8, 32, P16, 32, C.byref(pool3), None, P16, None) == SHAPE
    bad_order = lib.Epilogue(P16, None, 2, 5)
    assert f(P16, 1, 8, 8, 32, P16, 32, C.byref(bad_order), None, P16, None) == SHAPE
    assert f(P16, 1, 32, 32, 1 << 16, P16, 32, None, P16, None, None) == UNSUP     # patch > LDS
    assert f(P16, 1, 1 << 13, 1 << 13, 1024, P16, 32, None, P16, None, None) == UNSUP   # an image of 8 GiB
    g = lib.api._lib.bnn_conv_first_int8
    assert g(None, 1, 8, 8, 1, P16, 32, 3, 3, 1, -1, None, P16, None, None) == NULL
    assert g(P16, 1, 8, 8, 1, P16, 32, 3, 3, 1, 300, None, P16, None, None) == SHAPE
    assert g(P16, 1, 2, 2, 1, P16, 32, 5, 5, 0, 0, None, P16, None, None) == SHAPE  # empty output
    assert g(P16, 1, 8, 8, 1, P16, 32, 3, 3, 1, -1, None, None, None, None) == NULL
    assert g(P16, 1, 1, 1, 70000, P16, 32, 1, 1, 0, -1, None, P16, None, None) == UNSUP


def test_step_validation(lib):
    f = lib.api._lib.bnn_threshold_sign_maxpool
    assert f(None, 1, 4, 4, 8, P16, None, 1, 0, P16, None) == NULL
    assert f(P16, 1, 4, 4, 8, None, None, 1, 0, P16, None) == NULL
    assert f(P16, 1, 4, 4, 8, P16, None, 3, 0, P16, None) == SHAPE
    assert f(P16, 1, 3, 4, 8, P16, None, 2, 0, P16, None) == SHAPE
    assert f(P16, 1, 4, 4, 8, P16, None, 2, 2, P16, None) == SHAPE
    assert f(P16, 1, 4, 4, 0, P16, None, 1, 0, P16, None) == SHAPE
    assert f(P16, 1, 4, 4, 8, P16, None, 1, 0, P8, None) == ALIGN


def _vgg_descs(lib, first_kind=None, last_step=0):
    import workloads as W
    _, layers, _ = W.model_by_name("vgg_small")
    kinds = {"conv_first_int8": 0, "conv_binary": 1, "fc_binary": 2}
    descs = []
    for L in layers:
        d = lib.LayerDesc(kinds[L.kind], L.c_in, L.c_out, L.kh, L.kw, L.pad, -1,
                          1 if L.step else 0, L.pool, 0, P16, P16 if L.step else None, None, None, None)
        descs.append(d)
    return descs


def test_model_create_validation_and_workspace(lib):
    descs = _vgg_descs(lib)
    m = lib.bnn_model_create(descs, 256, 32, 32, 3)
    # largest packed activation: layer 1 output 32x32x128 bits per image
    assert lib.bnn_model_workspace_bytes(m) == 2 * 256 * 32 * 32 * 4 * 4
    assert lib.api._lib.bnn_model_num_layers(m.handle) == 9
    assert lib.api._lib.bnn_model_num_classes(m.handle) == 10
    # run_model argument checks happen before any HIP call
    r = lib.api._lib.bnn_run_model
    cb0 = lib.api.HOST_LAYER_FN(0)
    assert r(m.handle, None, P16, P16, 1 << 30, 2, None, cb0, None, None) == NULL
    assert r(m.handle, P16, P16, P16, 16, 2, None, cb0, None, None) == WS
    assert r(m.handle, P16, P16, P16, 1 << 30, 0, None, cb0, None, None) == NULL   # TIMED needs timings
    assert r(m.handle, P16, P8, P16, 1 << 30, 2, None, cb0, None, None) == ALIGN
    assert r(m.handle, P16, P16, P16, 1 << 30, 7, None, cb0, None, None) == UNSUP
    lib.bnn_model_destroy(m)

    bad = _vgg_descs(lib)
    bad[3].c_in = 64                         # channel mismatch
    with pytest.raises(lib.BnnError) as e:
        lib.bnn_model_create(bad, 4, 32, 32, 3)
    assert e.value.status == SHAPE
    bad = _vgg_descs(lib)
    bad[-1].has_step = 1                     # last layer must emit logits
    with pytest.raises(lib.BnnError) as e:
        lib.bnn_model_create(bad, 4, 32, 32, 3)
    assert e.value.status == UNSUP
    bad = _vgg_descs(lib)
    bad[2].thr_dev = None
    with pytest.raises(lib.BnnError) as e:
        lib.bnn_model_create(bad, 4, 32, 32, 3)
    assert e.value.status == NULL
    bad = _vgg_descs(lib)
    with pytest.raises(lib.BnnError) as e:   # 31x31 input: odd size meets a pool
        lib.bnn_model_create(bad, 4, 31, 31, 3)
    assert e.value.status == SHAPE
    bad = _vgg_descs(lib)
    bad[0].kind = 1
    with pytest.raises(lib.BnnError) as e:
        lib.bnn_model_create(bad, 4, 32, 32, 3)
    assert e.value.status == UNSUP


def test_product_has_no_environment_switches():
    # dispatch depends on shapes only: the library reads no environment variable
    import subprocess
    so = os.path.join(ROOT, "paper_2301_05126_amd", "libbnn.so")
    syms = subprocess.run(["nm", "-D", "--undefined-only", so], capture_output=True, text=True).stdout
    assert "getenv" not in syms


def test_test_hook_library_is_separate(lib):
    # the hook that reaches the tile kernels with small shapes lives in its own library
    assert not hasattr(lib.api._lib, "bnn_test_conv_binary_tiles")
    hook = os.path.join(ROOT, "tests", "hooks", "libbnn_test_hooks.so")
    if os.path.exists(hook):
        assert hasattr(C.CDLL(hook), "bnn_test_conv_binary_tiles")


def test_kernel_choice_of_the_benchmark_shapes(lib):
    # host-side query (no GPU work): the shapes of the parity tests that are meant to reach the
    # 256 x 128 block tile do reach it, and so do the layers bench.py times
    from tests.gpu_util import KERNEL_SMALL, TILE_256x128, TILE_64x64, conv_kernel_choice
    import workloads as W
    from tests.test_gpu_bigtile import BIG_TILE_SHAPES
    for n, hw, ci, co in BIG_TILE_SHAPES:
        assert conv_kernel_choice(n, hw, hw, ci, co) == TILE_256x128, (n, hw, ci, co)
    _, layers, _ = W.model_by_name("vgg_small")
    for L in layers:
        if L.kind == "conv_binary":
            assert conv_kernel_choice(4096, L.h_in, L.w_in, L.c_in, L.c_out) == TILE_256x128
            assert conv_kernel_choice(1, L.h_in, L.w_in, L.c_in, L.c_out) == KERNEL_SMALL
            assert conv_kernel_choice(1, L.h_in, L.w_in, L.c_in, L.c_out, tiles_only=True) == TILE_64x64
    for hw, c in W.CONV_SWEEP_SHAPES:
        assert conv_kernel_choice(1024, hw, hw, c, c) in (TILE_256x128, 1, 2)
    assert conv_kernel_choice(4, 8, 8, 2048, 32) == -1       # more than 1024 channels: unsupported


def test_run_model_noalloc_validation(lib):
    # the entry point without a workspace argument refuses, on the host and before any HIP call,
    # what does not fit its fixed device array
    f = lib.api._lib.bnn_run_model_noalloc

    def vgg(batch):
        mk = lambda kind, ci, co, pool=1, step=1: lib.LayerDesc(kind, ci, co, 3, 3, 1, -1, step, pool, 0,
                                                                P16, P16 if step else None, None, None, None)
        descs = [mk(0, 3, 128), mk(1, 128, 128, 2), mk(1, 128, 256), mk(1, 256, 256, 2), mk(1, 256, 512),
                 mk(1, 512, 512, 2), mk(2, 8192, 1024), mk(2, 1024, 1024), mk(2, 1024, 10, 1, 0)]
        return lib.bnn_model_create(descs, batch, 32, 32, 3)

    small, big = vgg(512), vgg(513)
    assert lib.bnn_model_workspace_bytes(small) == lib.api.NOALLOC_SCRATCH_BYTES
    assert lib.bnn_model_workspace_bytes(big) > lib.api.NOALLOC_SCRATCH_BYTES
    assert f(big.handle, P16, P16, None) == WS
    assert f(None, P16, P16, None) == NULL
    assert f(small.handle, None, P16, None) == NULL
    assert f(small.handle, P16, None, None) == NULL
    assert f(small.handle, P8, P16, None) == ALIGN
    text = open(os.path.join(ROOT, "include", "bnn.h")).read()
    assert "#define BNN_NOALLOC_SCRATCH_BYTES (16u << 20)" in text
