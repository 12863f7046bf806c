"""CPU tests of the host-only helpers: Alg. 1 mapping and batch-norm folding."""
import math

import numpy as np
import pytest

from oracle import host_refs


@pytest.fixture(scope="module")
def P():
    import paper_2301_05126_amd as P
    return P


def test_map_layers_hand_example(P):
    # 2 batch sizes, 3 layers, implementations {0: host, 1: gpu}; worked by hand:
    # batch 0: minima 5 (host), 4 (gpu), 1 (host) = 10;  batch 1: 3, 3, 3.5 = 9.5 -> batch 1
    cpu = [[[5, 1], [9, 1], [1, 1]], [[3, 1], [8, 1], [3.5, 1]]]
    gpu = [[[0, 6], [0, 3], [0, 2]], [[0, 7], [0, 2], [0, 4]]]
    best, mapping, total = P.bnn_map_layers(cpu, gpu)
    assert (best, mapping, total) == (1, [0, 1, 0], 9.5)
    assert host_refs.map_layers(cpu, gpu) == (1, [0, 1, 0], 9.5)


def test_map_layers_matches_reference_and_brute_force(P):
    rng = np.random.default_rng(7)
    for _ in range(50):
        nb, nl, ni = rng.integers(1, 5), rng.integers(1, 7), rng.integers(1, 9)
        # coarse grid so that ties occur and the first-minimum rule matters
        cpu = rng.integers(0, 6, size=(nb, nl, ni)).astype(float)
        gpu = rng.integers(0, 6, size=(nb, nl, ni)).astype(float)
        got = P.bnn_map_layers(cpu, gpu)
        assert got == host_refs.map_layers(cpu.tolist(), gpu.tolist())
        # brute force: the total is the minimum over batch sizes of the sum of per-layer minima,
        # and no other mapping at that batch size is cheaper
        tot = (cpu + gpu).min(axis=2).sum(axis=1)
        assert got[2] == tot.min() and got[0] == int(np.argmin(tot))
        assert sum((cpu + gpu)[got[0], l, got[1][l]] for l in range(nl)) == got[2]


def test_map_layers_errors(P):
    with pytest.raises(P.BnnError):
        P.bnn_map_layers([[[1.0, -1.0]]], [[[0.0, 0.0]]])
    with pytest.raises(P.BnnError):
        P.bnn_map_layers([[[math.nan]]], [[[0.0]]])


def test_fold_batchnorm_agrees_with_direct_evaluation(P):
    rng = np.random.default_rng(11)
    n = 64
    gamma = rng.normal(0, 1.5, n)
    gamma[:4] = [0.0, 0.0, 1.0, -1.0]
    beta = rng.normal(0, 2, n)
    beta[:2] = [0.5, -0.5]
    mean = rng.normal(0, 20, n)
    var = rng.uniform(0.5, 400, n)
    # exact-tie cases: tau is an integer
    gamma[4], beta[4], mean[4], var[4] = 2.0, -6.0, 4.0, 4.0 - 1e-5 + 0.0   # sqrt(4)=2 with eps -> tau = 4 + 6 = 10
    gamma[5], beta[5], mean[5], var[5] = -2.0, -6.0, 4.0, 4.0 - 1e-5
    eps = 1e-5
    thr, flip = P.bnn_fold_batchnorm(gamma, beta, mean, var, eps)
    for c in range(n):
        for x in range(-120, 121):
            want = host_refs.step_from_batchnorm(x, gamma[c], beta[c], mean[c], var[c], eps)
            got = 1 if ((x > int(thr[c])) != bool(flip[c])) else -1
            assert got == want, (c, x, gamma[c], beta[c], mean[c], var[c], int(thr[c]), int(flip[c]))


def test_fold_batchnorm_closed_forms_and_errors(P):
    # gamma = 1, beta = 0, var + eps = 1: BN(x) = x - mean  -> threshold floor(mean)
    thr, flip = P.bnn_fold_batchnorm([1.0, 1.0, -1.0], [0.0, 0.0, 0.0], [2.5, -3.0, 2.5], [1.0, 1.0, 1.0], 0.0)
    assert list(thr) == [2, -3, 2] and list(flip) == [0, 0, 1]
    with pytest.raises(P.BnnError):
        P.bnn_fold_batchnorm([1.0], [0.0], [0.0], [-1.0], 0.0)
