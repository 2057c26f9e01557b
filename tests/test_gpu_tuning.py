"""Every launch shape the tuner may pick (include/razer_tune.h), forced one at a time through
razer_tune_force, against the CPU oracle: the choice of a shape must never change a result beyond fp32
summation order.  Ragged N, ragged K, single and grouped launches, 16- and 64-element blocks."""
import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import binding, synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err

pytestmark = pytest.mark.gpu
W = 0
SV = (5.0, 8.0)


def _rand_weights(n, k, seed, block=16):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(n, k // block), dtype=np.uint8)
    wq = (codes, scales, np.float32(2.0 ** -9))
    return wq, razer.RazerTensor.from_host(*wq, W, SV)


def _check(oracle, family, shape, m, ns, k, block=16, seed=0):
    print("tuning family", family, "shape", shape, "m", m, "ns", ns, "k", k, "block", block, flush=True)
    a = synth.activation(m, k, seed=9700 + m + k)
    a_dev = bf16_bits_to_dev(a)
    ws = [_rand_weights(n, k, 9800 + seed + i + n, block) for i, n in enumerate(ns)]
    razer.razer_tune_force(family, shape)
    try:
        src, got_shape = razer.razer_tune_lookup(family, m, sum(ns), k)
        assert src == 1 and got_shape[:len(shape)] == tuple(shape)
        if len(ns) == 1:
            ys = [razer.razer_linear(ws[0][1], a_dev)]
        else:
            ys = razer.razer_linear_grouped([w[1] for w in ws], a_dev)
        torch.cuda.synchronize()
    finally:
        razer.razer_tune_force(family, None)
    for (wq, _), y in zip(ws, ys):
        y64, _ = oracle.linear(wq, a_bf16=a)
        err = max_rel_err(dev_to_bf16_bits(y), y64)
        assert err <= TOL, (family, shape, err)


SMALL_BATCH_SHAPES = [(1, 1, 2), (1, 1, 4), (1, 2, 2), (1, 2, 4), (1, 2, 8), (0, 4, 1), (0, 4, 2), (0, 4, 4), (0, 8, 1)]


@pytest.mark.parametrize("shape", SMALL_BATCH_SHAPES)
@pytest.mark.parametrize("m,ns,k,block", [(5, (1000,), 4160, 16), (16, (328, 200), 4160, 16), (9, (72,), 512, 64),
                                          (16, (100, 36, 4), 34944, 16), (12, (40, 24), 2048 + 128, 128)])
def test_small_batch_shapes(oracle, shape, m, ns, k, block):
    _check(oracle, binding.TUNE_SMALL_BATCH, shape, m, ns, k, block)


def test_small_batch_in_workgroup_shape_is_ignored_above_16_rows(oracle):
    """17..32 activation rows always take the K-sliced kernel: a forced K-in-workgroup shape falls back."""
    _check(oracle, binding.TUNE_SMALL_BATCH, (1, 2, 4), 20, (200,), 1024)
    _check(oracle, binding.TUNE_SMALL_BATCH, (1, 2, 4), 32, (64, 64), 4096)


@pytest.mark.parametrize("shape", [(2, 1), (2, 2), (4, 1), (8, 1)])
@pytest.mark.parametrize("m,ns,k,block", [(1, (333,), 4096 + 32, 16), (1, (100, 57, 8), 11008, 16), (1, (41,), 28672, 16),
                                          (1, (50,), 4096, 64), (3, (20,), 32768 + 2048, 16)])
def test_gemv_shapes(oracle, shape, m, ns, k, block):
    _check(oracle, binding.TUNE_GEMV, shape, m, ns, k, block)


@pytest.mark.parametrize("shape", [(4,), (8,)])
@pytest.mark.parametrize("m,ns,k,block", [(2, (97, 40), 4096, 16), (3, (333,), 4096 + 32, 16), (4, (100, 57), 11008, 16),
                                          (4, (70,), 16384, 16), (3, (120, 36), 4096 + 128, 64), (4, (50,), 11008 + 64, 32),
                                          (2, (33,), 8192, 128)])
def test_gemv_quad_shapes(oracle, shape, m, ns, k, block):
    _check(oracle, binding.TUNE_GEMV_QUAD, shape, m, ns, k, block)


@pytest.mark.parametrize("shape", [(1,), (3,), (16,)])
@pytest.mark.parametrize("m,ns,k", [(40, (300,), 2048 + 32), (100, (256, 132), 4096), (128, (200,), 1024)])
def test_gemm_slice_counts(oracle, shape, m, ns, k):
    _check(oracle, binding.TUNE_GEMM_SLICES, shape, m, ns, k)
