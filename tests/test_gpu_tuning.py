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


SMALL_BATCH_SHAPES = [(1, 1, 1), (1, 1, 2), (1, 1, 3), (1, 1, 4), (1, 2, 1), (1, 2, 2), (1, 2, 3), (1, 2, 4), (1, 2, 8),
                      (0, 4, 1), (0, 4, 2), (0, 4, 4), (0, 8, 1)]


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


@pytest.mark.parametrize("m,ns,k,block", [(8, (2100,), 1056, 16), (16, (4000,), 4096 + 64, 16), (12, (1400, 1400, 1396), 2048, 16),
                                          (5, (4100,), 11008, 16), (16, (8200,), 8192, 64)])
def test_untabled_small_batch_one_round_of_workgroups(oracle, m, ns, k, block):
    """Up to 16 activation rows, no table entry, and a number of 16-row groups that some G <= 4 turns into one
    round of workgroups: the heuristic takes the K-in-workgroup kernel (no workspace), results as the oracle's."""
    print("one-round heuristic m", m, "ns", ns, "k", k, "block", block, flush=True)
    assert razer.razer_tune_lookup(binding.TUNE_SMALL_BATCH, m, sum(ns), k)[0] == 0       # the heuristic applies
    if len(ns) == 1:
        assert razer.razer_workspace_bytes(binding.OP_LINEAR, ns[0], k, m) == 0
    else:                                       # (the grouped query also covers the fallback to one call per matrix)
        assert razer.razer_workspace_bytes_grouped(list(ns), k, m) == max(razer.razer_workspace_bytes(binding.OP_LINEAR, n, k, m) for n in ns)
    a = synth.activation(m, k, seed=9900 + m + k)
    a_dev = bf16_bits_to_dev(a)
    ws = [_rand_weights(n, k, 9950 + i + n, block) for i, n in enumerate(ns)]
    if len(ns) == 1:
        ys = [razer.razer_linear(ws[0][1], a_dev)]
    else:
        ys = razer.razer_linear_grouped([w[1] for w in ws], a_dev)
    torch.cuda.synchronize()
    for (wq, _), y in zip(ws, ys):
        y64, _ = oracle.linear(wq, a_bf16=a)
        assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL
