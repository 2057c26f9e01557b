"""razer_linear_static -- the entry point for callers that cannot allocate (its K-slices meet in a
static device array inside the library) -- against razer_linear with a caller-owned workspace:
same kernels, so the bf16 outputs must be identical bit for bit.  Two calls in a row share the
static array, the second with a smaller input, so stale contents of the first would show."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import binding, synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err

pytestmark = pytest.mark.gpu
W = 0


def _weights(oracle, n, k, seed):
    w = synth.weight(n, k, seed=seed, outlier_frac=0.002)
    wq = oracle.quantize(W, w)
    return wq, razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))


def test_static_workspace_entry_matches_razer_linear_on_two_calls_in_a_row(oracle):
    cases = [(1024, 4096, 16, 11), (320, 1536, 7, 12)]          # (n, k, m, seed): K-slices through the scratch
    for n, k, m, seed in cases:
        print("razer_linear_static", n, k, m, flush=True)
        assert razer.razer_workspace_bytes(2, n, k, m) > 0       # this size does use the scratch buffer
        wq, wt = _weights(oracle, n, k, seed)
        a = synth.activation(m, k, seed=seed + 100)
        a_dev = bf16_bits_to_dev(a)
        y_ws = razer.razer_linear(wt, a_dev)
        y_st = torch.full((m, n), 7.0, dtype=torch.bfloat16, device="cuda")
        razer.razer_linear_static(wt, a_dev, y_st)
        torch.cuda.synchronize()
        got = dev_to_bf16_bits(y_st)
        assert np.array_equal(got, dev_to_bf16_bits(y_ws))
        y64, _ = oracle.linear(wq, a_bf16=a)
        assert max_rel_err(got, y64) <= TOL


def test_static_workspace_entry_refuses_sizes_beyond_its_array(oracle):
    """Shapes whose K-slices exceed RAZER_STATIC_WORKSPACE_BYTES come back as RAZER_ERR_WORKSPACE
    before anything is launched (the pointers below are never dereferenced)."""
    L = binding.load_library()
    t = binding._Tensor()
    t.codes, t.scales, t.tensor_scale = 0x1000, 0x2000, 0x3000
    t.rows, t.cols = 28672, 8192
    t.cfg = binding._cfg(W, (5.0, 8.0))
    assert razer.razer_workspace_bytes(2, 28672, 8192, 32) > (32 << 20)
    st = L.razer_linear_static(ctypes.byref(t), ctypes.c_void_p(0x4000), None, 32, ctypes.c_void_p(0x5000), 28672, None)
    assert st == 5
    assert L.razer_linear_static(None, None, None, 1, None, 0, None) == 1
