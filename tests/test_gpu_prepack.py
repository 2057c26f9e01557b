"""The private interleaved weight layout (razer_prepack): the packed buffer holds exactly the canonical
bytes at the documented offsets, and razer_linear / razer_linear_grouped on a packed tensor give results
bit-identical to the canonical tensor's for every decode-regime kernel (1..4 activation rows, every launch
shape of the streaming and matrix-instruction GEMV, ragged N and K).  Uses outside that regime are refused."""
import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import binding, synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err

pytestmark = pytest.mark.gpu
W = 0
SV = (5.0, 8.0)


def _weights(n, k, seed):
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(n, k // 16), dtype=np.uint8)
    wq = (codes, scales, np.float32(2.0 ** -9))
    return wq, razer.RazerTensor.from_host(*wq, W, SV)


@pytest.mark.parametrize("n,k", [(5, 2048), (7, 4096 + 32), (3, 11008), (2, 32)])
def test_packed_buffer_is_the_documented_permutation(n, k):
    wq, wt = _weights(n, k, 50 + n)
    pk = razer.razer_prepack(wt)
    torch.cuda.synchronize()
    buf = pk.codes.cpu().numpy()
    runs = -(-k // 2048)
    assert buf.size == n * runs * 1152
    buf = buf.reshape(n, runs, 1152)
    for r in range(runs):
        ck = min(2048, k - r * 2048)                                  # elements of this run
        assert np.array_equal(buf[:, r, :ck // 2], wq[0][:, r * 1024:r * 1024 + ck // 2])
        assert np.array_equal(buf[:, r, 1024:1024 + ck // 16], wq[1][:, r * 128:r * 128 + ck // 16])
        assert not buf[:, r, ck // 2:1024].any() and not buf[:, r, 1024 + ck // 16:].any()   # padding is zero


@pytest.mark.parametrize("m", [1, 2, 3, 4])
@pytest.mark.parametrize("n,k", [(333, 4096), (64, 4096 + 32), (50, 11008), (41, 28672), (20, 16384 + 2048)])
def test_linear_on_packed_weights_is_bit_identical(oracle, m, n, k):
    print("prepack linear", m, n, k, flush=True)
    wq, wt = _weights(n, k, 60 + n + m)
    pk = razer.razer_prepack(wt)
    a = synth.activation(m, k, seed=61 + m + k)
    a_dev = bf16_bits_to_dev(a)
    shapes = [(2, 1), (2, 2), (4, 1), (8, 1)] if m <= 2 else [(4,), (8,)]
    fam = binding.TUNE_GEMV if m <= 2 else binding.TUNE_GEMV_QUAD
    for shape in [None] + shapes:
        razer.razer_tune_force(fam, shape)
        try:
            y_c = razer.razer_linear(wt, a_dev)
            y_p = razer.razer_linear(pk, a_dev)
            torch.cuda.synchronize()
        finally:
            razer.razer_tune_force(fam, None)
        assert torch.equal(y_c, y_p), (m, n, k, shape)
    y64, _ = oracle.linear(wq, a_bf16=a)
    assert max_rel_err(dev_to_bf16_bits(y_p), y64) <= TOL


@pytest.mark.parametrize("m", [1, 4])
def test_grouped_on_packed_weights_is_bit_identical(oracle, m):
    k = 4096
    ws = [_weights(n, k, 70 + n) for n in (100, 57, 200)]
    pks = [razer.razer_prepack(w[1]) for w in ws]
    a = synth.activation(m, k, seed=71 + m)
    a_dev = bf16_bits_to_dev(a)
    ys_c = razer.razer_linear_grouped([w[1] for w in ws], a_dev)
    ys_p = razer.razer_linear_grouped(pks, a_dev)
    torch.cuda.synchronize()
    for (wq, _), yc, yp in zip(ws, ys_c, ys_p):
        assert torch.equal(yc, yp)
        assert max_rel_err(dev_to_bf16_bits(yp), oracle.linear(wq, a_bf16=a)[0]) <= TOL


def test_uses_outside_the_decode_regime_are_refused():
    wq, wt = _weights(64, 4096, 80)
    pk = razer.razer_prepack(wt)
    a5 = bf16_bits_to_dev(synth.activation(5, 4096, seed=81))
    for call in (lambda: razer.razer_linear(pk, a5), lambda: razer.razer_dequant(pk), lambda: razer.razer_prepack(pk),
                 lambda: razer.razer_linear_grouped([pk, wt], a5[:1].contiguous())):
        with pytest.raises(razer.RazerError) as e:
            call()
        assert e.value.status == 4
    # a format the layout is not defined for
    w128 = razer.RazerTensor.from_host(wq[0], wq[1][:, ::8].copy(), wq[2], W, SV)
    assert w128.block == 128
    with pytest.raises(razer.RazerError) as e:
        razer.razer_prepack(w128)
    assert e.value.status == 4
