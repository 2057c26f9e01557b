"""Pins of the oracle's linear layer: the plain definition of the matmul on the
decoded operands, evaluated independently with numpy fp64."""
import numpy as np

from paper_2501_04052_amd import synth

W, A = 0, 1


def test_linear_w4a16_equals_fp64_matmul_of_decoded_weights(oracle):
    w = synth.weight(48, 256, seed=10, outlier_frac=0.01)
    a = synth.activation(5, 256, seed=11)
    wq = oracle.quantize(W, w)
    y64, y16 = oracle.linear(wq, a_bf16=a)
    sq = oracle.dequant(W, *wq, want=("sq",))["sq"]
    ref = (synth.bf16_bits_to_f32(a).astype(np.float64) @ sq.T) * float(wq[2])
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-300)
    assert np.array_equal(y16, synth.f32_to_bf16_bits(ref.astype(np.float32))) or \
        np.mean(y16 != synth.f32_to_bf16_bits(ref.astype(np.float32))) < 0.01   # double rounding only
    # against the decoded fp32 weights: same up to the single fp32 rounding of each weight
    wd = oracle.dequant(W, *wq)["f32"].astype(np.float64)
    ref2 = synth.bf16_bits_to_f32(a).astype(np.float64) @ wd.T
    assert np.allclose(y64, ref2, rtol=1e-5, atol=1e-6)


def test_linear_row_and_column_selection(oracle):
    w = synth.weight(40, 128, seed=12)
    a = synth.activation(9, 128, seed=13)
    wq = oracle.quantize(W, w)
    y64, y16 = oracle.linear(wq, a_bf16=a)
    rows = np.array([0, 3, 8], np.int64)
    cols = np.array([1, 2, 17, 39], np.int64)
    s64, s16 = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
    assert np.array_equal(s64, y64[np.ix_(rows, cols)])
    assert np.array_equal(s16, y16[np.ix_(rows, cols)])


def test_linear_w4a4_equals_fp64_matmul_of_both_decoded_operands(oracle):
    w = synth.weight(32, 256, seed=14, outlier_frac=0.01)
    a = synth.activation(7, 256, seed=15, outlier_frac=0.01)
    wq = oracle.quantize(W, w)
    aq = oracle.quantize(A, a, sv=(5.0, 0.0))
    y64, _ = oracle.linear(wq, a_q=aq)
    sw = oracle.dequant(W, *wq, want=("sq",))["sq"]
    sa = oracle.dequant(A, *aq, sv=(5.0, 0.0), want=("sq",))["sq"]
    ref = (sa @ sw.T) * float(wq[2]) * float(aq[2])
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-300)
    # and it approximates the unquantized product (sanity of the whole chain)
    exact = synth.bf16_bits_to_f32(a).astype(np.float64) @ w.astype(np.float64).T
    rel = np.linalg.norm(y64 - exact) / np.linalg.norm(exact)
    assert rel < 0.2


def test_quantized_linear_approximates_dense_linear(oracle):
    """The quantized layer tracks the fp64 product of the unquantized operands
    within the error a 4.5-bit format allows, and RaZeR is not worse than NVFP4."""
    w = synth.weight(64, 512, seed=16)
    a = synth.activation(8, 512, seed=17)
    exact = synth.bf16_bits_to_f32(a).astype(np.float64) @ w.astype(np.float64).T
    y_r, _ = oracle.linear(oracle.quantize(W, w), a_bf16=a)
    y_n, _ = oracle.linear(oracle.quantize(W, w, nsv=0), a_bf16=a)
    e_r = np.linalg.norm(y_r - exact) / np.linalg.norm(exact)
    e_n = np.linalg.norm(y_n - exact) / np.linalg.norm(exact)
    assert e_r < 0.12 and e_r <= e_n * 1.02
