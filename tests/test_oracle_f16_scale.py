"""Pins of the oracle for the format of the paper's own weight-only kernel (Sec. 4.3): blocks of 128
with one FP16 scale whose sign bit and most significant exponent bit carry the 2 metadata bits.
The scale codec is pinned to a library half-precision cast, the search to brute force, the encoder
to the never-worse-than-plain-FP4 invariant and to the block-128 encoder with the 8-bit scale where
the two scale grids coincide, and the linear layer to an independent fp64 matmul."""
import numpy as np
import pytest

from conftest import golden_rows
from paper_2501_04052_amd import synth

W, A, F16 = 0, 1, 2
MAGS = np.array([float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]])
BASE = np.concatenate([MAGS, -MAGS[1:]])


def unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1)


def _sum_in_index_order(e):
    """Eq. 4's squared-error norm written out: the plain sum over the block's elements in index
    order k = 0 .. block-1 (every term is exact in fp64; only the order of the additions rounds)."""
    acc = np.zeros(e.shape[0])
    for k in range(e.shape[1]):
        acc = acc + e[:, k]
    return acc


def test_scale_codec_is_ieee_half_with_the_top_exponent_bit_clear(oracle):
    """All 16384 codes decode like the IEEE half with the same low 14 bits (sign and exponent MSB
    zero); the largest is 2 - 2^-10; no code is Inf or NaN."""
    codes = np.arange(16384, dtype=np.uint16)
    lib_vals = codes.view(np.float16).astype(np.float64)
    ours = np.array([oracle.e4m10_value(int(c)) for c in codes])
    assert np.array_equal(ours, lib_vals)
    assert np.all(np.isfinite(ours)) and np.all(np.diff(ours) > 0)
    assert oracle.scale_max(F16) == 2.0 - 2.0 ** -10 == ours[-1]
    assert oracle.e4m10_value(0x3C00) == 1.0 and oracle.e4m10_value(1) == 2.0 ** -24


def test_scale_rounding_is_the_library_half_cast_saturated(oracle):
    """Eq. 2's rounding onto this grid = round-to-nearest-even cast to half (a library routine),
    saturated at the largest code."""
    rng = np.random.default_rng(1)
    ts = np.concatenate([rng.uniform(0, 2.2, 4000), 2.0 ** rng.uniform(-26, 1, 4000),
                         [0.0, 2.0 ** -25, 3 * 2.0 ** -25, 1.0, 1.9990234375, 1.99951171875, 2.0, 7.5]]).astype(np.float32)
    # exact ties between neighbouring codes
    ties = (np.arange(1, 2000, dtype=np.float64) + 0.5) * 2.0 ** -24
    ts = np.concatenate([ts, ties.astype(np.float32), (1.0 + (np.arange(50) + 0.5) / 1024).astype(np.float32)])
    want = np.minimum(ts.astype(np.float16).view(np.uint16).astype(np.int64), 0x3FFF)
    want[ts >= 2.0] = 0x3FFF                                       # the cast itself would leave the grid here
    got = np.array([oracle.round_scale(F16, float(t)) for t in ts])
    assert np.array_equal(got, want)


def test_layout_block_and_footprint(oracle):
    x = synth.weight(8, 512, seed=5)
    codes, scales, ts = oracle.quantize(F16, x)
    assert codes.shape == (8, 256) and scales.shape == (8, 4) and scales.dtype == np.uint16
    assert codes.nbytes + scales.nbytes == 8 * 512 * 4.125 / 8            # 4.125 bits per weight
    assert ts == np.float32(np.abs(x).max()) / np.float32((2.0 - 2.0 ** -10) * 6.0)   # Eq. 1 with this grid's maximum
    with pytest.raises(ValueError):
        oracle.quantize(F16, synth.weight(2, 192, seed=6))               # not a multiple of 128
    z = np.zeros((2, 128), np.float32)
    cz, sz, tz = oracle.quantize(F16, z)
    assert tz == 1.0 and not cz.any() and not sz.any()
    # the block that holds the tensor maximum gets the largest scale code
    r, c = np.unravel_index(np.abs(x).argmax(), x.shape)
    assert (scales[r, c // 128] & 0x3FFF) == 0x3FFF


@pytest.mark.parametrize("sv", [(5.0, 8.0), (5.0, 7.0), (4.5, 9.0)])
def test_search_is_brute_force_optimal(oracle, sv):
    """Blocks [6, free...] with tensor scale 1 given: the block scale is exactly 1 (code 0x3C00),
    X^Scaled is the block itself, and Eq. 4-5 can be brute-forced over all 16 decoded values."""
    rng = np.random.default_rng(110)
    x = rng.uniform(-6.2, 6.2, size=(1500, 128)).astype(np.float32)
    x[:, 0] = 6.0
    x[:, 1:] = np.clip(x[:, 1:], -6.0, 6.0)
    x[::7, 5] = 5.0
    x[::11, 100] = -5.0
    codes, scales, ts, sse = oracle.quantize(F16, x, sv=sv, given_tensor_scale=1.0, want_sse=True)
    assert np.all((scales & 0x3FFF) == 0x3C00)
    cand = [sv[0], sv[1], -sv[0], -sv[1]]
    xs = x.astype(np.float64)
    errs = []
    for v in cand:
        vals = np.concatenate([BASE, [v]])
        errs.append(_sum_in_index_order(np.min((xs[:, :, None] - vals[None, None, :]) ** 2, axis=2)))
    errs = np.stack(errs, axis=1)
    assert np.array_equal(scales[:, 0] >> 14, np.argmin(errs, axis=1))
    assert np.array_equal(sse[:, 0], errs.min(axis=1))
    dq = oracle.dequant(F16, codes, scales, ts, sv=sv, want=("sq",))["sq"]
    assert np.array_equal(_sum_in_index_order((xs - dq) ** 2), errs.min(axis=1))
    assert len(set((scales[:, 0] >> 14).tolist())) > 1


def test_never_worse_than_plain_fp4_under_identical_scale(oracle):
    x = synth.weight(48, 1024, seed=310, outlier_frac=0.01)
    c_r, s_r, ts_r, sse_r = oracle.quantize(F16, x, want_sse=True)
    c_n, s_n, ts_n, sse_n = oracle.quantize(F16, x, nsv=0, want_sse=True)
    assert ts_r == ts_n and np.array_equal(s_r & 0x3FFF, s_n)
    assert np.all(sse_r <= sse_n)
    cr = unpack(c_r).reshape(48, -1, 128)
    cn = unpack(c_n).reshape(48, -1, 128)
    used = (cr == 8).any(axis=2)
    assert used.any()
    assert np.all(sse_r[used] < sse_n[used])
    assert np.array_equal(cr[~used], cn[~used]) and np.all((s_r >> 14)[~used] == 0)
    assert np.array_equal(cr[cr != 8], cn[cr != 8])
    assert not (cn == 8).any()


def test_agrees_with_the_byte_scale_encoder_where_both_grids_hold_the_scale(oracle):
    """With the tensor scale given as 1 and every block maximum 6 * (an E3M3 value that is also a
    half below 2), Eq. 2 lands on a value both scale grids hold exactly, so the FP16-scale encoder
    and the 8-bit-scale encoder at block 128 must choose the same codes and special values."""
    rng = np.random.default_rng(7)
    scl = np.array([0.25, 0.5, 0.625, 1.0, 1.125, 1.5, 1.875])           # E3M3 values that are halves < 2
    x = rng.standard_normal((40, 3 * 128)).astype(np.float32)
    for r in range(40):
        for b in range(3):
            blk = x[r, 128 * b:128 * b + 128]
            s = scl[(r + b) % len(scl)]
            blk *= np.float32(5.9 * s) / np.abs(blk).max()
            blk[(r * 3 + b) % 128] = np.float32(6.0 * s)
    c8, s8, _ = oracle.quantize(W, x, given_tensor_scale=1.0, block=128)
    c16, s16, _ = oracle.quantize(F16, x, given_tensor_scale=1.0)
    assert np.array_equal(c8, c16)
    assert np.array_equal(s8 >> 6, s16 >> 14)
    v8 = np.array([oracle.scale_value(W, int(c) & 63) for c in s8.ravel()])
    v16 = np.array([oracle.scale_value(F16, int(c) & 0x3FFF) for c in s16.ravel()])
    assert np.array_equal(v8, v16)
    assert np.array_equal(oracle.dequant(W, c8, s8, 1.0)["f32"], oracle.dequant(F16, c16, s16, 1.0)["f32"])


def test_dequant_is_one_fp32_rounding_of_the_exact_product(oracle):
    rng = np.random.default_rng(9)
    codes = rng.integers(0, 256, size=(16, 192), dtype=np.uint8)
    scales = rng.integers(0, 65536, size=(16, 3), dtype=np.uint16)
    ts = np.float32(3.1e-3)
    out = oracle.dequant(F16, codes, scales, ts, sv=(5.0, 7.0), want=("f32", "bf16", "sq"))
    el = unpack(codes)
    sc = np.repeat(scales, 128, axis=1)
    s = (sc & 0x3FFF).astype(np.uint16).view(np.float16).astype(np.float64)
    meta = sc >> 14
    cand = np.array([5.0, 7.0, -5.0, -7.0])
    q = np.where(el == 8, cand[meta], np.where(el < 8, MAGS[el & 7], -MAGS[el & 7]))
    assert np.array_equal(out["sq"], s * q)
    assert np.array_equal(out["f32"], (np.float64(ts) * s * q).astype(np.float32))
    b = np.array([oracle.f64_to_bf16(float(v)) for v in out["f32"].ravel()[:4000]], dtype=np.uint16)
    assert np.array_equal(out["bf16"].ravel()[:4000], b)


def test_linear_equals_fp64_matmul_of_decoded_weights(oracle):
    n, k, m = 24, 512, 9
    wq = oracle.quantize(F16, synth.weight(n, k, seed=520, outlier_frac=0.01))
    a_bits = synth.activation(m, k, seed=521, outlier_frac=0.01)
    wd = oracle.dequant(F16, *wq, want=("sq",))["sq"]
    y64, y16 = oracle.linear(wq, a_bf16=a_bits)
    ref = synth.bf16_bits_to_f32(a_bits).astype(np.float64) @ wd.T * float(wq[2])
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-300)
    rows, cols = np.array([0, 8]), np.array([3, 23, 5])
    ys, _ = oracle.linear(wq, a_bf16=a_bits, rows=rows, cols=cols)
    assert np.array_equal(ys, y64[np.ix_(rows, cols)])
