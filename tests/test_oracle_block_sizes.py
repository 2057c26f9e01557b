"""Pins of the oracle for the block sizes of the paper's block-size study (Sec. 5.4: 32, 64, 128
besides the evaluated 16): brute force over all decoded values, the never-worse-than-NVFP4
invariant, reduction to the block-16 encoder when every run of 16 shares its scale, the footprint,
and the linear layer against an independent fp64 matmul."""
import numpy as np
import pytest

from conftest import golden_rows
from paper_2501_04052_amd import synth

W, A = 0, 1
MAGS = np.array([float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]])
BASE = np.concatenate([MAGS, -MAGS[1:]])
BLOCKS = [32, 64, 128]


def unpack(codes):
    return np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1)


def _sum_in_index_order(e):
    """Eq. 4's squared-error norm written out: the plain sum over the block's elements in index
    order k = 0 .. block-1 (every term is exact in fp64; only the order of the additions rounds)."""
    acc = np.zeros(e.shape[0])
    for k in range(e.shape[1]):
        acc = acc + e[:, k]
    return acc


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("fmt,sv", [(W, (5.0, 8.0)), (W, (5.0, 7.0)), (A, (5.0, 0.0))])
def test_search_is_brute_force_optimal(oracle, block, fmt, sv):
    """Blocks [6, free...] with tensor scale 1 given: the block scale is exactly 1, X^Scaled is the
    block itself, and Eq. 4-5 can be brute-forced over all 16 decoded values per element."""
    rng = np.random.default_rng(100 + block)
    x = rng.uniform(-6.2, 6.2, size=(1500, block)).astype(np.float32)
    x[:, 0] = 6.0
    x[:, 1:] = np.clip(x[:, 1:], -6.0, 6.0)
    x[::7, 5] = 5.0                                       # exact ties with the special value
    x[::11, 17] = -5.0
    codes, scales, ts, sse = oracle.quantize(fmt, x, sv=sv, given_tensor_scale=1.0, want_sse=True, block=block)
    assert scales.shape == (1500, 1) and sse.shape == (1500, 1)
    sh = 6 if fmt == W else 7
    assert np.all(oracle.scale_value(fmt, int(scales[0, 0] & ((1 << sh) - 1))) == 1.0)
    assert np.all((scales & ((1 << sh) - 1)) == (scales[0, 0] & ((1 << sh) - 1)))
    cand = [sv[0], sv[1], -sv[0], -sv[1]] if fmt == W else [sv[0], -sv[0]]
    xs = x.astype(np.float64)
    errs = []
    for v in cand:
        vals = np.concatenate([BASE, [v]])
        errs.append(_sum_in_index_order(np.min((xs[:, :, None] - vals[None, None, :]) ** 2, axis=2)))
    errs = np.stack(errs, axis=1)
    assert np.array_equal(scales[:, 0] >> sh, np.argmin(errs, axis=1))
    assert np.array_equal(sse[:, 0], errs.min(axis=1))
    dq = oracle.dequant(fmt, codes, scales, ts, sv=sv, want=("sq",))["sq"]
    assert np.array_equal(_sum_in_index_order((xs - dq) ** 2), errs.min(axis=1))
    assert len(set((scales[:, 0] >> sh).tolist())) > 1   # more than one special value gets chosen


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("fmt", [W, A])
def test_never_worse_than_plain_fp4_under_identical_scale(oracle, block, fmt):
    x = synth.weight(48, 1024, seed=300 + block, outlier_frac=0.01)
    if fmt == A:
        x = synth.bf16_bits_to_f32(synth.activation(48, 1024, seed=301 + block, outlier_frac=0.01))
    sv = (5.0, 8.0) if fmt == W else (5.0, 0.0)
    c_r, s_r, ts_r, sse_r = oracle.quantize(fmt, x, sv=sv, want_sse=True, block=block)
    c_n, s_n, ts_n, sse_n = oracle.quantize(fmt, x, sv=sv, nsv=0, want_sse=True, block=block)
    sh = 6 if fmt == W else 7
    assert ts_r == ts_n and np.array_equal(s_r & ((1 << sh) - 1), s_n & ((1 << sh) - 1))
    assert np.all(sse_r <= sse_n)
    cr = unpack(c_r).reshape(48, -1, block)
    cn = unpack(c_n).reshape(48, -1, block)
    used = (cr == 8).any(axis=2)
    assert used.any()
    assert np.all(sse_r[used] < sse_n[used])
    assert np.array_equal(cr[~used], cn[~used]) and np.all((s_r >> sh)[~used] == 0)
    assert np.array_equal(cr[cr != 8], cn[cr != 8])      # non-special elements keep their plain code
    assert not (cn == 8).any()


@pytest.mark.parametrize("block", BLOCKS)
def test_same_tensor_scale_and_block_scale_rule_as_block_16(oracle, block):
    """Eq. 1 does not depend on the block size, and a block's scale is Eq. 2 of its absolute maximum:
    the maximum of the block-16 maxima it spans.  Checked through the block-16 encoder: on a tensor
    where every run of `block` elements repeats one run of 16, both encoders must agree exactly."""
    base = synth.weight(32, 256, seed=400 + block, outlier_frac=0.01)
    reps = block // 16
    x = np.repeat(base.reshape(32, 16, 16), reps, axis=1).reshape(32, 256 * reps)   # each 16-run repeated
    c16, s16, t16 = oracle.quantize(W, x, block=16)
    cb, sb, tb = oracle.quantize(W, x, block=block)
    assert t16 == tb
    assert np.array_equal(sb, s16[:, ::reps])            # same scale code and same special value
    assert np.array_equal(np.repeat(sb, reps, axis=1), s16)
    assert np.array_equal(cb, c16)
    d16 = oracle.dequant(W, c16, s16, t16)["f32"]
    db = oracle.dequant(W, cb, sb, tb)["f32"]
    assert np.array_equal(d16, db)


@pytest.mark.parametrize("block", BLOCKS)
def test_footprint_and_bad_shapes(oracle, block):
    x = synth.weight(8, 256, seed=5)
    codes, scales, ts = oracle.quantize(W, x, block=block)
    assert codes.nbytes + scales.nbytes == 8 * 256 * (4 + 8 / block) / 8
    with pytest.raises(ValueError):
        oracle.quantize(W, synth.weight(2, block + 16, seed=6), block=block)
    with pytest.raises(ValueError):
        oracle.quantize(W, synth.weight(2, 96, seed=6), block=48)


@pytest.mark.parametrize("wb,ab", [(32, 16), (64, 64), (128, 32)])
def test_linear_equals_fp64_matmul_of_decoded_operands(oracle, wb, ab):
    n, k, m = 24, 512, 9
    wq = oracle.quantize(W, synth.weight(n, k, seed=500 + wb, outlier_frac=0.01), block=wb)
    a_bits = synth.activation(m, k, seed=501 + ab, outlier_frac=0.01)
    aq = oracle.quantize(A, a_bits, sv=(5.0, 0.0), block=ab)
    wd = oracle.dequant(W, *wq, want=("sq",))["sq"]
    ad = oracle.dequant(A, *aq, sv=(5.0, 0.0), want=("sq",))["sq"]
    y64, y16 = oracle.linear(wq, a_bf16=a_bits)
    ref = synth.bf16_bits_to_f32(a_bits).astype(np.float64) @ wd.T * float(wq[2])
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-300)
    y64q, _ = oracle.linear(wq, a_q=aq)
    refq = ad @ wd.T * float(wq[2]) * float(aq[2])
    assert np.allclose(y64q, refq, rtol=1e-12, atol=1e-300)
