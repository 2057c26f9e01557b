"""Pins of the oracle's encoder / decoder: brute force over all decoded values
(Eq. 4), the NVFP4 special case (Eq. 1-3), the never-worse-than-NVFP4
invariant, exact round trips and the footprint."""
import numpy as np
import pytest

from conftest import golden_rows
from paper_2501_04052_amd import synth

W, A = 0, 1
MAGS = np.array([float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]])
BASE = np.concatenate([MAGS, -MAGS[1:]])                 # the 15 distinct FP4 values


def unpack(codes):
    lo = codes & 15
    hi = codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)


def nvfp4_round_thresholds(xs):
    """Textbook round-to-nearest-even FP4 cast written with decision thresholds
    (independent of the oracle's search over the table)."""
    a = np.abs(xs.astype(np.float64))
    # midpoints between neighbours; '<=' where the lower neighbour has the even code
    code = np.zeros(a.shape, np.int64)
    code = np.where(a > 0.25, 1, code)      # 0.25 ties to 0   (code 0 even)
    code = np.where(a >= 0.75, 2, code)     # 0.75 ties to 1.0 (code 2 even)
    code = np.where(a > 1.25, 3, code)      # 1.25 ties to 1.0
    code = np.where(a >= 1.75, 4, code)     # 1.75 ties to 2.0 (code 4)
    code = np.where(a > 2.5, 5, code)       # 2.5 ties to 2.0
    code = np.where(a >= 3.5, 6, code)      # 3.5 ties to 4.0 (code 6)
    code = np.where(a > 5.0, 7, code)       # 5.0 ties to 4.0
    neg = (xs < 0) & (code != 0)
    return code + 8 * neg


def test_fp4_rounding_matches_threshold_cast(oracle):
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.uniform(-7, 7, 5000),
                         np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 6.5, 100.0, 0.0, -0.0]),
                         -np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0, 6.5, 100.0]),
                         rng.uniform(-1e-3, 1e-3, 100)]).astype(np.float32)
    ref = nvfp4_round_thresholds(xs)
    got = np.array([oracle.round_fp4(v) for v in xs])
    assert np.array_equal(got, ref)
    assert 8 not in set(got.tolist())                    # plain rounding never emits the remap code


def _seq_sum(e):
    """Sum over the 16 elements in index order (the order the error norm of
    Eq. 4 is accumulated in); every term is exact in fp64."""
    acc = np.zeros(e.shape[0])
    for k in range(e.shape[1]):
        acc = acc + e[:, k]
    return acc


def _blocks_with_known_scale(free, max_elem=6.0, scale_value=1.0):
    """Blocks of 16 = scale_value * [max_elem, free..., 0...].  With tensor scale 1
    given and scale_value a power of two that max_elem/6 rounds to, the block
    scale is exactly scale_value and X^Scaled == [max_elem, free..., 0...], so
    the search can be brute-forced without re-deriving any scaling arithmetic."""
    n, f = free.shape
    x = np.zeros((n, 16), np.float32)
    x[:, 0] = max_elem
    x[:, 1:1 + f] = free
    return x, (x * np.float32(scale_value)).astype(np.float32)


# (format, special values, block max in the scaled domain, scale code, scale value)
# The last two cases sit on the smallest (subnormal) scale, the only place where
# the scaled block maximum can exceed 6 by enough for +-8 to win.
SEARCH_CASES = [(W, (5.0, 8.0), 6.0, 24, 1.0), (W, (5.0, 7.0), 6.0, 24, 1.0),
                (W, (4.5, 9.0), 6.25, 24, 1.0), (A, (5.0, 0.0), 6.0, 56, 1.0),
                (W, (5.0, 8.0), 8.5, 1, 1.0 / 32), (W, (5.0, 9.0), 8.5, 1, 1.0 / 32),
                (A, (5.0, 0.0), 8.5, 1, 1.0 / 512)]


@pytest.mark.parametrize("fmt,sv,bmax,s_code,s_val", SEARCH_CASES)
def test_special_value_search_is_brute_force_optimal(oracle, fmt, sv, bmax, s_code, s_val):
    """Eq. 4-5 on tiny blocks: exhaustive grid over three free elements."""
    lim = np.floor(bmax * 2) / 2
    g = np.arange(-lim, lim + 0.01, 0.5, dtype=np.float32)
    g = np.concatenate([g, np.array([4.4, 4.6, 5.4, 5.6, -4.4, -4.6, -5.4, -5.6, 0.2, -0.3], np.float32)])
    a, b, c = np.meshgrid(g, g, g, indexing="ij")
    free = np.stack([a.ravel(), b.ravel(), c.ravel()], axis=1)
    xs32, x = _blocks_with_known_scale(free, bmax, s_val)
    codes, scales, ts, sse = oracle.quantize(fmt, x, sv=sv, given_tensor_scale=1.0, want_sse=True)
    sh = 6 if fmt == W else 7
    assert np.all((scales[:, 0] & ((1 << sh) - 1)) == s_code)
    assert oracle.scale_value(fmt, s_code) == s_val
    cand = [sv[0], sv[1], -sv[0], -sv[1]] if fmt == W else [sv[0], -sv[0]]
    xs = xs32.astype(np.float64)
    # brute force: for each candidate, each element takes the nearest of all 16 decoded values
    best = None
    for v in cand:
        vals = np.concatenate([BASE, [v]])
        err = _seq_sum(np.min((xs[:, :, None] - vals[None, None, :]) ** 2, axis=2))
        best = err[:, None] if best is None else np.concatenate([best, err[:, None]], axis=1)
    meta_ref = np.argmin(best, axis=1)                   # first minimum = smallest index on ties
    assert np.array_equal(scales[:, 0] >> sh, meta_ref)
    assert np.array_equal(sse[:, 0], best.min(axis=1))
    if bmax > 7 and fmt == W:
        assert (meta_ref % 2 == 1).any()                 # the second pair does get chosen here
    # the codes decode to values achieving that error
    dq = oracle.dequant(fmt, codes, scales, ts, sv=sv, want=("sq",))["sq"] / s_val
    assert np.array_equal(_seq_sum((xs - dq) ** 2), best.min(axis=1))


def test_special_value_search_random_blocks(oracle):
    """Same brute force on dense random blocks (all 15 elements free)."""
    rng = np.random.default_rng(21)
    free = rng.uniform(-6.2, 6.2, size=(4000, 15)).astype(np.float32)
    x, _ = _blocks_with_known_scale(free)
    sv = (5.0, 8.0)
    codes, scales, ts, sse = oracle.quantize(W, x, sv=sv, given_tensor_scale=1.0, want_sse=True)
    xs = x.astype(np.float64)
    errs = []
    for v in (5.0, 8.0, -5.0, -8.0):
        vals = np.concatenate([BASE, [v]])
        # sequential k order like the definition; all terms exact in fp64
        errs.append(_seq_sum(np.min((xs[:, :, None] - vals[None, None, :]) ** 2, axis=2)))
    errs = np.stack(errs, axis=1)
    assert np.array_equal(scales[:, 0] >> 6, np.argmin(errs, axis=1))
    assert np.array_equal(sse[:, 0], errs.min(axis=1))


@pytest.mark.parametrize("fmt", [W, A])
def test_never_worse_than_nvfp4_under_identical_scale(oracle, fmt):
    w = synth.weight(64, 512, seed=77, outlier_frac=0.01)
    if fmt == A:
        w = synth.bf16_bits_to_f32(synth.activation(64, 512, seed=78, outlier_frac=0.01))
    sv = (5.0, 8.0) if fmt == W else (5.0, 0.0)
    c_r, s_r, ts_r, sse_r = oracle.quantize(fmt, w, sv=sv, want_sse=True)
    c_n, s_n, ts_n, sse_n = oracle.quantize(fmt, w, sv=sv, nsv=0, want_sse=True)
    sh = 6 if fmt == W else 7
    mask = (1 << sh) - 1
    assert ts_r == ts_n
    assert np.array_equal(s_r & mask, s_n & mask)        # identical block scales
    assert np.all(s_n >> sh == 0)
    assert np.all(sse_r <= sse_n)
    cr = unpack(c_r).reshape(64, -1, 16)
    cn = unpack(c_n).reshape(64, -1, 16)
    used = (cr == 8).any(axis=2)
    assert used.any() and (~used).any()
    assert np.all(sse_r[used] < sse_n[used])             # a taken special value strictly helps
    assert np.array_equal(sse_r[~used], sse_n[~used])
    assert np.array_equal(cr[~used], cn[~used])          # unused -> bit-identical to NVFP4
    assert np.all((s_r >> sh)[~used] == 0)               # canonical metadata when unused
    assert not (cn == 8).any()
    # every non-special element keeps its NVFP4 code
    keep = cr != 8
    assert np.array_equal(cr[keep], cn[keep])
    # strictly more error in the real (unscaled) domain is impossible as well
    d_r = oracle.dequant(fmt, c_r, s_r, ts_r, sv=sv)["f32"].astype(np.float64)
    d_n = oracle.dequant(fmt, c_n, s_n, ts_n, sv=sv)["f32"].astype(np.float64)
    e_r = ((w - d_r) ** 2).reshape(64, -1, 16).sum(axis=2)
    e_n = ((w - d_n) ** 2).reshape(64, -1, 16).sum(axis=2)
    assert np.all(e_r <= e_n * (1 + 1e-6) + 1e-30)


def test_nvfp4_special_case_matches_textbook_quantizer(oracle):
    """With no special value the encoder is Eq. 1-3: absmax tensor scale, RNE
    block scale, RNE element cast -- checked with numpy fp32 arithmetic and the
    library FP8 cast."""
    import torch
    a = synth.bf16_bits_to_f32(synth.activation(32, 256, seed=5, outlier_frac=0.02))
    codes, scales, ts = oracle.quantize(A, a, nsv=0)
    amax = np.abs(a).max()
    assert ts == np.float32(amax) / np.float32(448.0 * 6.0)
    blk = a.reshape(32, -1, 16)
    t = np.abs(blk).max(axis=2) / (np.float32(ts) * np.float32(6.0))
    s_code = torch.from_numpy(t.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(scales, s_code)
    s = torch.from_numpy(s_code).view(torch.float8_e4m3fn).float().numpy()
    den = (np.float32(ts) * s).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        xs = (blk / den[:, :, None]).astype(np.float32)
    ref = nvfp4_round_thresholds(xs)
    ref = np.where(s[:, :, None] == 0, 0, ref)
    assert np.array_equal(unpack(codes).reshape(32, -1, 16), ref)


@pytest.mark.parametrize("fmt", [W, A])
def test_round_trip_of_representable_tensors(oracle, fmt):
    """A tensor built from representable (tensor scale, block scale, element)
    triples, each block holding +-6 and one block at the largest scale,
    re-encodes to codes that decode bit-identically."""
    rng = np.random.default_rng(9)
    ncodes, qs, sh = (64, 30.0, 6) if fmt == W else (127, 448.0, 7)
    rows, nb = 24, 8
    sv = (5.0, 8.0) if fmt == W else (5.0, 0.0)
    s_codes = rng.integers(ncodes // 2, ncodes, size=(rows, nb))   # normal-range scales
    s_codes[0, 0] = ncodes - 1
    s = np.array([[oracle.scale_value(fmt, c) for c in r] for r in s_codes])
    elem_codes = rng.integers(0, 16, size=(rows, nb, 16))
    elem_codes[elem_codes == 8] = 0
    elem_codes[:, :, 0] = 7 + 8 * rng.integers(0, 2, size=(rows, nb))   # +-6 in every block
    # sprinkle +-5 (reachable special) consistently per block
    meta = rng.integers(0, 2, size=(rows, nb)) * (2 if fmt == W else 1)  # +5 or -5
    spec = rng.random((rows, nb, 16)) < 0.15
    spec[:, :, 0] = False
    q = np.vectorize(oracle.fp4_value)(elem_codes)
    svv = np.where(meta == 0, 5.0, -5.0)
    q = np.where(spec, svv[:, :, None], q)
    delta32 = 2.0 ** -9
    x = (delta32 * s[:, :, None] * q).astype(np.float32).reshape(rows, nb * 16)
    assert np.abs(x).max() == np.float32(delta32 * qs * 6.0)
    codes, scales, ts = oracle.quantize(fmt, x, sv=sv)
    assert ts == np.float32(delta32)                      # Eq. 1 recovers the power-of-two scale
    assert np.array_equal(scales & ((1 << sh) - 1), s_codes)
    back = oracle.dequant(fmt, codes, scales, ts, sv=sv, want=("f32", "bf16"))
    assert np.array_equal(back["f32"].view(np.uint32), x.view(np.uint32))
    got = unpack(codes).reshape(rows, nb, 16)
    assert np.array_equal(got == 8, spec)
    assert np.array_equal((scales >> sh)[spec.any(axis=2)], meta[spec.any(axis=2)])
    assert np.array_equal(back["bf16"], synth.f32_to_bf16_bits(x))


def test_dequant_of_hand_built_block(oracle):
    """Decode a block holding every code once, against the printed value set."""
    codes = np.array([[(2 * i) | ((2 * i + 1) << 4) for i in range(8)]], np.uint8)
    for meta, want_sv in enumerate([5.0, 8.0, -5.0, -8.0]):
        scales = np.array([[(meta << 6) | 0b100100]], np.uint8)          # E=4, M=4 -> 2^1 * 1.5 = 3
        out = oracle.dequant(W, codes, scales, 0.25, sv=(5.0, 8.0), want=("f32", "sq"))
        vals = np.concatenate([MAGS, [want_sv], -MAGS[1:]])
        assert np.array_equal(out["sq"][0], 3.0 * vals)
        assert np.array_equal(out["f32"][0], (0.75 * vals).astype(np.float32))
    scales = np.array([[(1 << 7) | 0b0111000]], np.uint8)                 # activation: E=7,M=0 -> 1.0
    out = oracle.dequant(A, codes, scales, 2.0, sv=(5.0, 0.0), want=("f32",))
    assert out["f32"][0][8] == -10.0 and out["f32"][0][7] == 12.0


def test_zero_and_tiny_blocks(oracle):
    x = np.zeros((2, 64), np.float32)
    codes, scales, ts = oracle.quantize(W, x)
    assert ts == 1.0 and not codes.any() and not scales.any()
    # a block far below the tensor maximum: its scale rounds to 0 and it decodes to zeros
    x[0, 0] = 100.0
    x[1, 16:32] = 1e-4
    codes, scales, ts = oracle.quantize(W, x)
    assert scales[1, 1] == 0 and not codes[1, 8:16].any()
    # small negative values that round to zero keep code 0, never the remap code
    x[1, 32:48] = -0.01
    x[1, 32] = 3.0
    codes, scales, ts = oracle.quantize(W, x)
    assert 8 not in set(unpack(codes)[1, 32:48].tolist()) or (scales[1, 2] >> 6) != 0
    d = oracle.dequant(W, codes, scales, ts)["f32"]
    assert np.all(d[1, 33:48] == 0.0)


def test_footprint_is_4p5_bits_per_element(oracle):
    w = synth.weight(16, 256, seed=1)
    codes, scales, ts = oracle.quantize(W, w)
    assert codes.nbytes + scales.nbytes == w.size * 9 // 16
    assert codes.nbytes + scales.nbytes + 4 == w.size * 9 // 16 + 4
    assert np.float32(ts).nbytes == 4


def test_error_bound_half_grid_gap(oracle):
    """Every in-range scaled element lands within half the local FP4 gap."""
    w = synth.weight(32, 512, seed=3)
    codes, scales, ts = oracle.quantize(W, w)
    sq = oracle.dequant(W, codes, scales, ts, want=("sq",))["sq"]
    s = np.vectorize(lambda c: oracle.scale_value(W, c))(scales & 63)
    den = (np.float32(ts) * s.astype(np.float32)).astype(np.float32)
    ok = np.repeat(den, 16, axis=1) > 0
    xs = np.where(ok, w / np.where(ok, np.repeat(den, 16, axis=1), 1), 0).astype(np.float64)
    q = np.where(ok, sq / np.where(ok, np.repeat(s, 16, axis=1), 1), 0)
    a = np.abs(xs)
    gap = np.select([a <= 2, a <= 4, a <= 6], [0.25, 0.5, 1.0], default=np.inf)
    assert np.all(np.abs(xs - q)[ok] <= gap[ok] + 1e-12)
    assert a[ok].max() <= 6.0 * (1 + 1 / 16) + 1e-6      # RNE block scale keeps the block max near 6


def test_single_pair_error_is_lowest_at_5_and_never_above_plain_fp4(oracle):
    """Sec. 4.2 (discussion of the special-value error figure): adding one pair of special values to
    NVFP4 lowers the quantization error for every allowed pair, with the minimum at +-5, for weights
    and for activations alike."""
    w = synth.weight(128, 2048, seed=31, outlier_frac=0.001)
    a = synth.bf16_bits_to_f32(synth.activation(128, 2048, seed=32, outlier_frac=0.005))

    def err(fmt, x, v, nsv):
        sv = (v, v) if fmt == W else (v, 0.0)
        c, s, t = oracle.quantize(fmt, x, sv=sv, nsv=nsv)
        d = oracle.dequant(fmt, c, s, t, sv=sv)["f32"].astype(np.float64)
        return float(((x - d) ** 2).sum())

    for fmt, x in ((W, w), (A, a)):
        base = err(fmt, x, 5.0, 0)
        rel = {v: err(fmt, x, v, -1) / base for v in (2.5, 3.5, 4.5, 5.0, 5.5, 6.5, 7.0, 8.0, 9.5)}
        assert all(r <= 1.0 for r in rel.values())
        assert min(rel, key=rel.get) == 5.0
        assert rel[5.0] < 0.95 and rel[4.5] < rel[3.5] and rel[5.5] < rel[6.5]     # a dip around 5
        assert rel[8.0] > 0.999                       # beyond 6.375 a pair (almost) never gets used
