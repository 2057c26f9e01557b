"""Pin of the special-value search (Eq. 4) to exact arithmetic, for every block size of the
block-size study (Sec. 5.4: 16, 32, 64, 128), the activation format and the FP16-scale format of
Sec. 4.3.  The squared-error norm of every allowed special value is formed with rational numbers
(no rounding, so no summation order), from scaled elements recomputed here with numpy fp32
arithmetic; the oracle's choice must be the exact minimiser wherever the exact minimum is unique,
and its fp64 error must agree with the exact one to within the rounding of a sum of `block` terms.
A dropped element, a wrong candidate order, a run left out of a long block or a min/max mix-up in
the search all fail here."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import golden_rows
from paper_2501_04052_amd import synth

W, A, F16 = 0, 1, 2
MAGS = np.array([float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]])
BASE = np.concatenate([MAGS, -MAGS[1:]])


def _exact_sse(xs_block, v):
    """Exact sum over the block of min_q (xs - q)^2, q in the 15 FP4 values joined by v."""
    vals = np.concatenate([BASE, [v]])
    near = vals[np.argmin(np.abs(xs_block.astype(np.float64)[:, None] - vals[None, :]), axis=1)]
    total = Fraction(0)
    for x, q in zip(xs_block.tolist(), near.tolist()):
        e = Fraction(x) - Fraction(q)
        total += e * e
    return total


CASES = [(W, 16, (5.0, 8.0)), (W, 32, (5.0, 8.0)), (W, 64, (5.0, 7.0)), (W, 128, (5.0, 9.0)),
         (A, 16, (5.0, 0.0)), (A, 64, (5.0, 0.0)), (F16, 128, (5.0, 8.0))]


@pytest.mark.parametrize("fmt,block,sv", CASES)
def test_chosen_special_value_is_the_exact_minimiser(oracle, fmt, block, sv):
    rows, cols = 16, 1024
    if fmt == A:
        x = synth.bf16_bits_to_f32(synth.activation(rows, cols, seed=700 + block, outlier_frac=0.01))
    else:
        x = synth.weight(rows, cols, seed=710 + block, outlier_frac=0.01)
    # a few blocks that sit on a subnormal block scale, where the larger special values can win
    x[0, :block] *= np.float32(1e-3)
    kw = {} if fmt == F16 else {"block": block}
    codes, scales, ts, sse = oracle.quantize(fmt, x, sv=sv, want_sse=True, **kw)
    sh = {W: 6, A: 7, F16: 14}[fmt]
    cand = [sv[0], sv[1], -sv[0], -sv[1]] if fmt != A else [sv[0], -sv[0]]
    ts32 = np.float32(ts)
    checked = unique = 0
    for r in range(rows):
        for b in range(cols // block):
            word = int(scales[r, b])
            s = np.float32(oracle.scale_value(fmt, word & ((1 << sh) - 1)))
            if s == 0:
                continue
            den = np.float32(ts32 * s)                                   # fp32 product, as Eq. 3's denominator
            xs = (x[r, b * block:(b + 1) * block] / den).astype(np.float32)
            exact = [_exact_sse(xs, v) for v in cand]
            best = min(exact)
            winners = [m for m, e in enumerate(exact) if e == best]
            meta = word >> sh
            got = float(sse[r, b])
            assert abs(Fraction(got) - exact[meta]) <= exact[meta] * Fraction(block, 2 ** 52)
            if len(winners) == 1:
                second = min(e for m, e in enumerate(exact) if m != winners[0])
                # closer together than a sum of `block` roundings could tell apart: either is acceptable
                if second - best > best * Fraction(block, 2 ** 51):
                    assert meta == winners[0]
                    unique += 1
            else:
                assert meta == winners[0]                               # exact tie: smallest metadata index
            checked += 1
    assert checked >= rows * cols // block - 2 and unique >= max(8, checked // 8)
