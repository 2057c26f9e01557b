"""Pins of the oracle's number formats against what the paper prints and
against library routines (never against the oracle's own formulas)."""
import itertools

import numpy as np
import pytest
import torch

from conftest import golden_rows

W, A = 0, 1


def test_fp4_table_matches_printed_set(oracle):
    mags = [float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]]
    assert len(mags) == 8
    for c in range(8):
        assert oracle.fp4_value(c) == mags[c]
        assert oracle.fp4_value(c + 8) == -mags[c]
    # code 8 is the redundant (negative) zero
    assert oracle.fp4_value(8) == 0.0 and np.signbit(oracle.fp4_value(8))
    assert oracle.REMAP_CODE == 8
    # exactly 15 distinct values
    assert len({oracle.fp4_value(c) for c in range(16)}) == 15


def test_e4m3_values_match_library_fp8(oracle):
    codes = torch.arange(127, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).float().numpy()
    for c in range(127):
        assert oracle.e4m3_value(c) == float(ref[c]), c
    assert oracle.scale_max(A) == 448.0


def test_e3m3_is_e4m3_shifted_by_bias(oracle):
    # E3M3 with bias 3 has the value of the E4M3 code with the same bits times 2^4.
    codes = torch.arange(64, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).float().numpy() * 16.0
    for c in range(64):
        assert oracle.e3m3_value(c) == float(ref[c]), c
    assert oracle.scale_max(W) == 30.0
    assert oracle.e3m3_value(1) == 1.0 / 32.0
    # strictly increasing grid
    vals = [oracle.e3m3_value(c) for c in range(64)]
    assert all(b > a for a, b in zip(vals, vals[1:]))


def _sweep_points(maxv, grid_vals):
    rng = np.random.default_rng(11)
    pts = [rng.uniform(0, maxv, 4000).astype(np.float32),
           np.exp(rng.uniform(np.log(1e-4), np.log(maxv), 4000)).astype(np.float32)]
    g = np.array(grid_vals, np.float64)
    mids = ((g[1:] + g[:-1]) / 2).astype(np.float32)            # exact ties
    pts += [mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(1e9)),
            np.array(grid_vals, np.float32)]
    return np.concatenate(pts)


def test_e4m3_rounding_matches_library_cast(oracle):
    grid = [oracle.e4m3_value(c) for c in range(127)]
    t = _sweep_points(448.0, grid)
    t = t[t <= 448.0]
    ref = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.round_scale(A, x) for x in t])
    assert np.array_equal(got, ref)
    # beyond the grid: saturate at the largest finite code
    assert oracle.round_scale(A, 1e9) == 126
    assert oracle.round_scale(A, 470.0) == 126


def test_e3m3_rounding_matches_library_cast_of_shifted_value(oracle):
    grid = [oracle.e3m3_value(c) for c in range(64)]
    t = _sweep_points(30.0, grid)
    t = t[t <= 30.0]
    ref = torch.from_numpy(t / np.float32(16)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.round_scale(W, x) for x in t])
    ok = ref < 64
    assert np.array_equal(got[ok], ref[ok])
    assert np.all(got[~ok] == 63)                     # 31 would round up past the grid
    assert oracle.round_scale(W, 1e9) == 63 and oracle.round_scale(W, 31.5) == 63
    assert oracle.round_scale(W, 0.0) == 0
    assert oracle.round_scale(W, 1.0 / 64.0) == 0     # tie between 0 and 1/32 -> even code 0
    assert oracle.round_scale(W, 3.0 / 64.0) == 2     # tie between codes 1 and 2 -> 2


def test_scale_rounding_is_brute_force_nearest(oracle):
    rng = np.random.default_rng(5)
    for fmt, n, mx in ((W, 64, 30.0), (A, 127, 448.0)):
        grid = np.array([oracle.scale_value(fmt, c) for c in range(n)])
        for t in rng.uniform(0, mx * 1.05, 500).astype(np.float32):
            c = oracle.round_scale(fmt, t)
            assert abs(grid[c] - float(t)) == np.min(np.abs(grid - float(t)))


def test_decoder_offset_register_worked_example(oracle):
    rows = golden_rows("decoder_offset_example.txt")
    bits, off, mag, signed = rows[0]
    reg = int(bits, 2)
    assert oracle.sv_from_offset_reg(reg) - 6.0 == float(off)
    assert oracle.sv_from_offset_reg(reg) == float(mag)
    # weights: metadata bit 1 = sign, bit 0 = selector (sv0 here)
    assert oracle.candidate(W, float(mag), 8.0, 0b10) == float(signed)
    assert oracle.element_value(W, float(mag), 8.0, 8, 0b10) == float(signed)
    assert oracle.element_value(A, float(mag), 0.0, 8, 0b1) == float(signed)
    lo, hi, step = (float(v) for v in rows[1])
    offs = sorted({oracle.sv_from_offset_reg(r) - 6.0 for r in range(16)})
    assert offs[0] == lo and offs[-1] == hi
    assert all(abs((b - a) - step) < 1e-12 for a, b in zip(offs, offs[1:]))
    assert oracle.offset_reg_from_sv(float(mag)) == reg
    # magnitudes that are FP4 values, off-grid or out of range are rejected
    for bad in (6.0, 4.0, 3.0, 5.25, 10.0, 2.0):
        assert oracle.offset_reg_from_sv(bad) == -1


def test_paper_special_value_sets_are_encodable(oracle):
    for _model, sv0, sv1 in golden_rows("weight_special_values.txt"):
        assert oracle.offset_reg_from_sv(float(sv0)) >= 0
        assert oracle.offset_reg_from_sv(float(sv1)) >= 0


def test_candidate_order_and_metadata_bits(oracle):
    assert [oracle.candidate(W, 5.0, 8.0, m) for m in range(4)] == [5.0, 8.0, -5.0, -8.0]
    assert [oracle.candidate(A, 5.0, 0.0, m) for m in range(2)] == [5.0, -5.0]
    for code in range(16):
        if code != 8:
            for m in range(4):
                assert oracle.element_value(W, 5.0, 8.0, code, m) == oracle.fp4_value(code)


def test_two_pass_identity(oracle):
    """App. D.3: decoding B_main and B_comp as plain FP4 and adding them gives
    the RaZeR value for every code and every metadata value."""
    mags = [float(v) for v in golden_rows("fp4_e2m1_values.txt")[0]]
    ex = golden_rows("two_pass_example.txt")
    sv = [float(r[0]) for r in ex]
    main = {float(r[1]) for r in ex}
    assert len(main) == 1
    main_code = mags.index(main.pop())
    comp_codes = [mags.index(float(r[2])) for r in ex]
    for code, meta in itertools.product(range(16), range(4)):
        bm, bc = oracle.two_pass_split(code, meta, main_code, comp_codes)
        plain = oracle.fp4_value(bm) + oracle.fp4_value(bc)
        assert plain == oracle.element_value(W, sv[0], sv[1], code, meta)
        if code != 8:
            assert bm == code and oracle.fp4_value(bc) == 0.0


def test_two_pass_reachable_set(oracle):
    want = sorted(float(v) for v in golden_rows("two_pass_reachable_set.txt")[0])
    base = {oracle.fp4_value(c) for c in range(8)}
    sums = {a + b for a in base for b in base} - base
    assert sorted(sums) == want


def test_f64_to_bf16_matches_library(oracle):
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(3000).astype(np.float32),
                        (rng.standard_normal(500) * 1e-39).astype(np.float32),   # subnormal range
                        (rng.standard_normal(500) * 1e30).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, -3.4e38,
                                  np.inf, -np.inf], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f64_to_bf16(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, ref)
    # a double strictly between an fp32 tie and its neighbour must not double-round
    assert oracle.f64_to_bf16(1.00390625 + 1e-12) == 0x3F81
    assert oracle.f64_to_bf16(1.00390625) == 0x3F80
