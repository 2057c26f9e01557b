"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.
Codes, scale bytes, tensor scales and decoded values must match bit for bit;
bf16 linear outputs within 8e-3 max relative error."""
import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err, tensor_to_host

pytestmark = pytest.mark.gpu
W, A = 0, 1


def _rand_tensor(rng, fmt, rows, cols):
    codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(rows, cols // 16), dtype=np.uint8)
    if fmt == A:
        scales[(scales & 127) == 127] = 126                       # the NaN code is never written
    return codes, scales, np.float32(rng.uniform(1e-4, 1e-2))


# ------------------------------------------------------------------ dequant
@pytest.mark.parametrize("fmt,sv", [(W, (5.0, 8.0)), (W, (4.5, 9.0)), (A, (5.0, 0.0))])
@pytest.mark.parametrize("rows,cols", [(1, 32), (37, 1056), (256, 4096)])
def test_dequant_bit_exact(oracle, fmt, sv, rows, cols):
    print("dequant", fmt, sv, rows, cols, flush=True)
    rng = np.random.default_rng(100 + rows)
    codes, scales, ts = _rand_tensor(rng, fmt, rows, cols)
    ref = oracle.dequant(fmt, codes, scales, ts, sv=sv, want=("f32", "bf16"))
    t = razer.RazerTensor.from_host(codes, scales, ts, fmt, sv)
    out32 = razer.razer_dequant(t, torch.float32).cpu().numpy()
    assert np.array_equal(out32.view(np.uint32), ref["f32"].view(np.uint32))
    out16 = dev_to_bf16_bits(razer.razer_dequant(t, torch.bfloat16))
    assert np.array_equal(out16, ref["bf16"])


def test_dequant_strided_output_and_empty(oracle):
    rng = np.random.default_rng(7)
    codes, scales, ts = _rand_tensor(rng, W, 9, 64)
    t = razer.RazerTensor.from_host(codes, scales, ts, W, (5.0, 8.0))
    buf = torch.full((9, 96), 7.0, dtype=torch.float32, device="cuda")
    razer.razer_dequant(t, out=buf[:, :64])
    ref = oracle.dequant(W, codes, scales, ts)["f32"]
    assert np.array_equal(buf[:, :64].cpu().numpy(), ref)
    assert torch.all(buf[:, 64:] == 7.0)
    empty = razer.RazerTensor.from_host(codes[:0], scales[:0], ts, W, (5.0, 8.0))
    assert razer.razer_dequant(empty).shape == (0, 64)


# ------------------------------------------------------------------ quantize
def _check_quantize(oracle, x_host, fmt, sv, x_dev=None, given=None):
    if x_dev is None:
        x_dev = bf16_bits_to_dev(x_host) if x_host.dtype == np.uint16 else torch.from_numpy(x_host).cuda()
    ts_dev = None if given is None else torch.tensor([given], dtype=torch.float32, device="cuda")
    t = razer.razer_quantize(x_dev, fmt, sv, tensor_scale=ts_dev)
    torch.cuda.synchronize()
    codes, scales, ts = tensor_to_host(t)
    rc, rs, rts = oracle.quantize(fmt, x_host, sv=sv, given_tensor_scale=given)
    assert np.float32(ts).view(np.uint32) == np.float32(rts).view(np.uint32)
    bad = np.argwhere(scales != rs)
    assert bad.size == 0, ("scale bytes differ", bad[:5], scales[tuple(bad[0])], rs[tuple(bad[0])])
    bad = np.argwhere(codes != rc)
    assert bad.size == 0, ("codes differ", bad[:5])
    return t, (rc, rs, rts)


@pytest.mark.parametrize("rows,cols", [(1, 32), (3, 96), (67, 1056), (128, 4096)])
def test_quantize_weights_bit_exact(oracle, rows, cols):
    print("quantize W", rows, cols, flush=True)
    w = synth.weight(rows, cols, seed=200 + rows, outlier_frac=0.002 if cols >= 1024 else 0.0)
    _check_quantize(oracle, w, W, (5.0, 8.0))
    _check_quantize(oracle, w, W, (5.0, 7.0))


@pytest.mark.parametrize("rows,cols", [(1, 32), (5, 160), (130, 2048)])
def test_quantize_activations_bit_exact(oracle, rows, cols):
    print("quantize A", rows, cols, flush=True)
    a = synth.activation(rows, cols, seed=300 + rows, outlier_frac=0.005 if cols >= 1024 else 0.0)
    _check_quantize(oracle, a, A, (5.0, 0.0))
    # fp32 input in the activation format and bf16 input in the weight format
    _check_quantize(oracle, synth.bf16_bits_to_f32(a) * np.float32(1.37), A, (5.0, 0.0))
    _check_quantize(oracle, a, W, (5.0, 8.0))


def test_quantize_wide_dynamic_range_hits_subnormal_and_zero_scales(oracle):
    """A few huge outliers push most blocks onto the smallest scales, where the second
    special-value pair becomes reachable and some blocks decode to zero."""
    w = synth.weight(64, 2048, seed=17)
    w[3, 100] = 40.0
    w[10, 7] = -55.0
    rng = np.random.default_rng(4)
    w *= np.exp(rng.uniform(-4, 2, size=(64, 1))).astype(np.float32)     # per-row magnitude spread
    t, (rc, rs, _) = _check_quantize(oracle, w, W, (5.0, 8.0))
    assert (rs & 63 == 0).any() and ((rs & 63) < 8).any()
    assert ((rs >> 6) & 1).any()                                          # +-8 chosen somewhere
    a = synth.bf16_bits_to_f32(synth.activation(32, 1024, seed=18)) * np.float32(1e-3)
    a[0, 0] = 3000.0
    _check_quantize(oracle, a.astype(np.float32), A, (5.0, 0.0))


def test_quantize_edge_cases(oracle):
    z = np.zeros((4, 64), np.float32)
    t, _ = _check_quantize(oracle, z, W, (5.0, 8.0))
    assert float(t.tensor_scale.cpu()[0]) == 1.0
    w = synth.weight(16, 256, seed=5)
    _check_quantize(oracle, w, W, (5.0, 8.0), given=float(np.float32(2.0 ** -12)))
    _check_quantize(oracle, w, W, (5.0, 8.0), given=1e-5)                 # saturating block scales
    # exact ties of the element rounding and of the special-value choice
    ties = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 4.5, 5.5, -4.5, -5.5, -5.0, 6.0, -0.25, 0.0, -0.0],
                    np.float32)
    x = np.tile(ties, (2, 2)).astype(np.float32)
    _check_quantize(oracle, x, W, (5.0, 8.0), given=1.0)
    _check_quantize(oracle, x, A, (5.0, 0.0), given=1.0)
    # leading dimension larger than cols
    big = torch.from_numpy(synth.weight(8, 192, seed=6)).cuda()
    t = razer.razer_quantize(big, W, (5.0, 8.0), cols=128)
    rc, rs, rts = oracle.quantize(W, np.ascontiguousarray(big.cpu().numpy()[:, :128]))
    codes, scales, ts = tensor_to_host(t)
    assert np.array_equal(codes, rc) and np.array_equal(scales, rs) and ts == rts
    # empty tensor
    e = razer.razer_quantize(torch.empty((0, 64), dtype=torch.float32, device="cuda"))
    assert e.codes.numel() == 0 and float(e.tensor_scale.cpu()[0]) == 1.0


def test_quantize_then_dequant_round_trip_on_device(oracle):
    w = synth.weight(40, 512, seed=8)
    t, (rc, rs, rts) = _check_quantize(oracle, w, W, (5.0, 8.0))
    out = razer.razer_dequant(t).cpu().numpy()
    assert np.array_equal(out, oracle.dequant(W, rc, rs, rts)["f32"])


# ------------------------------------------------------------------ linear
def _linear_case(oracle, m, n, k, seed, w_out=0.002):
    w = synth.weight(n, k, seed=seed, outlier_frac=w_out if k >= 1024 else 0.0)
    a = synth.activation(m, k, seed=seed + 1)
    wq = oracle.quantize(W, w)
    y64, _ = oracle.linear(wq, a_bf16=a)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    return max_rel_err(dev_to_bf16_bits(y), y64)


@pytest.mark.parametrize("m", [1, 2, 3, 4])
@pytest.mark.parametrize("n,k", [(1, 32), (7, 96), (130, 2048), (66, 4096 + 160), (33, 11008), (20, 28672),
                                 (12, 2048 * 17 + 64)])
def test_linear_gemv_matches_oracle(oracle, m, n, k):
    print("gemv", m, n, k, flush=True)
    err = _linear_case(oracle, m, n, k, seed=400 + m + n)
    assert err <= TOL, err


@pytest.mark.parametrize("m,n,k", [(3, 16400, 544), (4, 16389, 8192 + 512), (4, 16384, 2048)])
def test_linear_gemv_many_rows_matches_oracle(oracle, m, n, k):
    """3-4 activation rows against at least 16384 weight rows: the matrix-instruction GEMV with 8
    groups of rows per workgroup (one and two 512-element runs per lane), ragged last workgroup."""
    print("gemv many rows", m, n, k, flush=True)
    rng = np.random.default_rng(450 + m + k)
    wq = _rand_tensor(rng, W, n, k)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    a = synth.activation(m, k, seed=451 + m)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    y64, _ = oracle.linear(wq, a_bf16=a)
    assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL


@pytest.mark.parametrize("m,n,k", [(5, 40, 64), (8, 300, 1056), (16, 256, 2048), (33, 100, 96), (64, 513, 1024),
                                   (17, 70, 32), (32, 129, 4096 + 32), (12, 65, 8192 + 512), (31, 64, 544),
                                   (100, 130, 4096), (129, 384, 512), (300, 260, 1120), (512, 512, 1024),
                                   (257, 257, 224)])
def test_linear_gemm_matches_oracle(oracle, m, n, k):
    print("gemm", m, n, k, flush=True)
    err = _linear_case(oracle, m, n, k, seed=500 + m)
    assert err <= TOL, err


@pytest.mark.parametrize("m,n,k", [(33, 100, 96), (48, 130, 1024), (64, 513, 4096 + 32), (64, 64, 11008), (65, 100, 544),
                                   (96, 260, 2048), (128, 513, 4096 + 32), (128, 32, 11008), (100, 1, 4096),
                                   (128, 300, 64), (40, 70, 32)])
def test_linear_mid_batch_matches_oracle(oracle, m, n, k):
    """33..128 activation rows: the register-decode kernel with 64- and 128-row tiles; one to sixteen
    K-slices (the slices meet in the workspace), ragged last K-tile, ragged rows on both sides."""
    print("gemm mid batch", m, n, k, flush=True)
    err = _linear_case(oracle, m, n, k, seed=900 + m)
    assert err <= TOL, err


def test_linear_mid_batch_random_codes_all_scale_bytes(oracle):
    rng = np.random.default_rng(78)
    n, k = 200, 2048
    codes, scales, ts = _rand_tensor(rng, W, n, k)
    for m in (40, 128):
        a = synth.activation(m, k, seed=70 + m)
        y64, _ = oracle.linear((codes, scales, ts), a_bf16=a, w_sv=(5.0, 7.0))
        wt = razer.RazerTensor.from_host(codes, scales, ts, W, (5.0, 7.0))
        assert max_rel_err(dev_to_bf16_bits(razer.razer_linear(wt, bf16_bits_to_dev(a))), y64) <= TOL


def test_linear_shapes_around_every_dispatch_boundary(oracle):
    """Seeded random (n, k) at every activation-row count where the dispatch changes kernels (4|5, 32|33,
    64|65, 128|129, 256|257) plus a few in between; single calls and grouped calls on the same operands."""
    rng = np.random.default_rng(4242)
    ms = [1, 4, 5, 17, 32, 33, 64, 65, 100, 128, 129, 200, 256, 257, 300]
    for i, m in enumerate(ms):
        for rep in range(2):
            n = int(rng.integers(1, 160)) * int(rng.choice([1, 1, 4]))
            k = 32 * int(rng.integers(1, 70)) if rep == 0 else 32 * int(rng.integers(64, 200))
            print("boundary shapes", m, n, k, flush=True)
            codes, scales, ts = _rand_tensor(rng, W, n, k)
            scales = (scales & 0xC0) | (16 + (scales & 15))        # moderate scales: well-conditioned sums
            a = synth.activation(m, k, seed=5000 + 2 * i + rep)
            a_dev = bf16_bits_to_dev(a)
            y64, _ = oracle.linear((codes, scales, ts), a_bf16=a)
            wt = razer.RazerTensor.from_host(codes, scales, ts, W, (5.0, 8.0))
            y = razer.razer_linear(wt, a_dev)
            torch.cuda.synchronize()
            assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL, (m, n, k)
            # the same matrix twice and a second one in a grouped call
            n2 = int(rng.integers(1, 100)) * 4
            c2, s2, t2 = _rand_tensor(rng, W, n2, k)
            s2 = (s2 & 0xC0) | (16 + (s2 & 15))
            wt2 = razer.RazerTensor.from_host(c2, s2, t2, W, (5.0, 8.0))
            ys = razer.razer_linear_grouped([wt, wt2, wt], a_dev)
            torch.cuda.synchronize()
            assert max_rel_err(dev_to_bf16_bits(ys[0]), y64) <= TOL, ("grouped", m, n, k)
            assert torch.equal(ys[0], ys[2])
            assert max_rel_err(dev_to_bf16_bits(ys[1]), oracle.linear((c2, s2, t2), a_bf16=a)[0]) <= TOL, ("grouped 2", m, n2, k)


def test_linear_special_values_matter(oracle):
    """Decoding the remapped code as a plain zero must show up as an error: guards
    against a kernel that silently drops the special values."""
    n, k, m = 64, 1024, 3
    w = synth.weight(n, k, seed=31)
    a = synth.activation(m, k, seed=32)
    wq = oracle.quantize(W, w)
    y64, _ = oracle.linear(wq, a_bf16=a)
    codes = wq[0]
    frac = np.mean(((codes & 15) == 8) | ((codes >> 4) == 8))
    assert frac > 0.01
    y_plain, _ = oracle.linear((wq[0], wq[1] & 63, wq[2]), a_bf16=a, w_sv=(5.0, 8.0))
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    yg = dev_to_bf16_bits(razer.razer_linear(wt, bf16_bits_to_dev(a)))
    assert max_rel_err(yg, y64) <= TOL
    assert max_rel_err(yg, y_plain) > 10 * TOL
    # other special-value sets, both kernels
    for sv in ((5.0, 7.0), (4.5, 9.0), (2.5, 9.5)):
        for mm in (2, 40):
            aa = synth.activation(mm, k, seed=33 + mm)
            wq2 = oracle.quantize(W, w, sv=sv)
            y2, _ = oracle.linear(wq2, a_bf16=aa, w_sv=sv)
            wt2 = razer.RazerTensor.from_host(*wq2, W, sv)
            assert max_rel_err(dev_to_bf16_bits(razer.razer_linear(wt2, bf16_bits_to_dev(aa))), y2) <= TOL


def test_linear_random_codes_all_scale_bytes(oracle):
    """Arbitrary code / scale bytes (not produced by the encoder) decode identically in the
    fused kernels: every scale code, every metadata value, every nibble."""
    rng = np.random.default_rng(77)
    n, k = 96, 1024
    codes, scales, ts = _rand_tensor(rng, W, n, k)
    for m in (1, 4, 24):
        a = synth.activation(m, k, seed=60 + m)
        y64, _ = oracle.linear((codes, scales, ts), a_bf16=a)
        wt = razer.RazerTensor.from_host(codes, scales, ts, W, (5.0, 8.0))
        assert max_rel_err(dev_to_bf16_bits(razer.razer_linear(wt, bf16_bits_to_dev(a))), y64) <= TOL


def _w4a4_both_forms(wt, at, m):
    """razer_linear with a RaZeR activation operand in its two forms: with the workspace the W4A4 query asks for
    (activations decoded once, then the weight-only path) and with the plain linear figure (one fused kernel)."""
    from paper_2501_04052_amd import binding
    need = max(256, razer.razer_workspace_bytes(binding.OP_LINEAR, wt.rows, wt.cols, m))
    fused_ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert need < razer.razer_workspace_bytes(binding.OP_LINEAR_W4A4, wt.rows, wt.cols, m)
    ys = [razer.razer_linear(wt, at), razer.razer_linear(wt, at, workspace=fused_ws)]
    torch.cuda.synchronize()
    return ys



@pytest.mark.parametrize("m,n,k", [(4, 64, 256), (130, 260, 512), (257, 128, 1056)])
def test_linear_w4a4_matches_oracle(oracle, m, n, k):
    print("w4a4", m, n, k, flush=True)
    w = synth.weight(n, k, seed=600 + m, outlier_frac=0.002 if k >= 1024 else 0.0)
    a = synth.activation(m, k, seed=601 + m, outlier_frac=0.005)
    wq = oracle.quantize(W, w)
    aq = oracle.quantize(A, a, sv=(5.0, 0.0))
    y64, _ = oracle.linear(wq, a_q=aq)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    at = razer.razer_quantize(bf16_bits_to_dev(a), A, (5.0, 0.0))       # on-the-fly activation encode
    ac, asc, ats = tensor_to_host(at)
    assert np.array_equal(ac, aq[0]) and np.array_equal(asc, aq[1]) and ats == aq[2]
    for y in _w4a4_both_forms(wt, at, m):
        assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL


def test_linear_w4a4_shapes_around_every_dispatch_boundary(oracle):
    """W4A4 (both operands decoded): seeded random (n, k) at the activation-row counts where the tile
    shape changes (32|33, 64|65, 128|129, 256|257), with and without K-slices."""
    rng = np.random.default_rng(4343)
    for i, m in enumerate([1, 5, 32, 33, 64, 65, 128, 129, 256, 257]):
        n = int(rng.integers(1, 300))
        k = 32 * int(rng.integers(1, 40)) if i % 2 == 0 else 32 * int(rng.integers(100, 180))
        print("w4a4 boundary shapes", m, n, k, flush=True)
        wc, ws, wts = _rand_tensor(rng, W, n, k)
        ws = (ws & 0xC0) | (16 + (ws & 15))
        ac, asc, ats = _rand_tensor(rng, A, m, k)
        asc = (asc & 0x80) | (48 + (asc & 15))                      # E4M3 codes 48..63: values 0.5..1.875
        y64, _ = oracle.linear((wc, ws, wts), a_q=(ac, asc, ats))
        wt = razer.RazerTensor.from_host(wc, ws, wts, W, (5.0, 8.0))
        at = razer.RazerTensor.from_host(ac, asc, ats, A, (5.0, 0.0))
        for y in _w4a4_both_forms(wt, at, m):
            assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL, (m, n, k)


def test_linear_strided_output_and_empty(oracle):
    n, k = 40, 256
    w = synth.weight(n, k, seed=70)
    wq = oracle.quantize(W, w)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    for m in (2, 20):
        a = synth.activation(m, k, seed=71 + m)
        y64, _ = oracle.linear(wq, a_bf16=a)
        buf = torch.full((m, 64), 3.0, dtype=torch.bfloat16, device="cuda")
        razer.razer_linear(wt, bf16_bits_to_dev(a), out=buf[:, :n])
        assert max_rel_err(dev_to_bf16_bits(buf[:, :n]), y64) <= TOL
        assert torch.all(buf[:, n:] == 3.0)
    y = razer.razer_linear(wt, torch.empty((0, k), dtype=torch.bfloat16, device="cuda"))
    assert y.shape == (0, n)


@pytest.mark.parametrize("m,k", [(1, 2048 + 96), (2, 2048 + 96), (3, 2048 + 96), (4, 2048 + 96), (20, 2048 + 96),
                                 (1, 11008), (4, 11008), (1, 28672), (2, 2048 * 17 + 64)])
def test_linear_grouped_matches_oracle(oracle, m, k):
    """Several weight matrices on the same activation rows in one call (one launch for m <= 4); the
    K values cover the 2-group and 8-group streaming kernels and the multi-pass kernel for long rows."""
    print("grouped", m, k, flush=True)
    ns = [100, 64, 37, 9]
    a = synth.activation(m, k, seed=800 + m)
    a_dev = bf16_bits_to_dev(a)
    for count in (1, 2, 4):
        wqs = [oracle.quantize(W, synth.weight(n, k, seed=810 + i, outlier_frac=0.002)) for i, n in enumerate(ns[:count])]
        wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
        bufs = [torch.full((m, n + 8), 2.0, dtype=torch.bfloat16, device="cuda") for n in ns[:count]]
        razer.razer_linear_grouped(wts, a_dev, outs=[b[:, :n] for b, n in zip(bufs, ns)])
        torch.cuda.synchronize()
        for wq, b, n in zip(wqs, bufs, ns):
            y64, _ = oracle.linear(wq, a_bf16=a)
            assert max_rel_err(dev_to_bf16_bits(b[:, :n]), y64) <= TOL
            assert torch.all(b[:, n:] == 2.0)
    # different special values per matrix: falls back to one launch each, same results
    wq2 = oracle.quantize(W, synth.weight(50, k, seed=820), sv=(5.0, 7.0))
    wts = [razer.RazerTensor.from_host(*wqs[0], W, (5.0, 8.0)), razer.RazerTensor.from_host(*wq2, W, (5.0, 7.0))]
    ys = razer.razer_linear_grouped(wts, a_dev)
    assert max_rel_err(dev_to_bf16_bits(ys[1]), oracle.linear(wq2, a_bf16=a, w_sv=(5.0, 7.0))[0]) <= TOL
    assert max_rel_err(dev_to_bf16_bits(ys[0]), oracle.linear(wqs[0], a_bf16=a)[0]) <= TOL


@pytest.mark.parametrize("m,k,ns", [(5, 512 + 64, [132, 64, 200]), (16, 11008, [132, 64, 200]),
                                    (17, 1024, [132, 64, 200]), (32, 512 + 64, [132, 64, 200]),
                                    # enough workgroups that each walks through two 64-row blocks; 4100 rows
                                    # leave the last workgroup of the first matrix one ragged block
                                    (8, 8192, [4100, 4096])])
def test_linear_grouped_small_batch_one_launch(oracle, m, k, ns):
    """5 <= m <= 32: the matrices' K-slices share one workspace and one reduction launch."""
    print("grouped small batch", m, k, ns, flush=True)
    rng = np.random.default_rng(2000 + m)
    a = synth.activation(m, k, seed=2001 + m)
    a_dev = bf16_bits_to_dev(a)
    wqs = [_rand_tensor(rng, W, n, k) for n in ns]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    bufs = [torch.full((m, n + 4), 2.0, dtype=torch.bfloat16, device="cuda") for n in ns]
    # the large case: the K-sliced kernel with two 64-row blocks per workgroup, for the group and for the single
    # calls alike (left to itself the dispatch picks a launch shape per problem size, and with it a summation order)
    from paper_2501_04052_amd import binding
    if max(ns) > 1000:
        razer.razer_tune_force(binding.TUNE_SMALL_BATCH, (0, 4, 2))
    try:
        razer.razer_linear_grouped(wts, a_dev, outs=[b[:, :n] for b, n in zip(bufs, ns)])
        torch.cuda.synchronize()
        for wt, wq, b, n in zip(wts, wqs, bufs, ns):
            y64, _ = oracle.linear(wq, a_bf16=a)
            assert max_rel_err(dev_to_bf16_bits(b[:, :n]), y64) <= TOL
            assert torch.all(b[:, n:] == 2.0)
            # the same kernels, one matrix per call: identical bits (same slices, same order)
            assert torch.equal(b[:, :n], razer.razer_linear(wt, a_dev))
    finally:
        razer.razer_tune_force(binding.TUNE_SMALL_BATCH, None)


@pytest.mark.parametrize("m,ns,k", [(2000, [2760, 2688, 2944], 160), (2000, [8200, 8192, 8192, 8448], 64),
                                    (300, [4100, 4096, 4200], 1088)])
def test_linear_grouped_gemm_one_launch(oracle, m, ns, k):
    """m > 32 with enough output tiles over all matrices: one launch of the register-decode GEMM
    (128-wide weight tiles in the first case, 256-wide in the second, one round of 128-wide tiles
    with K halved inside the workgroup in the third); ragged m, n and K-tile."""
    print("grouped gemm", m, ns, k, flush=True)
    rng = np.random.default_rng(2100 + k)
    a = synth.activation(m, k, seed=2101 + k)
    a_dev = bf16_bits_to_dev(a)
    wqs = [_rand_tensor(rng, W, n, k) for n in ns]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    bufs = [torch.full((m, n + 8), 2.0, dtype=torch.bfloat16, device="cuda") for n in ns]
    razer.razer_linear_grouped(wts, a_dev, outs=[b[:, :n] for b, n in zip(bufs, ns)])
    torch.cuda.synchronize()
    for wq, b, n in zip(wqs, bufs, ns):
        y64, _ = oracle.linear(wq, a_bf16=a)
        assert max_rel_err(dev_to_bf16_bits(b[:, :n]), y64) <= TOL
        assert torch.all(b[:, n:] == 2.0)


@pytest.mark.parametrize("m,k,ns", [(33, 512 + 64, [132, 64, 200]), (64, 4096, [132, 64, 200]), (100, 11008, [132, 64]),
                                    (128, 2048 + 32, [132, 64, 200, 4]), (48, 1024, [130, 61])])
def test_linear_grouped_mid_batch_one_launch(oracle, m, k, ns):
    """33 <= m <= 128: one launch of the register-decode GEMM over all matrices, K-slices of all of
    them in one workspace and one reduction launch (one slice in the first case, eight and more in the
    others); the last case (row counts that are not multiples of 4) runs matrix by matrix."""
    print("grouped mid batch", m, k, ns, flush=True)
    rng = np.random.default_rng(2200 + m)
    a = synth.activation(m, k, seed=2201 + m)
    a_dev = bf16_bits_to_dev(a)
    wqs = [_rand_tensor(rng, W, n, k) for n in ns]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    bufs = [torch.full((m, n + (8 if n % 4 == 0 else 3)), 2.0, dtype=torch.bfloat16, device="cuda") for n in ns]
    razer.razer_linear_grouped(wts, a_dev, outs=[b[:, :n] for b, n in zip(bufs, ns)])
    torch.cuda.synchronize()
    for wq, b, n in zip(wqs, bufs, ns):
        y64, _ = oracle.linear(wq, a_bf16=a)
        assert max_rel_err(dev_to_bf16_bits(b[:, :n]), y64) <= TOL
        assert torch.all(b[:, n:] == 2.0)


# ------------------------------------------------------------------ block sizes 32, 64, 128 (Sec. 5.4)
BLOCKS = [32, 64, 128]


def _rand_tensor_b(rng, fmt, rows, cols, block):
    codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(rows, cols // block), dtype=np.uint8)
    if fmt == A:
        scales[(scales & 127) == 127] = 126
    return codes, scales, np.float32(rng.uniform(1e-4, 1e-2))


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("fmt,sv", [(W, (5.0, 8.0)), (A, (5.0, 0.0))])
def test_block_sizes_quantize_and_dequant_bit_exact(oracle, block, fmt, sv):
    print("block encode/decode", block, fmt, flush=True)
    for rows, cols, seed in ((37, 3 * 128, 1), (5, 128, 2), (130, 1024 + 128, 3)):
        if fmt == W:
            x = synth.weight(rows, cols, seed=900 + seed + block, outlier_frac=0.01)
            x[0, :block] = 0.0                                          # an all-zero block
            x[1, block:2 * block] *= np.float32(1e-4)                   # a block whose scale rounds to 0
        else:
            x = synth.activation(rows, cols, seed=901 + seed + block, outlier_frac=0.01)
        x_dev = bf16_bits_to_dev(x) if x.dtype == np.uint16 else torch.from_numpy(x).cuda()
        t = razer.razer_quantize(x_dev, fmt, sv, block=block)
        torch.cuda.synchronize()
        codes, scales, ts = tensor_to_host(t)
        rc, rs, rts = oracle.quantize(fmt, x, sv=sv, block=block)
        assert np.float32(ts).view(np.uint32) == np.float32(rts).view(np.uint32)
        assert scales.shape == rs.shape and np.array_equal(scales, rs), "scale bytes differ"
        assert np.array_equal(codes, rc), "codes differ"
        ref = oracle.dequant(fmt, rc, rs, rts, sv=sv, want=("f32", "bf16"))
        assert np.array_equal(razer.razer_dequant(t, torch.float32).cpu().numpy().view(np.uint32), ref["f32"].view(np.uint32))
        assert np.array_equal(dev_to_bf16_bits(razer.razer_dequant(t, torch.bfloat16)), ref["bf16"])
    # random scale bytes (every code, every metadata value) through the decoder
    rng = np.random.default_rng(77 + block)
    codes, scales, ts = _rand_tensor_b(rng, fmt, 19, 512, block)
    t = razer.RazerTensor.from_host(codes, scales, ts, fmt, sv)
    assert t.block == block
    ref = oracle.dequant(fmt, codes, scales, ts, sv=sv, want=("f32",))["f32"]
    assert np.array_equal(razer.razer_dequant(t, torch.float32).cpu().numpy().view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("m,n,k", [(1, 130, 2048 + 256), (3, 66, 11008), (4, 20, 28672),
                                   (2, 12, 2048 * 17 + 128), (8, 300, 1024 + 128), (20, 70, 8192 + 512),
                                   (40, 100, 256), (200, 260, 1152), (300, 513, 1024), (64, 257, 128)])
def test_block_sizes_linear_matches_oracle(oracle, block, m, n, k):
    """Every kernel family (GEMV streaming / multi-pass, small batch, tiled GEMM) with 32-, 64- and
    128-element blocks, random codes and scale bytes."""
    print("block linear", block, m, n, k, flush=True)
    rng = np.random.default_rng(1200 + block + m + n)
    wq = _rand_tensor_b(rng, W, n, k, block)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    a = synth.activation(m, k, seed=1300 + m, outlier_frac=0.005)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    y64, _ = oracle.linear(wq, a_bf16=a)
    assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL


@pytest.mark.parametrize("wb,ab", [(32, 16), (16, 64), (64, 64), (128, 32)])
@pytest.mark.parametrize("m,n,k", [(3, 40, 256), (100, 130, 1152), (300, 260, 512)])
def test_block_sizes_w4a4_matches_oracle(oracle, wb, ab, m, n, k):
    print("block w4a4", wb, ab, m, n, k, flush=True)
    wq = oracle.quantize(W, synth.weight(n, k, seed=1400 + wb, outlier_frac=0.01), block=wb)
    a_bits = synth.activation(m, k, seed=1401 + ab, outlier_frac=0.01)
    at = razer.razer_quantize(bf16_bits_to_dev(a_bits), A, (5.0, 0.0), block=ab)
    aq = tensor_to_host(at)
    ra = oracle.quantize(A, a_bits, sv=(5.0, 0.0), block=ab)
    assert np.array_equal(aq[0], ra[0]) and np.array_equal(aq[1], ra[1])
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    y64, _ = oracle.linear(wq, a_q=ra)
    for y in _w4a4_both_forms(wt, at, m):
        assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL


@pytest.mark.parametrize("block", [32, 64, 128])
@pytest.mark.parametrize("m,k,ns", [(1, 512, (33, 50)), (2, 4096, (40, 9, 64)), (1, 11008, (70, 35)), (4, 8192, (24, 24, 24, 5)),
                                    (3, 34816, (10, 7))])
def test_block_sizes_grouped_small_batch_one_launch(oracle, block, m, k, ns):
    """m <= 4: matrices of one block size share a launch (one, two and many K-slices per row, a ragged
    last slice, rows longer than a workgroup covers in one pass)."""
    print("block grouped", block, m, k, ns, flush=True)
    a = synth.activation(m, k, seed=1500 + m)
    wqs = [oracle.quantize(W, synth.weight(n, k, seed=1501 + n + i), block=block) for i, n in enumerate(ns)]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    for wq, wt, y in zip(wqs, wts, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL
        # and bit for bit what the single-matrix call gives
        assert torch.equal(y, razer.razer_linear(wt, bf16_bits_to_dev(a)))


@pytest.mark.parametrize("block", [32, 64, 128])
@pytest.mark.parametrize("m,k,ns", [(8, 1024, (132, 64, 200)), (32, 4096 + 128, (64, 260)), (16, 11008, (132, 64)),
                                    (64, 4096, (132, 64, 200)), (100, 2048 + 128, (132, 64)), (300, 1152, (4100, 4096, 4200))])
def test_block_sizes_grouped_larger_batches_one_launch(oracle, block, m, k, ns):
    """5 <= m: the grouped small-batch kernel and the grouped register-decode GEMM (with and without
    K-slices, two-K-group round) take 32-, 64- and 128-element blocks as well."""
    print("block grouped batch", block, m, k, ns, flush=True)
    rng = np.random.default_rng(1700 + block + m)
    a = synth.activation(m, k, seed=1701 + m)
    a_dev = bf16_bits_to_dev(a)
    wqs = [_rand_tensor_b(rng, W, n, k, block) for n in ns]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, a_dev)
    torch.cuda.synchronize()
    if m * max(ns) * k > 3e9:                                       # large case: sampled outputs
        rows = np.unique(np.concatenate([synth.sample_indices(m, 24, 9700), [0, m - 1]]))
        for wq, y, n in zip(wqs, ys, ns):
            cols = np.unique(np.concatenate([synth.sample_indices(n, 96, 9701), [0, n - 1]]))
            y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
            got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
            assert max_rel_err(got, y64) <= TOL
    else:
        for wq, y in zip(wqs, ys):
            assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL


def test_block_sizes_grouped_mixed_geometry_is_a_sequence(oracle):
    k = 512
    a = synth.activation(2, k, seed=1520)
    wqs = [oracle.quantize(W, synth.weight(n, k, seed=1521 + n), block=b) for n, b in ((33, 64), (50, 16), (20, 128))]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
    for wq, y in zip(wqs, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL
    # larger batches of a block size other than 16 run matrix by matrix
    a = synth.activation(40, k, seed=1530)
    wqs = [oracle.quantize(W, synth.weight(n, k, seed=1531 + n), block=32) for n in (36, 64)]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
    for wq, y in zip(wqs, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL


def test_special_value_sweep_tool_agrees_with_oracle(oracle):
    """The selection tool (error of every allowed pair through the HIP encoder + decoder) ranks the
    pairs like the oracle does and picks +-5 first."""
    from paper_2501_04052_amd import sv_sweep
    w = synth.weight(64, 1024, seed=1600, outlier_frac=0.002)
    x = torch.from_numpy(w).cuda()
    (v0, v1), one, two = sv_sweep.best_pairs(x)
    assert v0 == 5.0 and v1 != 5.0
    for v in (4.5, 5.0, 7.0):
        c, s, t = oracle.quantize(W, w, sv=(v, v))
        d = oracle.dequant(W, c, s, t, sv=(v, v))["f32"].astype(np.float64)
        ref = float(((w - d) ** 2).sum())
        got = sv_sweep.quantization_error(x, W, (v, v))
        assert abs(got - ref) <= 1e-9 * ref


# ------------------------------------------------------------------ streams, graphs, determinism
def test_linear_on_side_stream_and_under_graph_replay(oracle):
    """Every kernel family on a non-default stream, captured into a HIP graph and replayed with the
    program's own eager work in between: each replay must equal the eager result bit for bit."""
    rng = np.random.default_rng(1700)
    k = 2048 + 64
    wq = _rand_tensor(rng, W, 300, k)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    side = torch.cuda.Stream()
    for m in (1, 4, 12, 40, 300):                     # GEMV, small batch (workspace), GEMM, split-K GEMM
        a_dev = bf16_bits_to_dev(synth.activation(m, k, seed=1701 + m))
        out = torch.empty((m, 300), dtype=torch.bfloat16, device="cuda")
        need = razer.razer_workspace_bytes(razer.binding.OP_LINEAR, 300, k, m)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        eager = razer.razer_linear(wt, a_dev, workspace=ws).clone()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            razer.razer_linear(wt, a_dev, out=out, workspace=ws)          # warm-up on the side stream
            side.synchronize()
            assert torch.equal(out, eager)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                razer.razer_linear(wt, a_dev, out=out, workspace=ws)
        torch.cuda.synchronize()
        for rep in range(3):
            out.fill_(float(rep))                                         # eager work between replays
            ws.random_(0, 255)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), (m, rep)
    y64, _ = oracle.linear(wq, a_bf16=synth.activation(300, k, seed=1701 + 300))
    assert max_rel_err(dev_to_bf16_bits(eager), y64) <= TOL


def test_grouped_linear_under_graph_replay(oracle):
    """The grouped launches (grouped GEMV, matrix-instruction GEMV, grouped small-batch kernel with
    its grouped reduction through the prepared-call path) captured into a HIP graph: every replay,
    with eager work in between, equals the eager result bit for bit."""
    rng = np.random.default_rng(1750)
    k = 1024 + 64
    ns = [132, 64, 200]
    wqs = [_rand_tensor(rng, W, n, k) for n in ns]
    wts = [razer.RazerTensor.from_host(*wq, W, (5.0, 8.0)) for wq in wqs]
    side = torch.cuda.Stream()
    for m in (1, 4, 12):
        a = synth.activation(m, k, seed=1751 + m)
        a_dev = bf16_bits_to_dev(a)
        eager = [y.clone() for y in razer.razer_linear_grouped(wts, a_dev)]
        outs = [torch.empty((m, n), dtype=torch.bfloat16, device="cuda") for n in ns]
        call = razer.prepare_linear_grouped(wts, a_dev, outs)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            call(side.cuda_stream)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                call(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            for o in outs:
                o.fill_(float(rep))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for o, e in zip(outs, eager):
                assert torch.equal(o, e), (m, rep)
        for wq, e in zip(wqs, eager):
            assert max_rel_err(dev_to_bf16_bits(e), oracle.linear(wq, a_bf16=a)[0]) <= TOL


def test_linear_is_deterministic(oracle):
    """The kernels that split K (small batch, GEMM with few tiles) add their slices in a fixed order."""
    rng = np.random.default_rng(1800)
    wq = _rand_tensor(rng, W, 200, 4096)
    wt = razer.RazerTensor.from_host(*wq, W, (5.0, 8.0))
    for m in (8, 100, 260):
        a_dev = bf16_bits_to_dev(synth.activation(m, 4096, seed=1801 + m))
        ref = razer.razer_linear(wt, a_dev)
        for _ in range(4):
            assert torch.equal(razer.razer_linear(wt, a_dev), ref)
