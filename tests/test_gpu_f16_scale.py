"""GPU parity for the format of the paper's own weight-only kernel (Sec. 4.3: blocks of 128, one
FP16 scale word with the metadata in its sign and top exponent bits): encoder and decoder bit-exact
against the oracle, the linear layer within the bf16 output tolerance."""
import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err, tensor_to_host

pytestmark = pytest.mark.gpu
F16 = razer.WEIGHT_F16


def _rand_tensor(rng, rows, cols):
    codes = rng.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)
    scales = rng.integers(0, 65536, size=(rows, cols // 128), dtype=np.uint16)     # every word is a valid scale
    return codes, scales, np.float32(rng.uniform(1e-4, 1e-2))


@pytest.mark.parametrize("sv", [(5.0, 8.0), (4.5, 9.0)])
@pytest.mark.parametrize("rows,cols,dtype", [(37, 3 * 128, "f32"), (5, 128, "f32"), (130, 1024 + 128, "f32"),
                                             (64, 4096, "f32"), (33, 512, "bf16")])
def test_quantize_and_dequant_bit_exact(oracle, sv, rows, cols, dtype):
    print("f16-scale encode/decode", sv, rows, cols, dtype, flush=True)
    if dtype == "f32":
        x = synth.weight(rows, cols, seed=3000 + rows + cols, outlier_frac=0.01)
        x[0, :128] = 0.0                                            # an all-zero block
        x[1, 128:256] *= np.float32(1e-9) if cols >= 256 else 1.0    # a block whose scale rounds to 0
        x_dev = torch.from_numpy(x).cuda()
    else:
        x = synth.activation(rows, cols, seed=3001 + rows, outlier_frac=0.01)
        x_dev = bf16_bits_to_dev(x)
    t = razer.razer_quantize(x_dev, F16, sv)
    torch.cuda.synchronize()
    assert t.block == 128 and t.scales.dtype == torch.int16
    codes, scales, ts = tensor_to_host(t)
    rc, rs, rts = oracle.quantize(F16, x, sv=sv)
    assert np.float32(ts).view(np.uint32) == np.float32(rts).view(np.uint32)
    assert scales.shape == rs.shape and np.array_equal(scales, rs), "scale words differ"
    assert np.array_equal(codes, rc), "codes differ"
    assert len(set((rs >> 14).ravel().tolist())) >= 2              # the special value is used
    ref = oracle.dequant(F16, rc, rs, rts, sv=sv, want=("f32", "bf16"))
    assert np.array_equal(razer.razer_dequant(t, torch.float32).cpu().numpy().view(np.uint32), ref["f32"].view(np.uint32))
    assert np.array_equal(dev_to_bf16_bits(razer.razer_dequant(t, torch.bfloat16)), ref["bf16"])


def test_given_tensor_scale_and_saturating_block_scale(oracle):
    """A static tensor scale that is too small makes Eq. 2 overflow the scale grid: it saturates at the
    largest code and the elements at +-6."""
    x = synth.weight(16, 512, seed=3100, outlier_frac=0.02)
    given = np.float32(np.abs(x).max() / 40.0)
    ts_dev = torch.tensor([float(given)], dtype=torch.float32, device="cuda")
    t = razer.razer_quantize(torch.from_numpy(x).cuda(), F16, (5.0, 8.0), tensor_scale=ts_dev)
    torch.cuda.synchronize()
    codes, scales, ts = tensor_to_host(t)
    rc, rs, rts = oracle.quantize(F16, x, given_tensor_scale=given)
    assert ts == given == rts
    assert np.array_equal(scales, rs) and np.array_equal(codes, rc)
    assert ((rs & 0x3FFF) == 0x3FFF).any()


def test_dequant_every_scale_word_field(oracle):
    rng = np.random.default_rng(3200)
    codes, scales, ts = _rand_tensor(rng, 64, 1024)
    scales[0, :4] = [0x0000, 0x3FFF, 0xFFFF, 0x8001]                 # zero scale, largest, all bits, smallest subnormal
    t = razer.RazerTensor.from_host(codes, scales, ts, F16, (5.0, 7.0))
    ref = oracle.dequant(F16, codes, scales, ts, sv=(5.0, 7.0), want=("f32", "bf16"))
    assert np.array_equal(razer.razer_dequant(t, torch.float32).cpu().numpy().view(np.uint32), ref["f32"].view(np.uint32))
    assert np.array_equal(dev_to_bf16_bits(razer.razer_dequant(t, torch.bfloat16)), ref["bf16"])


@pytest.mark.parametrize("m", [1, 2, 3, 4, 7, 20])
@pytest.mark.parametrize("n,k", [(100, 128), (37, 2048 + 128), (64, 11008), (9, 28672), (20, 2048 * 17 + 128)])
def test_linear_matches_oracle(oracle, m, n, k):
    """Every GEMV kernel family (2-group and 8-group streaming, multi-pass for long rows), ragged row
    counts, 1..20 activation rows (beyond 4 in passes)."""
    print("f16-scale linear", m, n, k, flush=True)
    rng = np.random.default_rng(3300 + m + n)
    wq = _rand_tensor(rng, n, k)
    wq[1][:] = (wq[1] & 0xC000) | (0x2C00 + (wq[1] & 0x0FFF))        # scales 2^-4 .. 2^-1: sums stay well conditioned
    wt = razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0))
    a = synth.activation(m, k, seed=3301 + m + k)
    buf = torch.full((m, n + 8), 2.0, dtype=torch.bfloat16, device="cuda")
    razer.razer_linear(wt, bf16_bits_to_dev(a), out=buf[:, :n])
    torch.cuda.synchronize()
    y64, _ = oracle.linear(wq, a_bf16=a)
    assert max_rel_err(dev_to_bf16_bits(buf[:, :n]), y64) <= TOL
    assert torch.all(buf[:, n:] == 2.0)


@pytest.mark.parametrize("m,n,k", [(5, 40, 128), (16, 300, 1024 + 128), (33, 257, 2048), (64, 100, 4096), (100, 640, 1152),
                                   (300, 200, 2048 + 384), (129, 8, 128 * 9), (48, 1000, 34944), (50, 72, 128), (64, 4104, 1152)])
def test_linear_matrix_core_path_matches_oracle(oracle, m, n, k):
    """From 5 activation rows up the format runs on the matrix cores with bare FP4 operands and a per-block
    fold in fp32 (up to 64 rows: the K-in-workgroup kernel with one, two or four 16-row fragments; beyond: tiled
    kernels with K-slices): ragged M and N, odd and even numbers of blocks, several passes per wave, every scale
    word field (zero, subnormal and saturated scales included)."""
    print("f16-scale matrix-core linear", m, n, k, flush=True)
    rng = np.random.default_rng(3700 + m + n)
    wq = _rand_tensor(rng, n, k)
    wq[1][0, 0] = 0x0000
    wq[1][-1, -1] = 0xFFFF
    wt = razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0))
    a = synth.activation(m, k, seed=3701 + m + k, outlier_frac=0.01)
    buf = torch.full((m, n + 8), 2.0, dtype=torch.bfloat16, device="cuda")
    razer.razer_linear(wt, bf16_bits_to_dev(a), out=buf[:, :n])
    torch.cuda.synchronize()
    y64, _ = oracle.linear(wq, a_bf16=a)
    assert max_rel_err(dev_to_bf16_bits(buf[:, :n]), y64) <= TOL
    assert torch.all(buf[:, n:] == 2.0)


@pytest.mark.parametrize("m,n,k", [(300, 12776, 1152), (2000, 4000, 128 * 9), (1030, 6464, 128), (2048, 11008, 1024 + 128),
                                   (4100, 4096 + 8, 256)])
def test_linear_two_group_kernel_many_tiles(oracle, m, n, k):
    """From about 192 tiles of 256 x 128 up the format runs on the two-group LDS-staged kernel (bare FP4 operands,
    second accumulator set per block, fold after every second K-tile): ragged M, N; one block, odd and even
    numbers of blocks; every scale word field.  Sampled outputs plus the last rows and columns."""
    print("f16-scale two-group kernel", m, n, k, flush=True)
    rng = np.random.default_rng(3900 + m + n + k)
    wq = _rand_tensor(rng, n, k)
    wq[1][0, 0] = 0x0000
    wq[1][-1, -1] = 0xFFFF
    wt = razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0))
    a = synth.activation(m, k, seed=3901 + m + k, outlier_frac=0.01)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(m, 40, 9400), np.arange(m - 6, m), np.arange(0, 3)]))
    cols = np.unique(np.concatenate([synth.sample_indices(n, 160, 9401), np.arange(n - 36, n), np.arange(0, 6)]))
    y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
    got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    assert max_rel_err(got, y64) <= TOL


MV_SHAPES = [None, (1, 1, 1), (1, 1, 2), (1, 1, 3), (1, 1, 4), (1, 2, 1), (1, 2, 2), (1, 2, 3), (1, 2, 4), (1, 2, 8)]


@pytest.mark.parametrize("shape", MV_SHAPES)
@pytest.mark.parametrize("m,ns,k", [(5, (1000,), 4096 + 128), (16, (328, 200), 1152), (9, (72,), 128), (17, (40, 24, 4), 34944),
                                    (32, (333,), 2048 + 384), (24, (100, 36), 11008)])
def test_small_batch_kernel_every_launch_shape(oracle, shape, m, ns, k):
    """5..32 activation rows run on the K-in-workgroup matrix-core kernel with bare FP4 operands and the block
    scale folded per 128-element step (one and two 16-row activation fragments; single and grouped launches;
    ragged N; one block to 273 blocks per row, several passes per wave): the default launch shape and every
    shape the tuner may force, every scale word field."""
    from paper_2501_04052_amd import binding
    print("f16-scale small batch", shape, m, ns, k, flush=True)
    rng = np.random.default_rng(3800 + m + k)
    wqs = [_rand_tensor(rng, n, k) for n in ns]
    wqs[0][1][0, 0] = 0x0000
    wqs[-1][1][-1, -1] = 0xFFFF
    wts = [razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0)) for wq in wqs]
    a = synth.activation(m, k, seed=3801 + m + k, outlier_frac=0.01)
    if shape is not None:
        razer.razer_tune_force(binding.TUNE_SMALL_BATCH, shape)
    try:
        if len(ns) == 1:
            buf = torch.full((m, ns[0] + 8), 2.0, dtype=torch.bfloat16, device="cuda")
            razer.razer_linear(wts[0], bf16_bits_to_dev(a), out=buf[:, :ns[0]])
            ys = [buf[:, :ns[0]]]
        else:
            ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
        torch.cuda.synchronize()
    finally:
        razer.razer_tune_force(binding.TUNE_SMALL_BATCH, None)
    for wq, y in zip(wqs, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL
    if len(ns) == 1:
        assert torch.all(buf[:, ns[0]:] == 2.0)


def test_linear_on_encoded_weights_full_layer_shape(oracle):
    """The Llama-7B q projection, encoded on the GPU in this format: M = 1, 4, 16 whole output, M = 512 and
    2048 on sampled outputs."""
    w = synth.weight(4096, 4096, seed=3400, outlier_frac=0.001)
    t = razer.razer_quantize(torch.from_numpy(w).cuda(), F16, (5.0, 8.0))
    torch.cuda.synchronize()
    wq = tensor_to_host(t)
    rq = oracle.quantize(F16, w)
    assert np.array_equal(wq[0], rq[0]) and np.array_equal(wq[1], rq[1]) and wq[2] == rq[2]
    for m in (1, 4, 16):
        a = synth.activation(m, 4096, seed=3401 + m)
        y = razer.razer_linear(t, bf16_bits_to_dev(a))
        torch.cuda.synchronize()
        y64, _ = oracle.linear(rq, a_bf16=a)
        assert max_rel_err(dev_to_bf16_bits(y), y64) <= TOL
    for m in (512, 2048):                                                # prefill-shaped: sampled rows x columns
        a = synth.activation(m, 4096, seed=3401 + m)
        y = razer.razer_linear(t, bf16_bits_to_dev(a))
        torch.cuda.synchronize()
        rows = synth.sample_indices(m, 64, 9000)
        cols = synth.sample_indices(4096, 256, 9001)
        y64, _ = oracle.linear(rq, a_bf16=a, rows=rows, cols=cols)
        got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
        assert max_rel_err(got, y64) <= TOL


@pytest.mark.parametrize("m,k,ns", [(1, 4096, (40, 9, 64)), (1, 11008, (70, 35)), (4, 8192, (24, 24, 24, 5)), (2, 34816, (10, 7))])
def test_grouped_small_batch_one_launch(oracle, m, k, ns):
    print("f16 grouped", m, k, ns, flush=True)
    rng = np.random.default_rng(3600 + m)
    a = synth.activation(m, k, seed=3601 + m)
    wqs = [_rand_tensor(rng, n, k) for n in ns]
    for wq in wqs:
        wq[1][:] = (wq[1] & 0xC000) | (0x2C00 + (wq[1] & 0x0FFF))    # scales 2^-4 .. 2^-1: sums stay well conditioned
    wts = [razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    for wq, wt, y in zip(wqs, wts, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL
        assert torch.equal(y, razer.razer_linear(wt, bf16_bits_to_dev(a)))


def test_grouped_and_error_paths(oracle):
    rng = np.random.default_rng(3500)
    k = 512
    a = synth.activation(2, k, seed=3501)
    wqs = [_rand_tensor(rng, n, k) for n in (33, 50)]
    wts = [razer.RazerTensor.from_host(*wq, F16, (5.0, 8.0)) for wq in wqs]
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))          # one launch (m <= 4)
    for wq, y in zip(wqs, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a)[0]) <= TOL
    a9 = synth.activation(9, k, seed=3503)
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a9))         # matrix by matrix (rows not multiples of 4)
    for wq, y in zip(wqs, ys):
        assert max_rel_err(dev_to_bf16_bits(y), oracle.linear(wq, a_bf16=a9)[0]) <= TOL
    # W4A4 is not built for this weight format
    aq = razer.razer_quantize(bf16_bits_to_dev(synth.activation(2, k, seed=3502)), razer.ACT, (5.0, 0.0))
    with pytest.raises(razer.RazerError) as e:
        razer.razer_linear(wts[0], aq)
    assert e.value.status == 4
