"""GPU parity at the full sizes of the benchmark configurations, in the launch configurations
bench.py times: encoders bit-exact on whole tensors, linear outputs either whole (M <= 16) or on
sampled rows x columns (64 x 256, full K) that the oracle computes one by one."""
import numpy as np
import pytest
import torch

import paper_2501_04052_amd as razer
from paper_2501_04052_amd import binding, synth
from gpu_util import TOL, bf16_bits_to_dev, dev_to_bf16_bits, max_rel_err, tensor_to_host

pytestmark = pytest.mark.gpu
W, A = 0, 1
SV = (5.0, 8.0)


def _say(*a):
    print(*a, flush=True)


def _rand_packed(n, k, seed):
    """Random packed bytes: every code, every scale byte (all 64 scale codes, zero and subnormal scales
    included, all four metadata values)."""
    rng = np.random.default_rng(seed)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(n, k // 16), dtype=np.uint8)
    return codes, scales, np.float32(2.0 ** -10)


def _check_linear(oracle, wq, wt, m, seed, sampled):
    n, k = wq[0].shape[0], wq[0].shape[1] * 2
    a = synth.activation(m, k, seed=seed)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    if sampled:
        rows = synth.sample_indices(m, 64, 9000)
        cols = synth.sample_indices(n, 256, 9001)
        y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
        got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    else:
        y64, _ = oracle.linear(wq, a_bf16=a)
        got = dev_to_bf16_bits(y)
    err = max_rel_err(got, y64)
    _say("   linear m=%d n=%d k=%d sampled=%s max rel err %.2e" % (m, n, k, sampled, err))
    assert err <= TOL, err


def _encode_and_check(oracle, x_host, fmt, sv):
    x_dev = bf16_bits_to_dev(x_host) if x_host.dtype == np.uint16 else torch.from_numpy(x_host).cuda()
    t = razer.razer_quantize(x_dev, fmt, sv)
    torch.cuda.synchronize()
    del x_dev
    ref = oracle.quantize(fmt, x_host, sv=sv)
    codes, scales, ts = tensor_to_host(t)
    assert np.float32(ts).view(np.uint32) == np.float32(ref[2]).view(np.uint32)
    assert np.array_equal(scales, ref[1]), "scale bytes differ"
    assert np.array_equal(codes, ref[0]), "codes differ"
    return t, ref


def test_config1_single_layer_4096(oracle):
    _say("config 1: 4096x4096 encode + M=1 linear + dequant")
    w = synth.weight(4096, 4096, seed=1000)
    wt, wq = _encode_and_check(oracle, w, W, SV)
    frac8 = np.mean((wq[1] >> 6) & 1)
    _say("   blocks choosing the second special-value pair: %.4f" % frac8)
    _check_linear(oracle, wq, wt, 1, 1001, sampled=False)
    ref = oracle.dequant(W, *wq, want=("bf16",))["bf16"]
    assert np.array_equal(dev_to_bf16_bits(razer.razer_dequant(wt, torch.bfloat16)), ref)


@pytest.mark.parametrize("name,n,k,idx", [("q", 4096, 4096, 0), ("gate", 11008, 4096, 4), ("down", 4096, 11008, 6)])
def test_config2_3_llama7b_layer(oracle, name, n, k, idx):
    _say("config 2/3: %s %dx%d, encode + M in {1,2,4,16} whole + M in {512,2048} sampled" % (name, n, k))
    w = synth.weight(n, k, seed=2000 + idx, outlier_frac=0.001)
    wt, wq = _encode_and_check(oracle, w, W, SV)
    del w
    for m in (1, 2, 4, 16):
        _check_linear(oracle, wq, wt, m, 2100 + m, sampled=False)
    for m in (512, 2048):
        _check_linear(oracle, wq, wt, m, 2100 + m, sampled=True)


@pytest.mark.parametrize("name,n,k,idx", [(name, n, k, i) for i, (name, n, k) in enumerate(synth.LLAMA_70B_LAYER)])
def test_config4_llama70b_layer(oracle, name, n, k, idx):
    """Every tensor of the 70B-shaped layer from the seeded Student-t generator (seed 4000 + index): encoded
    on the GPU and by the oracle, bit for bit, one tensor at a time; then the linear layer on those ENCODED
    weights -- M = 1 whole output for every tensor; M = 8 and M = 4096 for one tensor of each shape (whole
    output where the oracle finishes in seconds, else 64 sampled rows x 256 sampled columns)."""
    _say("config 4: %s %dx%d seed %d, encode + linear on the encoded weights" % (name, n, k, 4000 + idx))
    w = synth.weight(n, k, seed=4000 + idx, outlier_frac=0.001)
    wt, wq = _encode_and_check(oracle, w, W, SV)
    del w
    _check_linear(oracle, wq, wt, 1, 4101, sampled=False)
    if name in ("q", "k", "gate", "down"):
        _check_linear(oracle, wq, wt, 8, 4108, sampled=n * k > 2 ** 24)
        _check_linear(oracle, wq, wt, 4096, 4100 + 4096, sampled=True)


def test_config5_w4a4(oracle):
    _say("config 5: activation 4096x4096 encode (E4M3 + 1 bit, +-5) and W4A4 linear vs the encoded gate-shaped weight 11008x4096 (seed 5001)")
    a = synth.activation(4096, 4096, seed=5000, outlier_frac=0.005, outlier_gain=50.0)
    at, aq = _encode_and_check(oracle, a, A, (5.0, 0.0))
    frac = np.mean(((aq[0] & 15) == 8) | ((aq[0] >> 4) == 8))
    _say("   activation elements on the special value: %.4f" % frac)
    assert frac > 0.005
    w = synth.weight(11008, 4096, seed=5001, outlier_frac=0.001)   # the gate-shaped weight, encoded here too
    wt, wq = _encode_and_check(oracle, w, W, SV)
    del w
    rows = synth.sample_indices(4096, 64, 9000)
    cols = synth.sample_indices(11008, 256, 9001)
    y64, _ = oracle.linear(wq, a_q=aq, rows=rows, cols=cols)
    # both forms of the call: with room for the decoded activations (the binding's default), and with a token
    # workspace, which keeps the single fused kernel
    assert razer.razer_workspace_bytes(binding.OP_LINEAR_W4A4, 11008, 4096, 4096) == 4096 * 4096 * 2 + 256
    for label, ws in (("decoded activations + weight-only kernel", None),
                      ("fused kernel", torch.empty(max(256, razer.razer_workspace_bytes(binding.OP_LINEAR, 11008, 4096, 4096)),
                                                   dtype=torch.uint8, device="cuda"))):
        y = razer.razer_linear(wt, at, workspace=ws)
        torch.cuda.synchronize()
        got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
        err = max_rel_err(got, y64)
        _say("   w4a4 (%s) max rel err %.2e" % (label, err))
        assert err <= TOL, (label, err)


@pytest.mark.parametrize("m,n,k,ablock", [(300, 12776, 1088, 16), (2000, 4000, 1056, 16), (4100, 4096 + 8, 160, 16),
                                          (8192, 2048 + 40, 32, 16), (2048, 11008, 1024 + 64, 32), (1030, 6400 + 64, 4096, 64)])
def test_w4a4_decoded_activations_then_weight_only_kernel(oracle, m, n, k, ablock):
    """W4A4 with room in the workspace: the library decodes the activations once into bf16 and runs the weight-only
    path (here the register-decode kernel: 128- and 256-wide tiles, the two-K-group round; ragged M, N, K;
    activation blocks of 16, 32, 64): random code and scale bytes on both operands, sampled outputs against the
    oracle, and the same call with a token workspace (fused kernel) against the same values."""
    _say("w4a4 decoded-activation path m=%d n=%d k=%d activation block %d" % (m, n, k, ablock))
    need = razer.razer_workspace_bytes(binding.OP_LINEAR_W4A4, n, k, m)
    assert need == (m * k * 2 + 255) // 256 * 256 + 256 + razer.razer_workspace_bytes(binding.OP_LINEAR, n, k, m)
    rng = np.random.default_rng(7300 + m + n + k)
    wq = (rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8), rng.integers(0, 256, size=(n, k // 16), dtype=np.uint8),
          np.float32(2.0 ** -9))
    asc = rng.integers(0, 256, size=(m, k // ablock), dtype=np.uint8)
    asc = (asc & 0x80) | (40 + (asc & 31))                             # E4M3 codes 40..71: 2^-2 .. 3.75
    aq = (rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8), asc.astype(np.uint8), np.float32(2.0 ** -3))
    wt = razer.RazerTensor.from_host(*wq, W, SV)
    at = razer.RazerTensor.from_host(*aq, A, (5.0, 0.0))
    rows = np.unique(np.concatenate([synth.sample_indices(m, 40, 9300), np.arange(m - 6, m), np.arange(0, 3)]))
    cols = np.unique(np.concatenate([synth.sample_indices(n, 160, 9301), np.arange(n - 36, n), np.arange(0, 6)]))
    y64, _ = oracle.linear(wq, a_q=aq, rows=rows, cols=cols)
    fused_ws = torch.empty(max(256, razer.razer_workspace_bytes(binding.OP_LINEAR, n, k, m)), dtype=torch.uint8, device="cuda")
    for label, ws in (("decoded", None), ("fused", fused_ws)):
        y = razer.razer_linear(wt, at, workspace=ws)
        torch.cuda.synchronize()
        got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
        err = max_rel_err(got, y64)
        _say("   %s: max rel err %.2e over %d x %d sampled outputs" % (label, err, len(rows), len(cols)))
        assert err <= TOL, (label, err)


@pytest.mark.parametrize("m,n,k", [(8192, 2048 + 40, 32), (4100, 4096 + 8, 160), (16384, 4096, 96),
                                   (16300, 4096 + 31, 64 + 32), (2048, 11008, 4096 + 32),
                                   # about one 256 x 128 tile per compute unit: K halved inside the workgroup
                                   (2048, 4096, 4096), (2048, 4096, 11008), (300, 12776, 1088), (2000, 4000, 1056)])
def test_linear_many_tiles_register_decode_kernel(oracle, m, n, k):
    """Shapes with >= 512 output tiles take the GEMM kernel that decodes weights in registers and stages
    operands with global->LDS copies: ragged M, N and K tails (K = 32: half a K-tile; K % 64 = 32), one
    to 172 K-tiles (odd counts leave the second K group of the one-round variant an empty tile).  Sampled
    rows x columns plus the last rows and columns, all scale bytes."""
    _say("many-tile GEMM m=%d n=%d k=%d" % (m, n, k))
    rng = np.random.default_rng(7000 + m + n + k)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(n, k // 16), dtype=np.uint8)
    wq = (codes, scales, np.float32(2.0 ** -9))
    wt = razer.RazerTensor.from_host(*wq, W, SV)
    a = synth.activation(m, k, seed=7001 + m, outlier_frac=0.005, outlier_gain=50.0)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(m, 48, 9100), np.arange(m - 8, m), np.arange(0, 4)]))
    cols = np.unique(np.concatenate([synth.sample_indices(n, 192, 9101), np.arange(n - 40, n), np.arange(0, 8)]))
    y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
    got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    err = max_rel_err(got, y64)
    _say("   max rel err %.2e over %d x %d sampled outputs" % (err, len(rows), len(cols)))
    assert err <= TOL, err


_BLOCK_SHAPES = [(4100, 4096 + 8, 128 + 32 * 4), (2048, 4096, 4096 + 128), (8192, 4096 + 40, 384),
                 (100, 4096, 4096), (64, 11008, 1024 + 128), (2048, 11008, 1152)]


@pytest.mark.parametrize("block,m,n,k", [(b, m, n, k) for b in (32, 64, 128) for m, n, k in _BLOCK_SHAPES if k % b == 0])
def test_block_sizes_register_decode_kernel(oracle, block, m, n, k):
    """32-, 64- and 128-element blocks through the register-decode GEMM (one scale byte per lane and
    K-tile, copied with a 1-byte global->LDS copy): 128- and 256-wide tiles, the two-K-group round, 64- and
    128-row tiles with K-slices, ragged K-tiles (K a multiple of the block size only).  Sampled outputs."""
    _say("block %d register-decode GEMM m=%d n=%d k=%d" % (block, m, n, k))
    rng = np.random.default_rng(7100 + m + n + k + block)
    codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    scales = rng.integers(0, 256, size=(n, k // block), dtype=np.uint8)
    wq = (codes, scales, np.float32(2.0 ** -9))
    wt = razer.RazerTensor.from_host(*wq, W, SV)
    a = synth.activation(m, k, seed=7101 + m, outlier_frac=0.005, outlier_gain=50.0)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(m, 48, 9100), np.arange(max(m - 8, 0), m), np.arange(0, 4)]))
    cols = np.unique(np.concatenate([synth.sample_indices(n, 192, 9101), np.arange(n - 40, n), np.arange(0, 8)]))
    y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
    got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    err = max_rel_err(got, y64)
    _say("   max rel err %.2e over %d x %d sampled outputs" % (err, len(rows), len(cols)))
    assert err <= TOL, err


@pytest.mark.parametrize("m,n,k", [(64, 4096, 4096), (128, 4096, 11008), (256, 4096, 4096), (100, 11008, 4096)])
def test_config2_3_mid_batch_single_calls(oracle, m, n, k):
    """o- and down-shaped projections (and a gate-shaped one) at the batch sizes between decode and large
    GEMMs: register-decode kernel with 64 / 128-row tiles and K-slices, the LDS-staged split-K kernel at 256."""
    _say("mid batch at full size, m=%d n=%d k=%d" % (m, n, k))
    wq = _rand_packed(n, k, seed=8300 + m)
    wt = razer.RazerTensor.from_host(*wq, W, SV)
    a = synth.activation(m, k, seed=2300 + m)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(m, 32, 9400), [0, m - 1]]))
    cols = np.unique(np.concatenate([synth.sample_indices(n, 160, 9401), [0, n - 1]]))
    y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
    got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
    err = max_rel_err(got, y64)
    _say("   %d x %d outputs, max rel err %.2e" % (len(rows), len(cols), err))
    assert err <= TOL, err


def test_kv_cache_shaped_activation_tensors(oracle):
    """The joint weight / activation / KV-cache setting (App. on W-A-KV results) stores K and V in the
    activation format: a [tokens x heads][head_dim = 128] bf16 tensor with a calibrated (given) tensor
    scale, encoded and decoded through the same entry points.  Sampled rows against the oracle, bit for bit."""
    tokens, heads, hd = 4096, 32, 128
    _say("KV-cache-shaped tensor %d x %d" % (tokens * heads, hd))
    x = synth.activation(tokens * heads, hd, seed=7700, outlier_frac=0.002)
    given = np.float32(np.abs(synth.bf16_bits_to_f32(x[:4096])).max() / (448.0 * 6.0))   # "calibration" on a prefix
    ts = torch.tensor([given], dtype=torch.float32, device="cuda")
    t = razer.razer_quantize(bf16_bits_to_dev(x), A, (5.0, 0.0), tensor_scale=ts)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(tokens * heads, 4096, 9600), [0, tokens * heads - 1]]))
    rc, rs, rts = oracle.quantize(A, x[rows], sv=(5.0, 0.0), given_tensor_scale=given)
    idx = torch.from_numpy(rows).cuda()
    assert np.array_equal(t.codes[idx].cpu().numpy(), rc) and np.array_equal(t.scales[idx].cpu().numpy(), rs)
    assert np.float32(t.tensor_scale.cpu().numpy()[0]) == rts == given
    deq = razer.razer_dequant(t, torch.bfloat16)
    ref = oracle.dequant(A, rc, rs, rts, sv=(5.0, 0.0), want=("bf16",))["bf16"]
    assert np.array_equal(dev_to_bf16_bits(deq[idx]), ref)


@pytest.mark.parametrize("m,k", [(8, (1 << 24) + 64), (40, (1 << 22) + 64), (300, (1 << 22) + 64)])
def test_rows_longer_than_the_32_bit_offset_kernels_take(oracle, m, k):
    """The small-batch kernel and the register-decode GEMM address inside a tile with 32-bit offsets; rows
    beyond their limits must go to the kernels with 64-bit addressing, not overflow."""
    _say("very long rows, m=%d k=%d" % (m, k))
    n = 3
    wq = _rand_packed(n, k, seed=8400 + m)
    wt = razer.RazerTensor.from_host(*wq, W, SV)
    a = synth.activation(m, k, seed=2400 + m)
    y = razer.razer_linear(wt, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([synth.sample_indices(m, 6, 9500), [0, m - 1]]))
    y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=np.arange(n))
    got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()])
    err = max_rel_err(got, y64)
    _say("   max rel err %.2e" % err)
    assert err <= TOL, err


@pytest.mark.parametrize("m", [1, 4, 16, 64, 128, 256, 512, 2048])
def test_config2_3_grouped_launches_as_benchmarked(oracle, m):
    """The launch configuration bench.py times: {q,k,v} and {gate,up} of the Llama-7B-shaped layer each
    as ONE razer_linear_grouped call (grouped GEMV, matrix-instruction GEMV, grouped small-batch kernel
    with its grouped reduction, grouped register-decode GEMM -- with K-slices and the grouped reduction
    at M = 64, 128, 256).  Whole outputs up to M = 16, sampled rows x columns beyond."""
    _say("grouped launches at full size, m=%d" % m)
    a = synth.activation(m, 4096, seed=2100 + m)
    a_dev = bf16_bits_to_dev(a)
    for name, n, count, seed in (("qkv", 4096, 3, 8000), ("gate_up", 11008, 2, 8100)):
        wqs = [_rand_packed(n, 4096, seed=seed + i + m) for i in range(count)]
        wts = [razer.RazerTensor.from_host(*wq, W, SV) for wq in wqs]
        ys = razer.razer_linear_grouped(wts, a_dev)
        torch.cuda.synchronize()
        if m <= 16:
            rows, cols = np.arange(m), np.arange(n)
        else:
            rows = np.unique(np.concatenate([synth.sample_indices(m, 32, 9200), [0, m - 1]]))
            cols = np.unique(np.concatenate([synth.sample_indices(n, 128, 9201), [0, n - 1]]))
        for wq, y in zip(wqs, ys):
            y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
            got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
            err = max_rel_err(got, y64)
            _say("   %s m=%d: %d x %d outputs, max rel err %.2e" % (name, m, len(rows), len(cols), err))
            assert err <= TOL, err


@pytest.mark.parametrize("m", [1, 4])
def test_prepacked_layout_as_benchmarked(oracle, m):
    """bench.py's pre-packed legs: the Llama-7B-shaped layer repacked with razer_prepack, {q,k,v} and {gate,up} as
    grouped calls, o and down as single calls -- every output bit-identical to the canonical layout's, and the down
    projection (the long-row shape the layout is meant for) against the oracle."""
    _say("pre-packed layout at full size, m=%d" % m)
    for name, ns, k, seed in (("qkv", (4096, 4096, 4096), 4096, 8300), ("o", (4096,), 4096, 8310),
                              ("gate_up", (11008, 11008), 4096, 8320), ("down", (4096,), 11008, 8330)):
        a = synth.activation(m, k, seed=2100 + m + k)
        a_dev = bf16_bits_to_dev(a)
        wqs = [_rand_packed(n, k, seed=seed + i + m) for i, n in enumerate(ns)]
        wts = [razer.RazerTensor.from_host(*wq, W, SV) for wq in wqs]
        pks = [razer.razer_prepack(w) for w in wts]
        if len(ns) == 1:
            ys_c, ys_p = [razer.razer_linear(wts[0], a_dev)], [razer.razer_linear(pks[0], a_dev)]
        else:
            ys_c, ys_p = razer.razer_linear_grouped(wts, a_dev), razer.razer_linear_grouped(pks, a_dev)
        torch.cuda.synchronize()
        for yc, yp in zip(ys_c, ys_p):
            assert torch.equal(yc, yp), name
        if name == "down":
            err = max_rel_err(dev_to_bf16_bits(ys_p[0]), oracle.linear(wqs[0], a_bf16=a)[0])
            _say("   down, pre-packed, m=%d: max rel err %.2e" % (m, err))
            assert err <= TOL, err


@pytest.mark.parametrize("m", [1, 16, 64, 2048])
def test_fp16_scale_format_as_benchmarked(oracle, m):
    """bench.py's FP16-scale legs: {gate,up}-shaped tensors (2 x 11008 x 4096, blocks of 128, random scale words) as
    one razer_linear_grouped call -- grouped GEMV at M = 1, the grouped K-in-workgroup kernel at 16, per matrix the
    four-fragment kernel at 64 and the two-group tiled kernel at 2048.  Whole outputs up to M = 16, sampled beyond."""
    from paper_2501_04052_amd import binding
    _say("FP16-scale format at full size, m=%d" % m)
    n, k = 11008, 4096
    rng = np.random.default_rng(8400 + m)
    wqs = []
    for i in range(2):
        codes = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
        words = rng.integers(0, 65536, size=(n, k // 128), dtype=np.uint16)
        wqs.append((codes, words, np.float32(2.0 ** -10)))
    wts = [razer.RazerTensor.from_host(*wq, binding.WEIGHT_F16, SV) for wq in wqs]
    a = synth.activation(m, k, seed=8401 + m)
    ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
    torch.cuda.synchronize()
    if m <= 16:
        rows, cols = np.arange(m), np.arange(n)
    else:
        rows = np.unique(np.concatenate([synth.sample_indices(m, 32, 9500), [0, m - 1]]))
        cols = np.unique(np.concatenate([synth.sample_indices(n, 128, 9501), [0, n - 1]]))
    for wq, y in zip(wqs, ys):
        y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
        got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
        err = max_rel_err(got, y64)
        _say("   m=%d: %d x %d outputs, max rel err %.2e" % (m, len(rows), len(cols), err))
        assert err <= TOL, err


def test_config4_grouped_launches_as_benchmarked(oracle):
    """70B-shaped {q,k,v} (8192 + 1024 + 1024 rows) as one grouped call at M = 1, 8 and 4096."""
    wqs = [_rand_packed(n, 8192, seed=8200 + i) for i, n in enumerate((8192, 1024, 1024))]
    wts = [razer.RazerTensor.from_host(*wq, W, SV) for wq in wqs]
    for m in (1, 8, 4096):
        _say("70B grouped q,k,v m=%d" % m)
        a = synth.activation(m, 8192, seed=4100 + m)
        ys = razer.razer_linear_grouped(wts, bf16_bits_to_dev(a))
        torch.cuda.synchronize()
        rows = np.arange(m) if m <= 8 else np.unique(np.concatenate([synth.sample_indices(m, 32, 9300), [0, m - 1]]))
        for wq, y in zip(wqs, ys):
            n = wq[0].shape[0]
            cols = np.unique(np.concatenate([synth.sample_indices(n, 128, 9301), [0, n - 1]]))
            y64, _ = oracle.linear(wq, a_bf16=a, rows=rows, cols=cols)
            got = dev_to_bf16_bits(y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
            err = max_rel_err(got, y64)
            _say("   n=%d: max rel err %.2e" % (n, err))
            assert err <= TOL, err
