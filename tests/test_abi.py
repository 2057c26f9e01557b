"""The C-ABI library loads, exports every symbol the header declares, and turns
bad arguments into status codes before any GPU work (runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def razer():
    import paper_2501_04052_amd as r
    if not os.path.exists(r.lib_path()):
        from paper_2501_04052_amd import build
        build.build()
    r.load_library()
    return r


def test_header_symbols_are_exported(razer):
    header = open(os.path.join(ROOT, "include", "razer.h")).read()
    names = set(re.findall(r"\b(razer_[a-z_]+)\s*\(", header))
    assert {"razer_quantize", "razer_dequant", "razer_linear", "razer_workspace_bytes",
            "razer_status_string"} <= names
    lib = ctypes.CDLL(razer.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    from paper_2501_04052_amd import binding
    assert set(binding.EXPORTS) == names
    probe = open(os.path.join(ROOT, "include", "razer_probe.h")).read()
    pnames = set(re.findall(r"\b(razer_probe_[a-z_0-9]+)\s*\(", probe))
    assert pnames == set(binding.PROBE_EXPORTS)
    for n in pnames:
        assert hasattr(lib, n), n
    tune = open(os.path.join(ROOT, "include", "razer_tune.h")).read()
    tnames = set(re.findall(r"\b(razer_tune_[a-z_0-9]+)\s*\(", tune))
    assert tnames == set(binding.TUNE_EXPORTS)
    for n in tnames:
        assert hasattr(lib, n), n


def test_tuning_hooks_force_lookup_and_workspace(razer):
    """Forcing a launch shape is visible through the lookup and through the workspace query (the
    K-in-workgroup small-batch kernel needs none); clearing restores the table / heuristic; a forced
    shape the kernels are not built for falls back to the heuristic."""
    from paper_2501_04052_amd import binding as b
    fam = b.TUNE_SMALL_BATCH
    # 30000 rows: no table entry, and too many 16-row groups for one round of workgroups -> K-sliced by default
    base = razer.razer_workspace_bytes(2, 30000, 4096, 16)
    src0, shape0 = razer.razer_tune_lookup(fam, 16, 30000, 4096)
    assert src0 == 0 and shape0 is None and base == 8 * 16 * 30000 * 4
    razer.razer_tune_force(fam, (1, 1, 2))
    assert razer.razer_tune_lookup(fam, 16, 30000, 4096) == (1, (1, 1, 2, 0))
    assert razer.razer_workspace_bytes(2, 30000, 4096, 16) == 0
    assert razer.razer_workspace_bytes(2, 30000, 4096, 20) == 8 * 20 * 30000 * 4   # more than 16 rows: K-sliced kernel
    razer.razer_tune_force(fam, (0, 8, 1))
    assert razer.razer_workspace_bytes(2, 30000, 4096, 16) == 4 * 16 * 30000 * 4
    assert razer.razer_workspace_bytes(2, 4100, 4096, 16) == 4 * 16 * 4100 * 4
    razer.razer_tune_force(fam, (1, 3, 5))                                        # not a built shape
    assert razer.razer_workspace_bytes(2, 30000, 4096, 16) == base
    razer.razer_tune_force(fam, None)
    assert razer.razer_tune_lookup(fam, 16, 30000, 4096)[0] == 0
    assert razer.razer_workspace_bytes(2, 30000, 4096, 16) == base
    # 4100 rows = 257 groups of 16: two groups per workgroup make one round -> K inside the workgroup, no workspace
    assert razer.razer_tune_lookup(fam, 16, 4100, 4096)[0] == 0 and razer.razer_workspace_bytes(2, 4100, 4096, 16) == 0
    razer.razer_tune_force(-1, None)
    with pytest.raises(razer.RazerError):
        razer.razer_tune_force(9, (1, 2))
    assert razer.razer_tune_table_size() >= 0


def test_status_strings(razer):
    seen = {razer.razer_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert razer.razer_status_string(99) == "unknown status"


def test_workspace_sizes(razer):
    assert razer.razer_workspace_bytes(0, 4096, 4096) >= 4
    assert razer.razer_workspace_bytes(1, 4096, 4096) == 0
    # linear: only the 5..32-row kernel meets its K-slices in a workspace
    assert razer.razer_workspace_bytes(2, 4096, 4096, 1) == 0
    assert razer.razer_workspace_bytes(2, 4096, 4096, 2048) == 0
    assert razer.razer_workspace_bytes(2, 30000, 4096, 16) == 8 * 16 * 30000 * 4   # (a shape the tuned table does not list)
    assert razer.razer_workspace_bytes(2, 4100, 4096, 20) == 8 * 20 * 4100 * 4
    assert razer.razer_workspace_bytes(2, 4096, 512, 16) == 0
    # W4A4 query: room for the activations decoded to bf16 (rounded up to 256 bytes), one 256-byte cell for the
    # combined tensor scale, plus what the weight-only path needs for the same sizes
    for n, k, m in ((11008, 4096, 4096), (4096, 4096, 2048), (4096, 4096, 64), (4100, 4096, 16), (30000, 4096, 16), (512, 4096, 1024), (4096, 4096, 1),
                    (40, 96, 3)):
        a_bytes = (m * k * 2 + 255) // 256 * 256
        assert razer.razer_workspace_bytes(3, n, k, m) == a_bytes + 256 + razer.razer_workspace_bytes(2, n, k, m)
    assert razer.razer_workspace_bytes(3, 4096, 4096, 0) == 0


def test_grouped_workspace_query_covers_single_launch_and_fallback(razer):
    """The grouped query is never smaller than any per-matrix size (the fallback sequence of calls
    must fit) and, where K-slices are chosen for all matrices together, can exceed their sum."""
    q = razer.razer_workspace_bytes_grouped
    one = lambda n, k, m: razer.razer_workspace_bytes(2, n, k, m)
    assert q([4096, 4096, 4096], 4096, 1) == 0 and q([], 4096, 16) == 0 and q([4096] * 5, 4096, 16) == 0
    # small batch: K-slices of the matrices side by side (shapes the tuned table does not list)
    assert q([11000, 11000], 4096, 20) == 2 * one(11000, 4096, 20) > 0 and q([11000, 11000], 4096, 16) > 0
    for rows, k, m in (([4096, 4096, 4096], 4096, 64), ([11008, 11008], 4096, 128), ([1024, 23040], 4096, 256),
                       ([4096, 4096, 4096], 4096, 2048)):
        assert q(rows, k, m) >= max(one(n, k, m) for n in rows)
    # one small and one large matrix at m > 128: slices chosen over the group, more than the sum
    assert q([1024, 23040], 4096, 256) >= one(1024, 4096, 256) + one(23040, 4096, 256)


def test_bad_arguments_return_status_codes_without_gpu(razer):
    from paper_2501_04052_amd.binding import _Config, _Tensor, load_library
    L = load_library()
    cfg = _Config(); cfg.format = 0; cfg.sv[0] = 5.0; cfg.sv[1] = 8.0
    fake = ctypes.c_void_p(0x1000)          # aligned, never dereferenced: every call fails validation first
    odd = ctypes.c_void_p(0x1004)
    q = lambda **kw: L.razer_quantize(kw.get("cfg", ctypes.byref(cfg)), kw.get("x", fake), kw.get("dtype", 0),
                                      kw.get("rows", 4), kw.get("cols", 64), kw.get("ld", 64),
                                      kw.get("codes", fake), kw.get("scales", fake), kw.get("ts", fake),
                                      kw.get("flags", 0), kw.get("ws", fake), kw.get("wsb", 256), None)
    assert q(cfg=None) == 1 and q(x=None) == 1 and q(ts=None) == 1
    assert q(cols=48) == 2 and q(cols=-32) == 2 and q(ld=32) == 2 and q(rows=-1) == 2
    assert q(x=odd) == 3 and q(ld=66) == 3
    assert q(dtype=7) == 4 and q(flags=8) == 4
    assert q(ws=None) == 5 and q(wsb=1) == 5
    for bad in (6.0, 4.0, 5.25, 10.0, 2.0, float("nan")):
        c2 = _Config(); c2.format = 0; c2.sv[0] = bad; c2.sv[1] = 8.0
        assert q(cfg=ctypes.byref(c2)) == 4
    c3 = _Config(); c3.format = 3; c3.sv[0] = 5.0; c3.sv[1] = 8.0
    assert q(cfg=ctypes.byref(c3)) == 4
    # block sizes: 0 (= 16), 16, 32, 64, 128 only; cols must hold whole blocks
    for blk, cols, want in ((48, 96, 4), (8, 64, 4), (256, 256, 4), (-16, 64, 4), (64, 96, 2), (128, 64, 2)):
        c4 = _Config(); c4.format = 0; c4.sv[0] = 5.0; c4.sv[1] = 8.0; c4.block = blk
        assert q(cfg=ctypes.byref(c4), cols=cols, ld=cols) == want, (blk, cols)

    t = _Tensor(); t.codes = 0x1000; t.scales = 0x2000; t.tensor_scale = 0x3000
    t.rows = 8; t.cols = 64; t.cfg = cfg
    assert L.razer_dequant(None, fake, 0, 64, None) == 1
    assert L.razer_dequant(ctypes.byref(t), None, 0, 64, None) == 1
    assert L.razer_dequant(ctypes.byref(t), fake, 0, 32, None) == 2
    assert L.razer_dequant(ctypes.byref(t), odd, 0, 64, None) == 3
    assert L.razer_dequant(ctypes.byref(t), fake, 5, 64, None) == 4
    cb = _Config(); cb.format = 0; cb.sv[0] = 5.0; cb.sv[1] = 8.0; cb.block = 128
    t128 = _Tensor(); t128.codes = 0x1000; t128.scales = 0x2000; t128.tensor_scale = 0x3000
    t128.rows = 8; t128.cols = 64; t128.cfg = cb                  # 64 columns cannot hold a block of 128
    assert L.razer_dequant(ctypes.byref(t128), fake, 0, 64, None) == 2
    assert L.razer_linear(ctypes.byref(t128), fake, None, 1, fake, 8, None, 0, None) == 2
    # the FP16-scale weight format: blocks of 128 only, columns in whole blocks
    for blk, cols, want in ((16, 128, 4), (64, 128, 4), (32, 256, 4), (0, 192, 2), (128, 64, 2)):
        c5 = _Config(); c5.format = 2; c5.sv[0] = 5.0; c5.sv[1] = 8.0; c5.block = blk
        assert q(cfg=ctypes.byref(c5), cols=cols, ld=cols) == want, (blk, cols)
    c6 = _Config(); c6.format = 2; c6.sv[0] = 5.0; c6.sv[1] = 6.0                    # second special value invalid
    assert q(cfg=ctypes.byref(c6), cols=128, ld=128) == 4
    # linear: both or neither activation operand, wrong formats, shape mismatches
    assert L.razer_linear(ctypes.byref(t), None, None, 1, fake, 8, None, 0, None) == 1
    assert L.razer_linear(ctypes.byref(t), None, None, 0, None, 8, None, 0, None) == 0
    assert L.razer_linear(ctypes.byref(t), fake, ctypes.byref(t), 1, fake, 8, None, 0, None) == 1
    assert L.razer_linear(ctypes.byref(t), fake, None, 1, fake, 4, None, 0, None) == 2
    assert L.razer_linear(ctypes.byref(t), fake, None, -1, fake, 8, None, 0, None) == 2
    assert L.razer_linear(ctypes.byref(t), odd, None, 1, fake, 8, None, 0, None) == 3
    tb = _Tensor(); tb.codes = 0x1000; tb.scales = 0x2000; tb.tensor_scale = 0x3000
    tb.rows = 8; tb.cols = 1024; tb.cfg = cfg
    assert L.razer_linear(ctypes.byref(tb), fake, None, 8, fake, 8, None, 0, None) == 5      # needs a workspace
    assert L.razer_linear(ctypes.byref(tb), fake, None, 8, fake, 8, fake, 16, None) == 5     # too small
    # a GEMM with few output tiles splits K and needs the workspace as well
    assert L.razer_workspace_bytes(2, 8, 1024, 512) == 2 * 512 * 8 * 4
    assert L.razer_linear(ctypes.byref(tb), fake, None, 512, fake, 8, None, 0, None) == 5
    assert L.razer_workspace_bytes(2, 4096, 4096, 512) == 4 * 512 * 4096 * 4
    assert L.razer_workspace_bytes(2, 4096, 4096, 2048) == 0     # 256 tiles: no split
    assert L.razer_workspace_bytes(2, 11008, 4096, 2048) == 0
    ta = _Tensor(); ta.codes = 0x1000; ta.scales = 0x2000; ta.tensor_scale = 0x3000
    ta.rows = 2; ta.cols = 64; ta.cfg = cfg                      # weight format used as activation
    assert L.razer_linear(ctypes.byref(t), None, ctypes.byref(ta), 2, fake, 8, None, 0, None) == 4
    ca = _Config(); ca.format = 1; ca.sv[0] = 5.0
    ta.cfg = ca; ta.cols = 32
    assert L.razer_linear(ctypes.byref(t), None, ctypes.byref(ta), 2, fake, 8, None, 0, None) == 2
    tw = _Tensor(); tw.codes = 0x1000; tw.scales = 0x2000; tw.tensor_scale = 0x3000
    tw.rows = 8; tw.cols = 64; tw.cfg = ca                      # activation format used as weight
    assert L.razer_linear(ctypes.byref(tw), fake, None, 1, fake, 8, None, 0, None) == 4
    # grouped: null arrays, bad counts, mismatched K
    PT = ctypes.POINTER(_Tensor)
    t2 = _Tensor(); t2.codes = 0x1000; t2.scales = 0x2000; t2.tensor_scale = 0x3000
    t2.rows = 8; t2.cols = 96; t2.cfg = cfg
    arr = (PT * 2)(ctypes.pointer(t), ctypes.pointer(t2))
    ys = (ctypes.c_void_p * 2)(0x4000, 0x5000)
    lds = (ctypes.c_int64 * 2)(8, 8)
    assert L.razer_linear_grouped(None, 2, fake, 1, ys, lds, None, 0, None) == 1
    assert L.razer_linear_grouped(arr, 0, fake, 1, ys, lds, None, 0, None) == 2
    assert L.razer_linear_grouped(arr, 5, fake, 1, ys, lds, None, 0, None) == 2
    assert L.razer_linear_grouped(arr, 2, fake, 1, ys, lds, None, 0, None) == 2      # cols differ
    t2.cols = 64
    lds_bad = (ctypes.c_int64 * 2)(8, 4)
    assert L.razer_linear_grouped(arr, 2, fake, 1, ys, lds_bad, None, 0, None) == 2
    assert L.razer_linear_grouped(arr, 2, None, 1, ys, lds, None, 0, None) == 1
    assert L.razer_linear_grouped(arr, 2, odd, 1, ys, lds, None, 0, None) == 3
    assert L.razer_linear_grouped(arr, 2, None, 0, ys, lds, None, 0, None) == 0
    # grouped small batch without the workspace of even one matrix: the sequence of single calls reports it
    arr_b = (PT * 2)(ctypes.pointer(tb), ctypes.pointer(tb))
    assert L.razer_linear_grouped(arr_b, 2, fake, 8, ys, lds, None, 0, None) == 5
    assert L.razer_linear_grouped(arr_b, 2, fake, 8, ys, lds, fake, 16, None) == 5
    # empty problems are fine and launch nothing
    assert L.razer_linear(ctypes.byref(t), fake, None, 0, None, 8, None, 0, None) == 0


def test_every_table_entry_names_a_launch_shape_the_tuner_can_pick(razer):
    """csrc/razer_tuned.inc is written by the tuner: every entry must be one of the candidate shapes of its
    family for that (m, k) -- a stale or hand-edited table would silently fall back to the heuristic -- and the
    library must report exactly that entry through the lookup."""
    import re
    from paper_2501_04052_amd import tune
    text = open(tune.TABLE_PATH).read()
    entries = re.findall(r"\{(\d+), (\d+), (\d+), (\d+), \{(-?\d+), (-?\d+), (-?\d+), (-?\d+)\}\}", text)
    assert len(entries) == razer.razer_tune_table_size()
    seen = set()
    for fam, m, rows, k, *p in [tuple(map(int, e)) for e in entries]:
        assert (fam, m, rows, k) not in seen                        # one entry per key
        seen.add((fam, m, rows, k))
        assert tune.family_of(m, k) == fam
        cands = tune.candidates(fam, m, k)
        assert tuple(p[:len(cands[0])]) in cands, (fam, m, rows, k, p)
        assert all(v == 0 for v in p[len(cands[0]):])
        assert razer.razer_tune_lookup(fam, m, rows, k) == (2, tuple(p))
