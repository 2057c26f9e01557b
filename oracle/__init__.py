"""ctypes access to the RaZeR CPU oracle (``razer_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg import this package.  It never touches the
HIP library and the HIP library never touches it.

All arrays are host numpy arrays; bf16 data travels as ``uint16`` bit
patterns.  Formats: ``WEIGHT`` (E3M3 block scale + 2 metadata bits, special
values +-sv0, +-sv1) and ``ACT`` (E4M3 block scale + 1 metadata bit, special
values +-sv0), Sec. 4.1-4.2 of the paper.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "razer_oracle.c")
_LIB = os.path.join(_HERE, "librazer_oracle.so")

WEIGHT, ACT, WEIGHT_F16 = 0, 1, 2      # WEIGHT_F16: blocks of 128, one FP16 scale word (Sec. 4.3 kernel format)
REMAP_CODE = 0x8
BLOCK = 16


def build(force=False):
    """Compile the oracle with gcc (plain -O2, no contraction, no fast-math)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        L = _lib
        d, i, i64, f, vp = (ctypes.c_double, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                            ctypes.c_void_p)
        L.oracle_fp4_value.restype = d; L.oracle_fp4_value.argtypes = [i]
        L.oracle_e4m3_value.restype = d; L.oracle_e4m3_value.argtypes = [i]
        L.oracle_e3m3_value.restype = d; L.oracle_e3m3_value.argtypes = [i]
        L.oracle_e4m10_value.restype = d; L.oracle_e4m10_value.argtypes = [i]
        L.oracle_scale_value.restype = d; L.oracle_scale_value.argtypes = [i, i]
        L.oracle_scale_max.restype = d; L.oracle_scale_max.argtypes = [i]
        L.oracle_round_scale.restype = i; L.oracle_round_scale.argtypes = [i, f]
        L.oracle_sv_from_offset_reg.restype = d; L.oracle_sv_from_offset_reg.argtypes = [i]
        L.oracle_offset_reg_from_sv.restype = i; L.oracle_offset_reg_from_sv.argtypes = [d]
        L.oracle_candidate.restype = d; L.oracle_candidate.argtypes = [i, d, d, i]
        L.oracle_element_value.restype = d; L.oracle_element_value.argtypes = [i, d, d, i, i]
        L.oracle_round_fp4.restype = i; L.oracle_round_fp4.argtypes = [f]
        L.oracle_round_fp4_sv.restype = i
        L.oracle_round_fp4_sv.argtypes = [f, d, ctypes.POINTER(d)]
        L.oracle_f64_to_bf16.restype = ctypes.c_uint16; L.oracle_f64_to_bf16.argtypes = [d]
        L.oracle_tensor_scale.restype = f; L.oracle_tensor_scale.argtypes = [i, vp, i, i64]
        L.oracle_quantize.restype = i
        L.oracle_quantize.argtypes = [i, d, d, i, vp, i, i64, i64, i, vp, vp, vp, i, vp]
        L.oracle_dequant.restype = i
        L.oracle_dequant.argtypes = [i, d, d, vp, vp, f, i64, i64, i, vp, vp, vp]
        L.oracle_linear.restype = i
        L.oracle_linear.argtypes = [i, d, d, vp, vp, f, i64, i64, i, vp, d, vp, vp, f, i, i64,
                                    vp, i64, vp, i64, vp, vp]
        L.oracle_two_pass_split.restype = i
        L.oracle_two_pass_split.argtypes = [i, i, i, ctypes.POINTER(i), ctypes.POINTER(i),
                                            ctypes.POINTER(i)]
    return _lib


def set_threads(n):
    """Number of OpenMP threads the oracle's row loops use from now on (timing only)."""
    lib()
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


# ---- scalar helpers ---------------------------------------------------------
def fp4_value(code): return lib().oracle_fp4_value(int(code))
def e4m3_value(code): return lib().oracle_e4m3_value(int(code))
def e3m3_value(code): return lib().oracle_e3m3_value(int(code))
def e4m10_value(code): return lib().oracle_e4m10_value(int(code))
def scale_value(fmt, code): return lib().oracle_scale_value(fmt, int(code))
def scale_max(fmt): return lib().oracle_scale_max(fmt)
def round_scale(fmt, t): return lib().oracle_round_scale(fmt, float(np.float32(t)))
def sv_from_offset_reg(reg): return lib().oracle_sv_from_offset_reg(int(reg))
def offset_reg_from_sv(mag): return lib().oracle_offset_reg_from_sv(float(mag))
def candidate(fmt, sv0, sv1, meta): return lib().oracle_candidate(fmt, sv0, sv1, int(meta))
def element_value(fmt, sv0, sv1, code, meta):
    return lib().oracle_element_value(fmt, sv0, sv1, int(code), int(meta))
def round_fp4(xs): return lib().oracle_round_fp4(float(np.float32(xs)))


def round_fp4_sv(xs, v):
    err = ctypes.c_double()
    c = lib().oracle_round_fp4_sv(float(np.float32(xs)), float(v), ctypes.byref(err))
    return c, err.value


def f64_to_bf16(x): return lib().oracle_f64_to_bf16(float(x))


def two_pass_split(code, meta, main_mag_code, comp_mag_codes):
    arr = (ctypes.c_int * 2)(*comp_mag_codes)
    bm, bc = ctypes.c_int(), ctypes.c_int()
    lib().oracle_two_pass_split(int(code), int(meta), int(main_mag_code), arr,
                                ctypes.byref(bm), ctypes.byref(bc))
    return bm.value, bc.value


# ---- tensor functions --------------------------------------------------------
def tensor_scale(fmt, x):
    x = np.ascontiguousarray(x)
    is_bf16 = x.dtype == np.uint16
    assert is_bf16 or x.dtype == np.float32
    return float(lib().oracle_tensor_scale(fmt, _p(x), int(is_bf16), x.size))


def quantize(fmt, x, sv=(5.0, 8.0), nsv=-1, given_tensor_scale=None, want_sse=False, block=BLOCK):
    """Encode x [rows][cols] (float32, or uint16 holding bf16).

    Returns (codes u8 [rows][cols/2], scales u8 [rows][cols/block], tensor_scale
    float32 scalar[, block_sse f64 [rows][cols/block]]).  nsv=0 -> plain NVFP4
    under the same block-scale format.  block: 16 (the evaluated format), 32, 64 or 128.
    fmt = WEIGHT_F16: blocks of 128, scales are uint16 words (little-endian in memory)."""
    x = np.ascontiguousarray(x)
    is_bf16 = x.dtype == np.uint16
    assert is_bf16 or x.dtype == np.float32
    rows, cols = x.shape
    if fmt == WEIGHT_F16:
        block = 128
    codes = np.empty((rows, cols // 2), np.uint8)
    scales = np.empty((rows, cols // block), np.uint16 if fmt == WEIGHT_F16 else np.uint8)
    ts = np.zeros(1, np.float32)
    if given_tensor_scale is not None:
        ts[0] = given_tensor_scale
    sse = np.empty((rows, cols // block), np.float64) if want_sse else None
    rc = lib().oracle_quantize(fmt, float(sv[0]), float(sv[1]), int(nsv), _p(x), int(is_bf16),
                               rows, cols, int(block), _p(codes), _p(scales), _p(ts),
                               int(given_tensor_scale is not None), _p(sse))
    if rc != 0:
        raise ValueError("oracle_quantize: bad shape")
    return (codes, scales, np.float32(ts[0]), sse) if want_sse else (codes, scales, np.float32(ts[0]))


def dequant(fmt, codes, scales, ts, sv=(5.0, 8.0), want=("f32",)):
    """Decode to any of 'f32', 'bf16' (uint16 bits), 'sq' (f64 scale*element).
    The block size is read off the shapes: cols / scales.shape[1]."""
    codes = _c(codes, np.uint8); scales = _c(scales, np.uint16 if fmt == WEIGHT_F16 else np.uint8)
    rows, half = codes.shape
    cols = half * 2
    block = cols // scales.shape[1] if scales.shape[1] else BLOCK
    out = {}
    f32 = np.empty((rows, cols), np.float32) if "f32" in want else None
    b16 = np.empty((rows, cols), np.uint16) if "bf16" in want else None
    sq = np.empty((rows, cols), np.float64) if "sq" in want else None
    rc = lib().oracle_dequant(fmt, float(sv[0]), float(sv[1]), _p(codes), _p(scales), float(ts),
                              rows, cols, int(block), _p(f32), _p(b16), _p(sq))
    if rc != 0:
        raise ValueError("oracle_dequant: bad shape")
    for k, v in (("f32", f32), ("bf16", b16), ("sq", sq)):
        if v is not None:
            out[k] = v
    return out


def linear(w, a_bf16=None, a_q=None, w_sv=(5.0, 8.0), a_sv0=5.0, rows=None, cols=None):
    """Y = A W^T.  w = (codes, scales, ts) in the weight format; exactly one of
    a_bf16 (uint16 [m][k]) and a_q = (codes, scales, ts) in the activation
    format.  rows / cols: optional int64 index arrays selecting the output
    rows (of M) and columns (of N) to compute.  Block sizes are read off the
    shapes of the scale arrays.  Returns (y_f64, y_bf16)."""
    wc, ws, wts = w
    wc = _c(wc, np.uint8)
    w_fmt = WEIGHT_F16 if np.asarray(ws).dtype == np.uint16 else WEIGHT     # the scale words tell the format
    ws = _c(ws, np.uint16 if w_fmt == WEIGHT_F16 else np.uint8)
    n, k = wc.shape[0], wc.shape[1] * 2
    ac = asc = ab = None
    ats = 0.0
    w_block = k // ws.shape[1] if ws.shape[1] else BLOCK
    a_block = BLOCK
    if a_bf16 is not None:
        ab = _c(a_bf16, np.uint16); m = ab.shape[0]; assert ab.shape[1] == k
    else:
        ac, asc, ats = a_q
        ac = _c(ac, np.uint8); asc = _c(asc, np.uint8); m = ac.shape[0]
        assert ac.shape[1] * 2 == k
        a_block = k // asc.shape[1] if asc.shape[1] else BLOCK
    rs = None if rows is None else np.ascontiguousarray(rows, np.int64)
    cs = None if cols is None else np.ascontiguousarray(cols, np.int64)
    mm = m if rs is None else rs.size
    nn = n if cs is None else cs.size
    y64 = np.empty((mm, nn), np.float64)
    y16 = np.empty((mm, nn), np.uint16)
    rc = lib().oracle_linear(w_fmt, float(w_sv[0]), float(w_sv[1]), _p(wc), _p(ws), float(wts), n, k, int(w_block),
                             _p(ab), float(a_sv0), _p(ac), _p(asc), float(ats), int(a_block), m,
                             _p(rs), mm, _p(cs), nn, _p(y64), _p(y16))
    if rc != 0:
        raise ValueError("oracle_linear: bad arguments")
    return y64, y16
