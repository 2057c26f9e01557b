"""ctypes binding of the C ABI in include/razer.h.

Same names, same arguments; torch supplies device memory and the current
stream, nothing else.  Every step of the path runs in the library's kernels.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "librazer_hip.so")

WEIGHT, ACT, WEIGHT_F16 = 0, 1, 2
F32, BF16 = 0, 1
OP_QUANTIZE, OP_DEQUANT, OP_LINEAR, OP_LINEAR_W4A4 = 0, 1, 2, 3
GIVEN_TENSOR_SCALE = 1

LAYOUT_CANONICAL, LAYOUT_INTERLEAVED = 0, 1
EXPORTS = ["razer_workspace_bytes", "razer_workspace_bytes_grouped", "razer_prepack_bytes", "razer_prepack", "razer_quantize", "razer_dequant", "razer_linear",
           "razer_linear_grouped", "razer_linear_static", "razer_status_string"]
# measurement utilities (include/razer_probe.h)
PROBE_EXPORTS = ["razer_probe_dispatch_events", "razer_probe_stream_read", "razer_probe_mfma_bf16", "razer_probe_mfma_fp4"]
# launch-shape tuning hooks (include/razer_tune.h)
TUNE_EXPORTS = ["razer_tune_force", "razer_tune_lookup", "razer_tune_table_size"]
TUNE_GEMV, TUNE_GEMV_QUAD, TUNE_SMALL_BATCH, TUNE_GEMM_SLICES = 0, 1, 2, 3


class RazerError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, razer_status_string(status)))


class _Config(ctypes.Structure):
    _fields_ = [("format", ctypes.c_int32), ("sv", ctypes.c_float * 2), ("block", ctypes.c_int32),
                ("layout", ctypes.c_int32)]


class _Tensor(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("tensor_scale", ctypes.c_void_p), ("rows", ctypes.c_int64),
                ("cols", ctypes.c_int64), ("cfg", _Config)]


_lib = None


def lib_path():
    return _LIB_PATH


def load_library():
    """Load the built library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("librazer_hip.so is not built: run `python -m paper_2501_04052_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u32, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                             ctypes.c_size_t)
    L.razer_workspace_bytes.restype = sz
    L.razer_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64]
    L.razer_workspace_bytes_grouped.restype = sz
    L.razer_workspace_bytes_grouped.argtypes = [i32, ctypes.POINTER(i64), i64, i64]
    L.razer_prepack_bytes.restype = sz
    L.razer_prepack_bytes.argtypes = [ctypes.POINTER(_Tensor)]
    L.razer_prepack.restype = ctypes.c_int
    L.razer_prepack.argtypes = [ctypes.POINTER(_Tensor), vp, sz, vp]
    L.razer_quantize.restype = ctypes.c_int
    L.razer_quantize.argtypes = [ctypes.POINTER(_Config), vp, i32, i64, i64, i64, vp, vp, vp, u32,
                                 vp, sz, vp]
    L.razer_dequant.restype = ctypes.c_int
    L.razer_dequant.argtypes = [ctypes.POINTER(_Tensor), vp, i32, i64, vp]
    L.razer_linear.restype = ctypes.c_int
    L.razer_linear.argtypes = [ctypes.POINTER(_Tensor), vp, ctypes.POINTER(_Tensor), i64, vp, i64,
                               vp, sz, vp]
    L.razer_linear_static.restype = ctypes.c_int
    L.razer_linear_static.argtypes = [ctypes.POINTER(_Tensor), vp, ctypes.POINTER(_Tensor), i64, vp, i64, vp]
    L.razer_linear_grouped.restype = ctypes.c_int
    L.razer_linear_grouped.argtypes = [ctypes.POINTER(ctypes.POINTER(_Tensor)), i32, vp, i64,
                                       ctypes.POINTER(vp), ctypes.POINTER(i64), vp, sz, vp]
    L.razer_probe_dispatch_events.restype = None
    L.razer_probe_dispatch_events.argtypes = [vp, vp]
    L.razer_probe_stream_read.restype = ctypes.c_int
    L.razer_probe_stream_read.argtypes = [vp, sz, ctypes.c_int, vp, vp]
    L.razer_probe_mfma_bf16.restype = ctypes.c_int
    L.razer_probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, ctypes.POINTER(ctypes.c_double)]
    L.razer_probe_mfma_fp4.restype = ctypes.c_int
    L.razer_probe_mfma_fp4.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, ctypes.POINTER(ctypes.c_double)]
    L.razer_tune_force.restype = ctypes.c_int
    L.razer_tune_force.argtypes = [ctypes.c_int, ctypes.POINTER(i32)]
    L.razer_tune_lookup.restype = ctypes.c_int
    L.razer_tune_lookup.argtypes = [ctypes.c_int, i64, i64, i64, ctypes.POINTER(i32)]
    L.razer_tune_table_size.restype = ctypes.c_int
    L.razer_tune_table_size.argtypes = []
    L.razer_status_string.restype = ctypes.c_char_p
    L.razer_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def razer_status_string(status):
    return load_library().razer_status_string(int(status)).decode()


def razer_workspace_bytes(op, rows, cols, m=0):
    return int(load_library().razer_workspace_bytes(int(op), int(rows), int(cols), int(m)))


def razer_workspace_bytes_grouped(rows, cols, m):
    arr = (ctypes.c_int64 * len(rows))(*[int(r) for r in rows])
    return int(load_library().razer_workspace_bytes_grouped(len(rows), arr, int(cols), int(m)))


def razer_tune_force(family, shape=None):
    """Force the launch shape of a kernel family for this host thread (shape: up to 4 ints), or clear
    it (shape None; family -1 clears all).  For the tuner and for tests."""
    arr = None
    if shape is not None:
        vals = list(shape) + [0] * (4 - len(shape))
        arr = (ctypes.c_int32 * 4)(*vals)
    st = load_library().razer_tune_force(int(family), arr)
    if st != 0:
        raise RazerError(st, "razer_tune_force")


def razer_tune_lookup(family, m, rows, cols):
    """(source, shape): source 0 = heuristic (shape None), 1 = forced, 2 = built-in table."""
    arr = (ctypes.c_int32 * 4)()
    src = load_library().razer_tune_lookup(int(family), int(m), int(rows), int(cols), arr)
    return src, (tuple(arr) if src else None)


def razer_tune_table_size():
    return int(load_library().razer_tune_table_size())


def razer_probe_dispatch_events(start=None, stop=None):
    """start / stop: torch.cuda.Event(enable_timing=True) that have been recorded once (so that their
    HIP handles exist), or None to switch the recording off."""
    h = lambda e: None if e is None else ctypes.c_void_p(e.cuda_event)
    load_library().razer_probe_dispatch_events(h(start), h(stop))


def razer_probe_stream_read(buf, workgroups, sink):
    st = load_library().razer_probe_stream_read(_ptr(buf), buf.numel() * buf.element_size(), int(workgroups),
                                                _ptr(sink), _stream())
    if st != 0:
        raise RazerError(st, "razer_probe_stream_read")


def razer_probe_mfma_bf16(iters, workgroups, sink):
    """Returns the floating-point operations of the launch."""
    fl = ctypes.c_double()
    st = load_library().razer_probe_mfma_bf16(int(iters), int(workgroups), _ptr(sink), _stream(), ctypes.byref(fl))
    if st != 0:
        raise RazerError(st, "razer_probe_mfma_bf16")
    return fl.value


def razer_probe_mfma_fp4(iters, workgroups, sink):
    """Returns the floating-point operations of the launch."""
    fl = ctypes.c_double()
    st = load_library().razer_probe_mfma_fp4(int(iters), int(workgroups), _ptr(sink), _stream(), ctypes.byref(fl))
    if st != 0:
        raise RazerError(st, "razer_probe_mfma_fp4")
    return fl.value


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _cfg(fmt, sv, block=16, layout=LAYOUT_CANONICAL):
    c = _Config()
    c.format = fmt
    c.sv[0] = float(sv[0])
    c.sv[1] = float(sv[1]) if len(sv) > 1 else 0.0
    c.block = int(block)
    c.layout = int(layout)
    return c


class RazerTensor:
    """A quantized tensor: device buffers + shape + configuration (razer_tensor in the ABI)."""

    def __init__(self, codes, scales, tensor_scale, rows, cols, fmt, sv, block=16, layout=LAYOUT_CANONICAL):
        self.codes, self.scales, self.tensor_scale = codes, scales, tensor_scale
        self.rows, self.cols, self.fmt, self.sv, self.block = int(rows), int(cols), fmt, tuple(sv), int(block)
        self.layout = int(layout)                      # LAYOUT_INTERLEAVED: codes is the packed buffer, scales None

    def c_struct(self):
        t = _Tensor()
        t.codes = self.codes.data_ptr()
        t.scales = None if self.scales is None else self.scales.data_ptr()
        t.tensor_scale = self.tensor_scale.data_ptr()
        t.rows, t.cols = self.rows, self.cols
        t.cfg = _cfg(self.fmt, self.sv, self.block, self.layout)
        return t

    @staticmethod
    def from_host(codes, scales, tensor_scale, fmt, sv, device="cuda"):
        """Upload numpy codes [rows][cols/2], scales [rows][cols/block] and a scalar tensor scale
        (the block size is read off the shapes)."""
        import numpy as np
        rows, cols = codes.shape[0], codes.shape[1] * 2
        block = cols // scales.shape[1] if scales.shape[1] else 16
        scales = np.ascontiguousarray(scales)
        if scales.dtype == np.uint16:                  # WEIGHT_F16: 16-bit scale words travel as int16
            assert fmt == WEIGHT_F16
            scales = scales.view(np.int16)
        return RazerTensor(torch.from_numpy(np.ascontiguousarray(codes)).to(device),
                           torch.from_numpy(scales).to(device),
                           torch.tensor([float(tensor_scale)], dtype=torch.float32, device=device),
                           rows, cols, fmt, sv, block)


def razer_quantize(x, fmt=WEIGHT, sv=(5.0, 8.0), tensor_scale=None, out=None, workspace=None, cols=None, block=16):
    """Encode a 2-D device tensor x (float32 or bfloat16); blocks of 16 run along the last axis.

    tensor_scale: optional 1-element float32 device tensor used as a given (static) scale.
    cols: number of leading columns to encode when x's rows are longer (x.stride(0) is the ld).
    block: elements per scale byte (16, 32, 64 or 128).
    fmt = WEIGHT_F16: blocks of 128 with one 16-bit scale word each (scales is an int16 tensor).
    Returns a RazerTensor whose buffers live on x's device."""
    L = load_library()
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    rows = x.shape[0]
    cols = x.shape[1] if cols is None else cols
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    dev = x.device
    if fmt == WEIGHT_F16:
        block = 128
    if out is None:
        codes = torch.empty((rows, cols // 2), dtype=torch.uint8, device=dev)
        scales = torch.empty((rows, cols // block), dtype=torch.int16 if fmt == WEIGHT_F16 else torch.uint8, device=dev)
        ts = torch.empty(1, dtype=torch.float32, device=dev) if tensor_scale is None else tensor_scale
    else:
        codes, scales, ts = out.codes, out.scales, out.tensor_scale
    flags = 0 if tensor_scale is None else GIVEN_TENSOR_SCALE
    if tensor_scale is not None and ts is not tensor_scale:
        ts.copy_(tensor_scale)
    need = razer_workspace_bytes(OP_QUANTIZE, rows, cols)
    if workspace is None and not flags:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    cfg = _cfg(fmt, sv, block)
    ld = x.stride(0) if rows > 1 else max(x.stride(0), cols)
    st = L.razer_quantize(ctypes.byref(cfg), _ptr(x), dtype, rows, cols, ld, _ptr(codes), _ptr(scales),
                          _ptr(ts), flags, _ptr(workspace), 0 if workspace is None else workspace.numel(),
                          _stream())
    if st != 0:
        raise RazerError(st, "razer_quantize")
    return RazerTensor(codes, scales, ts, rows, cols, fmt, sv, block)


def razer_prepack(t):
    """The weight tensor t (canonical layout, scale bytes, 16-element blocks) in the library's private
    interleaved layout: a RazerTensor whose `codes` is the packed buffer (it shares t's tensor scale)."""
    L = load_library()
    cs = t.c_struct()
    nbytes = int(L.razer_prepack_bytes(ctypes.byref(cs)))
    packed = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=t.codes.device)
    st = L.razer_prepack(ctypes.byref(cs), _ptr(packed), nbytes, _stream())
    if st != 0:
        raise RazerError(st, "razer_prepack")
    return RazerTensor(packed, None, t.tensor_scale, t.rows, t.cols, t.fmt, t.sv, t.block, LAYOUT_INTERLEAVED)


def razer_dequant(t, dtype=torch.float32, out=None):
    """Decode a RazerTensor to float32 or bfloat16 [rows][cols]."""
    L = load_library()
    if out is None:
        out = torch.empty((t.rows, t.cols), dtype=dtype, device=t.codes.device)
    code = {torch.float32: F32, torch.bfloat16: BF16}[out.dtype]
    cs = t.c_struct()
    ld = out.stride(0) if t.rows > 1 else max(out.stride(0), t.cols)
    st = L.razer_dequant(ctypes.byref(cs), _ptr(out), code, ld, _stream())
    if st != 0:
        raise RazerError(st, "razer_dequant")
    return out


def razer_linear(w, a, out=None, workspace=None):
    """Y = A W^T.  w: RazerTensor [N][K] (weight format).  a: bfloat16 [M][K] device tensor
    (W4A16) or a RazerTensor [M][K] in the activation format (W4A4).  Returns bfloat16 [M][N]."""
    L = load_library()
    if isinstance(a, RazerTensor):
        m = a.rows
        a_struct = a.c_struct()
        a_ptr, aq_ptr = None, ctypes.byref(a_struct)
        dev = a.codes.device
    else:
        assert a.is_cuda and a.dtype == torch.bfloat16 and a.dim() == 2 and a.is_contiguous()
        assert a.shape[1] == w.cols
        m = a.shape[0]
        a_ptr, aq_ptr = _ptr(a), None
        dev = a.device
    if out is None:
        out = torch.empty((m, w.rows), dtype=torch.bfloat16, device=dev)
    ws = w.c_struct()
    ld_y = out.stride(0) if m > 1 else max(out.stride(0), w.rows)
    if workspace is None:
        need = razer_workspace_bytes(OP_LINEAR_W4A4 if aq_ptr is not None else OP_LINEAR, w.rows, w.cols, m)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    st = L.razer_linear(ctypes.byref(ws), a_ptr, aq_ptr, m, _ptr(out), ld_y, _ptr(workspace),
                        0 if workspace is None else workspace.numel(), _stream())
    if st != 0:
        raise RazerError(st, "razer_linear")
    return out


def razer_linear_static(w, a, out):
    """razer_linear without a workspace argument and without any allocation: `out` must be given
    (bfloat16 [M][N]); the library's static scratch array holds the K-slices."""
    L = load_library()
    if isinstance(a, RazerTensor):
        m = a.rows
        a_struct = a.c_struct()
        a_ptr, aq_ptr = None, ctypes.byref(a_struct)
    else:
        assert a.is_cuda and a.dtype == torch.bfloat16 and a.dim() == 2 and a.is_contiguous()
        assert a.shape[1] == w.cols
        m = a.shape[0]
        a_ptr, aq_ptr = _ptr(a), None
    assert out.shape == (m, w.rows) and out.dtype == torch.bfloat16
    ws = w.c_struct()
    ld_y = out.stride(0) if m > 1 else max(out.stride(0), w.rows)
    st = L.razer_linear_static(ctypes.byref(ws), a_ptr, aq_ptr, m, _ptr(out), ld_y, _stream())
    if st != 0:
        raise RazerError(st, "razer_linear_static")
    return out


def razer_linear_grouped(ws, a, outs=None):
    """y[i] = A ws[i]^T for up to 4 RazerTensors that share K and the bf16 activation rows a [M][K]
    (fused q/k/v, gate/up): one kernel launch when M <= 4.  Returns the list of bfloat16 outputs."""
    L = load_library()
    assert a.is_cuda and a.dtype == torch.bfloat16 and a.dim() == 2 and a.is_contiguous()
    m, count = a.shape[0], len(ws)
    if outs is None:
        outs = [torch.empty((m, w.rows), dtype=torch.bfloat16, device=a.device) for w in ws]
    structs = [w.c_struct() for w in ws]
    wptrs = (ctypes.POINTER(_Tensor) * count)(*[ctypes.pointer(s) for s in structs])
    yptrs = (ctypes.c_void_p * count)(*[o.data_ptr() for o in outs])
    lds = (ctypes.c_int64 * count)(*[(o.stride(0) if m > 1 else max(o.stride(0), w.rows))
                                     for o, w in zip(outs, ws)])
    need = razer_workspace_bytes_grouped([w.rows for w in ws], ws[0].cols, m)
    workspace = torch.empty(need, dtype=torch.uint8, device=a.device) if need else None
    st = L.razer_linear_grouped(wptrs, count, _ptr(a), m, yptrs, lds, _ptr(workspace), need, _stream())
    if st != 0:
        raise RazerError(st, "razer_linear_grouped")
    return outs


class PreparedCall:
    """The marshalled arguments of one razer_linear / razer_linear_grouped call, kept so that a
    serving loop can re-issue the same call without rebuilding them (the library itself keeps no
    state; this object only holds ctypes values and references to the tensors involved)."""

    def __init__(self, fn, args, keep, where):
        self._fn, self._args, self._keep, self._where = fn, args, keep, where

    def __call__(self, stream=None):
        """Enqueue on `stream` (a HIP stream handle as an int) or on torch's current stream."""
        st = self._fn(*self._args, _stream() if stream is None else ctypes.c_void_p(stream))
        if st != 0:
            raise RazerError(st, self._where)


def prepare_linear(w, a, out, workspace=None):
    """razer_linear(w, a, out=out, workspace=workspace) as a PreparedCall (W4A16, bf16 a)."""
    L = load_library()
    assert a.is_cuda and a.dtype == torch.bfloat16 and a.dim() == 2 and a.is_contiguous() and a.shape[1] == w.cols
    m = a.shape[0]
    assert out.shape == (m, w.rows) and out.dtype == torch.bfloat16
    need = razer_workspace_bytes(OP_LINEAR, w.rows, w.cols, m)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=a.device)
    ws = w.c_struct()
    ld_y = out.stride(0) if m > 1 else max(out.stride(0), w.rows)
    args = (ctypes.byref(ws), _ptr(a), None, m, _ptr(out), ld_y, _ptr(workspace),
            0 if workspace is None else workspace.numel())
    return PreparedCall(L.razer_linear, args, (ws, w, a, out, workspace), "razer_linear")


def prepare_linear_grouped(ws, a, outs):
    """razer_linear_grouped(ws, a, outs=outs) as a PreparedCall."""
    L = load_library()
    assert a.is_cuda and a.dtype == torch.bfloat16 and a.dim() == 2 and a.is_contiguous()
    m, count = a.shape[0], len(ws)
    structs = [w.c_struct() for w in ws]
    wptrs = (ctypes.POINTER(_Tensor) * count)(*[ctypes.pointer(s) for s in structs])
    yptrs = (ctypes.c_void_p * count)(*[o.data_ptr() for o in outs])
    lds = (ctypes.c_int64 * count)(*[(o.stride(0) if m > 1 else max(o.stride(0), w.rows))
                                     for o, w in zip(outs, ws)])
    need = razer_workspace_bytes_grouped([w.rows for w in ws], ws[0].cols, m)
    workspace = torch.empty(need, dtype=torch.uint8, device=a.device) if need else None
    args = (wptrs, count, _ptr(a), m, yptrs, lds, _ptr(workspace), need)
    return PreparedCall(L.razer_linear_grouped, args, (structs, ws, a, outs, workspace), "razer_linear_grouped")
