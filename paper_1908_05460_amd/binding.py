"""ctypes binding of libwgrad.so (declared in include/wgrad.h).

Argument marshalling only: every function takes torch tensors that already live
on the GPU (torch is used for device memory and streams), checks shapes and
dtypes, passes raw device pointers and the current HIP stream to the C ABI, and
raises on a non-zero status.  No arithmetic happens here and there is no CPU
fallback: if the library has not been built, ``load()`` raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwgrad.so")

EXACT, APPROX, ZERO, RANDOM = 0, 1, 2, 3
F32, BF16 = 0, 1
OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, LAUNCH_FAILED, SCRATCH_LIMIT = 0, -1, -2, -3, -4, -5

EXPORTS = ("conv_wgrad_exact", "conv_wgrad_approx", "conv_wgrad_select", "conv_wgrad_zero",
           "conv_wgrad_random", "conv_wgrad_workspace_bytes", "conv_wgrad_schedule_run",
           "conv_wgrad_schedule_workspace_bytes", "conv_wgrad_status_string",
           "conv_wgrad_approx_topk", "conv_wgrad_topk_workspace_bytes",
           "conv_wgrad_approx_nhwc", "conv_wgrad_exact_nhwc", "conv_wgrad_nhwc_workspace_bytes",
           "conv_wgrad_transpose_x", "conv_wgrad_permute_dw",
           "conv_wgrad_schedule_run_topk", "conv_wgrad_schedule_topk_workspace_bytes",
           "conv_wgrad_approx_static")
STATIC_SCRATCH_BYTES = 24 << 20
DW_OIHW, DW_OHWI, DW_HWIO = 0, 1, 2


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")]

    @property
    def Ho(self):
        return (self.H + 2 * self.pad_h - self.R) // self.stride_h + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad_w - self.S) // self.stride_w + 1


class WgradError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def _bind_hip_runtime():
    """libwgrad.so carries no dependency on a HIP runtime of its own: it must use the one
    PyTorch allocates memory and creates streams with.  Make that runtime's symbols visible
    (PyTorch wheels bundle libamdhip64.so under torch/lib; otherwise the system one)."""
    import torch
    bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    for cand in (bundled, "libamdhip64.so", "/opt/rocm/lib/libamdhip64.so"):
        try:
            ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)
            return
        except OSError:
            continue
    raise RuntimeError("no HIP runtime (libamdhip64.so) found for libwgrad.so to bind to")


def load():
    """Load libwgrad.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                           "(python -m paper_1908_05460_amd.build)")
    _bind_hip_runtime()
    L = ctypes.CDLL(LIB_PATH)
    P, vp, i32p, fp = ctypes.POINTER, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    L.conv_wgrad_exact.argtypes = [P(ConvDesc), vp, vp, fp, vp, ctypes.c_size_t, vp]
    L.conv_wgrad_approx.argtypes = [P(ConvDesc), vp, vp, fp, ctypes.c_float, i32p, fp, vp,
                                    ctypes.c_size_t, vp]
    L.conv_wgrad_approx_static.argtypes = [P(ConvDesc), vp, vp, fp, ctypes.c_float, i32p, fp, vp]
    L.conv_wgrad_approx_topk.argtypes = [P(ConvDesc), vp, vp, fp, ctypes.c_int, ctypes.c_float, i32p, fp, vp,
                                         ctypes.c_size_t, vp]
    L.conv_wgrad_topk_workspace_bytes.argtypes = [P(ConvDesc), ctypes.c_int]
    L.conv_wgrad_topk_workspace_bytes.restype = ctypes.c_size_t
    L.conv_wgrad_approx_nhwc.argtypes = [P(ConvDesc), vp, vp, fp, ctypes.c_int, ctypes.c_float, i32p, fp, vp,
                                         ctypes.c_size_t, vp]
    L.conv_wgrad_exact_nhwc.argtypes = [P(ConvDesc), vp, vp, fp, ctypes.c_int, vp, ctypes.c_size_t, vp]
    L.conv_wgrad_nhwc_workspace_bytes.argtypes = [P(ConvDesc), ctypes.c_int]
    L.conv_wgrad_nhwc_workspace_bytes.restype = ctypes.c_size_t
    L.conv_wgrad_transpose_x.argtypes = [P(ConvDesc), ctypes.c_int, vp, vp, vp]
    L.conv_wgrad_permute_dw.argtypes = [P(ConvDesc), ctypes.c_int, ctypes.c_int, fp, fp, vp]
    L.conv_wgrad_select.argtypes = [P(ConvDesc), vp, i32p, fp, vp]
    L.conv_wgrad_zero.argtypes = [P(ConvDesc), fp, vp]
    L.conv_wgrad_random.argtypes = [P(ConvDesc), fp, ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64, vp]
    L.conv_wgrad_workspace_bytes.argtypes = [P(ConvDesc), ctypes.c_int]
    L.conv_wgrad_workspace_bytes.restype = ctypes.c_size_t
    L.conv_wgrad_schedule_run.argtypes = [P(ConvDesc), P(vp), P(vp), P(vp), P(ctypes.c_uint8),
                                          ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                          ctypes.c_uint64, ctypes.c_uint64, vp, ctypes.c_size_t, vp]
    L.conv_wgrad_schedule_workspace_bytes.argtypes = [P(ConvDesc), P(ctypes.c_uint8), ctypes.c_int32]
    L.conv_wgrad_schedule_workspace_bytes.restype = ctypes.c_size_t
    L.conv_wgrad_schedule_run_topk.argtypes = [P(ConvDesc), P(vp), P(vp), P(vp), P(ctypes.c_uint8),
                                               ctypes.c_int32, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                               ctypes.c_uint64, ctypes.c_uint64, vp, ctypes.c_size_t, vp]
    L.conv_wgrad_schedule_run_topk.restype = ctypes.c_int
    L.conv_wgrad_schedule_topk_workspace_bytes.argtypes = [P(ConvDesc), P(ctypes.c_uint8), ctypes.c_int32, ctypes.c_int32]
    L.conv_wgrad_schedule_topk_workspace_bytes.restype = ctypes.c_size_t
    L.conv_wgrad_status_string.argtypes = [ctypes.c_int]
    L.conv_wgrad_status_string.restype = ctypes.c_char_p
    for f in ("conv_wgrad_exact", "conv_wgrad_approx", "conv_wgrad_select", "conv_wgrad_zero",
              "conv_wgrad_random", "conv_wgrad_schedule_run", "conv_wgrad_approx_topk",
              "conv_wgrad_approx_nhwc", "conv_wgrad_exact_nhwc", "conv_wgrad_transpose_x", "conv_wgrad_permute_dw"):
        getattr(L, f).restype = ctypes.c_int
    _lib = L
    return L


def status_string(status):
    return load().conv_wgrad_status_string(int(status)).decode()


def desc(N, C, H, W, K, R=3, S=3, stride=1, pad=1, dtype=F32, stride_w=None, pad_w=None):
    return ConvDesc(N, C, H, W, K, R, S, stride, stride if stride_w is None else stride_w,
                    pad, pad if pad_w is None else pad_w, dtype)


def desc_for(layer, N, dtype="fp32"):
    """Descriptor of a paper_1908_05460_amd.inputs.Layer."""
    return desc(N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad,
                BF16 if dtype == "bf16" else F32)


def workspace_bytes(d, method):
    return load().conv_wgrad_workspace_bytes(ctypes.byref(d), int(method))


# ---- torch marshalling ---------------------------------------------------------------

def _torch():
    import torch
    return torch


def _stream():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else None)


def _check_inputs(d, X, dY):
    torch = _torch()
    want = torch.bfloat16 if d.dtype == BF16 else torch.float32
    for name, t, shp in (("X", X, (d.N, d.C, d.H, d.W)), ("dY", dY, (d.N, d.K, d.Ho, d.Wo))):
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous() or t.dtype != want or tuple(t.shape) != shp:
            raise ValueError(f"{name}: need a contiguous {want} GPU tensor of shape {shp}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")


def alloc_workspace(nbytes, device="cuda"):
    """A 256-byte aligned device buffer (torch's allocator aligns to 512)."""
    torch = _torch()
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _ws_args(ws):
    if ws is None:
        return ctypes.c_void_p(None), 0
    return _ptr(ws), ws.numel() * ws.element_size()


def _new_dW(d, like):
    torch = _torch()
    return torch.empty((d.K, d.C, d.R, d.S), dtype=torch.float32, device=like.device)


def conv_wgrad_exact(d, X, dY, dW=None, ws=None):
    _check_inputs(d, X, dY)
    dW = _new_dW(d, X) if dW is None else dW
    if ws is None:
        ws = alloc_workspace(workspace_bytes(d, EXACT), X.device)
    p, n = _ws_args(ws)
    rc = load().conv_wgrad_exact(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), p, n, _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_exact")
    return dW


def conv_wgrad_approx(d, X, dY, scale=1.0, dW=None, idx_out=None, sum_out=None, ws=None):
    _check_inputs(d, X, dY)
    dW = _new_dW(d, X) if dW is None else dW
    if ws is None:
        ws = alloc_workspace(workspace_bytes(d, APPROX), X.device)
    p, n = _ws_args(ws)
    rc = load().conv_wgrad_approx(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), float(scale),
                                  _ptr(idx_out), _ptr(sum_out), p, n, _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_approx")
    return dW


def topk_workspace_bytes(d, k):
    return load().conv_wgrad_topk_workspace_bytes(ctypes.byref(d), int(k))


def conv_wgrad_approx_static(d, X, dY, scale=1.0, dW=None, idx_out=None, sum_out=None):
    """conv_wgrad_approx on the library's static scratch buffer: no workspace is passed or allocated."""
    _check_inputs(d, X, dY)
    dW = _new_dW(d, X) if dW is None else dW
    rc = load().conv_wgrad_approx_static(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), float(scale),
                                         _ptr(idx_out), _ptr(sum_out), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_approx_static")
    return dW


def conv_wgrad_approx_topk(d, X, dY, k, scale=1.0, dW=None, idx_out=None, sum_out=None, ws=None):
    _check_inputs(d, X, dY)
    dW = _new_dW(d, X) if dW is None else dW
    if ws is None:
        ws = alloc_workspace(topk_workspace_bytes(d, k), X.device)
    p, n = _ws_args(ws)
    rc = load().conv_wgrad_approx_topk(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), int(k), float(scale),
                                       _ptr(idx_out), _ptr(sum_out), p, n, _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_approx_topk")
    return dW


# ---- channel-last input, other filter-gradient layouts ----

def dw_shape(d, layout):
    return {DW_OIHW: (d.K, d.C, d.R, d.S), DW_OHWI: (d.K, d.R, d.S, d.C), DW_HWIO: (d.R, d.S, d.C, d.K)}[layout]


def _check_nhwc(d, X, dY):
    torch = _torch()
    want = torch.bfloat16 if d.dtype == BF16 else torch.float32
    if not X.is_cuda or not X.is_contiguous() or X.dtype != want or tuple(X.shape) != (d.N, d.H, d.W, d.C):
        raise ValueError(f"X: need a contiguous {want} GPU tensor of shape {(d.N, d.H, d.W, d.C)}, "
                         f"got {X.dtype} {tuple(X.shape)}")
    _check_inputs(d, None, dY)


def nhwc_workspace_bytes(d, method):
    return load().conv_wgrad_nhwc_workspace_bytes(ctypes.byref(d), int(method))


def conv_wgrad_approx_nhwc(d, X, dY, dw_layout=DW_OHWI, scale=1.0, dW=None, idx_out=None, sum_out=None, ws=None):
    torch = _torch()
    _check_nhwc(d, X, dY)
    dW = torch.empty(dw_shape(d, dw_layout), dtype=torch.float32, device=X.device) if dW is None else dW
    if ws is None:
        ws = alloc_workspace(nhwc_workspace_bytes(d, APPROX), X.device)
    p, n = _ws_args(ws)
    rc = load().conv_wgrad_approx_nhwc(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), int(dw_layout), float(scale),
                                       _ptr(idx_out), _ptr(sum_out), p, n, _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_approx_nhwc")
    return dW


def conv_wgrad_exact_nhwc(d, X, dY, dw_layout=DW_OHWI, dW=None, ws=None):
    torch = _torch()
    _check_nhwc(d, X, dY)
    dW = torch.empty(dw_shape(d, dw_layout), dtype=torch.float32, device=X.device) if dW is None else dW
    if ws is None:
        ws = alloc_workspace(nhwc_workspace_bytes(d, EXACT), X.device)
    p, n = _ws_args(ws)
    rc = load().conv_wgrad_exact_nhwc(ctypes.byref(d), _ptr(X), _ptr(dY), _ptr(dW), int(dw_layout), p, n, _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_exact_nhwc")
    return dW


def conv_wgrad_transpose_x(d, X, to_nhwc, out=None):
    torch = _torch()
    shp = (d.N, d.H, d.W, d.C) if to_nhwc else (d.N, d.C, d.H, d.W)
    out = torch.empty(shp, dtype=X.dtype, device=X.device) if out is None else out
    if X.numel() != d.N * d.C * d.H * d.W or not X.is_contiguous() or not out.is_contiguous() or out.dtype != X.dtype \
            or X.dtype != (torch.bfloat16 if d.dtype == BF16 else torch.float32):
        raise ValueError("transpose_x: contiguous tensors of the descriptor's size and element type are needed")
    rc = load().conv_wgrad_transpose_x(ctypes.byref(d), int(bool(to_nhwc)), _ptr(X), _ptr(out), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_transpose_x")
    return out


def conv_wgrad_permute_dw(d, dW, src_layout, dst_layout, out=None):
    torch = _torch()
    out = torch.empty(dw_shape(d, dst_layout), dtype=torch.float32, device=dW.device) if out is None else out
    if tuple(dW.shape) != dw_shape(d, src_layout) or dW.dtype != torch.float32 or not dW.is_contiguous():
        raise ValueError(f"permute_dw: need a contiguous float32 tensor of shape {dw_shape(d, src_layout)}")
    rc = load().conv_wgrad_permute_dw(ctypes.byref(d), int(src_layout), int(dst_layout), _ptr(dW), _ptr(out), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_permute_dw")
    return out


def conv_wgrad_select(d, dY, idx=None, sums=None):
    torch = _torch()
    _check_inputs(d, None, dY)
    idx = torch.empty((d.N, d.K), dtype=torch.int32, device=dY.device) if idx is None else idx
    sums = torch.empty((d.N, d.K), dtype=torch.float32, device=dY.device) if sums is None else sums
    rc = load().conv_wgrad_select(ctypes.byref(d), _ptr(dY), _ptr(idx), _ptr(sums), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_select")
    return idx, sums


def conv_wgrad_zero(d, dW):
    rc = load().conv_wgrad_zero(ctypes.byref(d), _ptr(dW), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_zero")
    return dW


def conv_wgrad_random(d, dW, sigma, seed, offset):
    rc = load().conv_wgrad_random(ctypes.byref(d), _ptr(dW), float(sigma), int(seed), int(offset), _stream())
    if rc != OK:
        raise WgradError(rc, "conv_wgrad_random")
    return dW


class Schedule:
    """Host-side tables for conv_wgrad_schedule_run over a fixed stack of layers."""

    def __init__(self, descs, Xs, dYs, dWs):
        n = len(descs)
        self.n = n
        self.descs = (ConvDesc * n)(*descs)
        self.X = (ctypes.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in Xs])
        self.dY = (ctypes.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in dYs])
        self.dW = (ctypes.c_void_p * n)(*[t.data_ptr() for t in dWs])
        self._keep = (Xs, dYs, dWs)

    def workspace_bytes(self, methods):
        m = (ctypes.c_uint8 * self.n)(*[int(x) for x in methods])
        return load().conv_wgrad_schedule_workspace_bytes(self.descs, m, self.n)

    def workspace_bytes_topk(self, methods, topk):
        m = (ctypes.c_uint8 * self.n)(*[int(x) for x in methods])
        return load().conv_wgrad_schedule_topk_workspace_bytes(self.descs, m, self.n, int(topk))

    def run_topk(self, methods, topk, ws, scale=1.0, sigma=1.0 / 128, seed=0, offset=0):
        m = (ctypes.c_uint8 * self.n)(*[int(x) for x in methods])
        p, nbytes = _ws_args(ws)
        rc = load().conv_wgrad_schedule_run_topk(self.descs, self.X, self.dY, self.dW, m, self.n, int(topk),
                                                 float(scale), float(sigma), int(seed), int(offset),
                                                 p, nbytes, _stream())
        if rc != OK:
            raise WgradError(rc, "conv_wgrad_schedule_run_topk")

    def run(self, methods, ws, scale=1.0, sigma=1.0 / 128, seed=0, offset=0):
        m = (ctypes.c_uint8 * self.n)(*[int(x) for x in methods])
        p, nbytes = _ws_args(ws)
        rc = load().conv_wgrad_schedule_run(self.descs, self.X, self.dY, self.dW, m, self.n,
                                            float(scale), float(sigma), int(seed), int(offset),
                                            p, nbytes, _stream())
        if rc != OK:
            raise WgradError(rc, "conv_wgrad_schedule_run")
