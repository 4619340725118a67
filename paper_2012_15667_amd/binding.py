"""Thin ctypes binding of libiolbconv.so: argument marshalling only.

Every step of the convolution runs in the library's HIP kernels; torch is used for device
memory and the current stream.  There is no CPU fallback: a missing library raises.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libiolbconv.so")

DIRECT, WINO_F2, WINO_F4, WINO_F3, WINO_F6 = 0, 1, 2, 3, 4
WINO_ALGO = {2: WINO_F2, 3: WINO_F3, 4: WINO_F4, 6: WINO_F6}     # algo id of F(m x m, 3 x 3)
PATH_FMA, PATH_MFMA, PATH_FUSED, PATH_POINT = 0, 1, 2, 3
LAYOUT_CHW, LAYOUT_HWC, LAYOUT_CWH = 0, 1, 2

EXPORTS = ["conv_direct", "conv_direct_noalloc", "conv_direct_noalloc_max_weight_floats", "conv_direct_cfg", "conv_direct_layout", "conv_direct_pad2", "conv_winograd", "conv_winograd_pad", "conv_winograd_workspace_bytes",
           "conv_winograd_ws", "conv_winograd_kernel_bytes", "conv_winograd_transform_kernels", "conv_winograd_pre",
           "iolb_tune", "iolb_tune_bound", "iolb_enumerate", "iolb_bounds", "iolb_winograd_matrices", "iolb_set_stream",
           "iolb_probe_hbm_copy", "iolb_probe_mfma_sink_bytes", "iolb_probe_mfma_f32",
           "iolb_probe_share_scratch_bytes", "iolb_probe_pipeline_share",
           "iolb_timing_enable", "iolb_timing_read", "iolb_release_workspace", "iolb_strerror",
           "iolb_last_hip_error"]


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "algo")]


class TileConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("b", "x", "y", "z", "alpha", "threads", "waves_m", "waves_n",
                                              "path", "wt_mode", "lds_bytes_used", "acc_regs_per_thread")] + \
               [("q_read_elems", ctypes.c_int64), ("q_write_elems", ctypes.c_int64)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}

    @classmethod
    def from_dict(cls, d):
        return cls(**{n: int(d[n]) for n, _ in cls._fields_})


class BoundsOut(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("Q", ctypes.c_int32), ("vertices", ctypes.c_int64),
                ("compulsory_elems", ctypes.c_int64), ("q_write_elems", ctypes.c_int64),
                ("t_bound_2s", ctypes.c_double), ("q_lower_lead", ctypes.c_double),
                ("q_lower_explicit", ctypes.c_double), ("q_dataflow", ctypes.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class IolbError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("iolbconv error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """The loaded library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libiolbconv.so is missing: run __graft_entry__.build() "
                               "(python -m paper_2012_15667_amd.build) first")
        L = ctypes.CDLL(LIB_PATH)
        i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.conv_direct.restype = i
        L.conv_direct.argtypes = [vp, vp, vp] + [i] * 9
        L.conv_direct_noalloc.restype = i
        L.conv_direct_noalloc.argtypes = [vp, vp, vp] + [i] * 9
        L.conv_direct_noalloc_max_weight_floats.restype = sz
        L.conv_direct_noalloc_max_weight_floats.argtypes = []
        L.conv_direct_cfg.restype = i
        L.conv_direct_cfg.argtypes = [vp, vp, vp] + [i] * 9 + [ctypes.POINTER(TileConfig)]
        L.conv_direct_pad2.restype = i
        L.conv_direct_pad2.argtypes = [vp, vp, vp] + [i] * 10
        L.conv_direct_layout.restype = i
        L.conv_direct_layout.argtypes = [vp, vp, vp] + [i] * 10 + [ctypes.POINTER(TileConfig)]
        L.conv_winograd.restype = i
        L.conv_winograd.argtypes = [vp, vp, vp] + [i] * 6
        L.conv_winograd_pad.restype = i
        L.conv_winograd_pad.argtypes = [vp, vp, vp] + [i] * 7
        L.conv_winograd_workspace_bytes.restype = sz
        L.conv_winograd_workspace_bytes.argtypes = [i] * 6
        L.conv_winograd_ws.restype = i
        L.conv_winograd_ws.argtypes = [vp, vp, vp] + [i] * 6 + [vp, sz, ctypes.POINTER(TileConfig)]
        L.conv_winograd_kernel_bytes.restype = sz
        L.conv_winograd_kernel_bytes.argtypes = [i] * 3
        L.conv_winograd_transform_kernels.restype = i
        L.conv_winograd_transform_kernels.argtypes = [vp, vp] + [i] * 3
        L.conv_winograd_pre.restype = i
        L.conv_winograd_pre.argtypes = [vp, vp, vp] + [i] * 6 + [vp, sz, ctypes.POINTER(TileConfig)]
        L.iolb_tune.restype = i
        L.iolb_tune.argtypes = [ctypes.POINTER(Shape), sz, i, ctypes.POINTER(TileConfig)]
        L.iolb_tune_bound.restype = i
        L.iolb_tune_bound.argtypes = [ctypes.POINTER(Shape), sz, i, ctypes.POINTER(TileConfig)]
        L.iolb_enumerate.restype = ctypes.c_int64
        L.iolb_enumerate.argtypes = [ctypes.POINTER(Shape), sz, i, i, ctypes.POINTER(TileConfig), ctypes.c_int64]
        L.iolb_bounds.restype = i
        L.iolb_bounds.argtypes = [ctypes.POINTER(Shape), ctypes.c_int64, ctypes.POINTER(BoundsOut)]
        L.iolb_winograd_matrices.restype = i
        L.iolb_winograd_matrices.argtypes = [i, vp, vp, vp]
        L.iolb_set_stream.restype = i
        L.iolb_set_stream.argtypes = [vp]
        L.iolb_timing_enable.restype = i
        L.iolb_timing_enable.argtypes = [i]
        L.iolb_timing_read.restype = i
        L.iolb_timing_read.argtypes = [i, ctypes.POINTER(i), ctypes.POINTER(ctypes.c_float)]
        L.iolb_probe_hbm_copy.restype = i
        L.iolb_probe_hbm_copy.argtypes = [vp, vp, sz, i, ctypes.POINTER(ctypes.c_float)]
        L.iolb_probe_mfma_sink_bytes.restype = sz
        L.iolb_probe_mfma_sink_bytes.argtypes = []
        L.iolb_probe_mfma_f32.restype = i
        L.iolb_probe_mfma_f32.argtypes = [vp, i, i, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
        L.iolb_probe_share_scratch_bytes.restype = sz
        L.iolb_probe_share_scratch_bytes.argtypes = []
        L.iolb_probe_pipeline_share.restype = i
        L.iolb_probe_pipeline_share.argtypes = [vp, i, ctypes.POINTER(ctypes.c_int), i, ctypes.POINTER(ctypes.c_float),
                                                ctypes.POINTER(ctypes.c_double)]
        L.iolb_release_workspace.restype = i
        L.iolb_release_workspace.argtypes = []
        L.iolb_strerror.restype = ctypes.c_char_p
        L.iolb_strerror.argtypes = [i]
        L.iolb_last_hip_error.restype = ctypes.c_char_p
        L.iolb_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _check(code):
    if code < 0:
        L = lib()
        text = L.iolb_strerror(int(code)).decode()
        if code == -5:
            text += ": " + L.iolb_last_hip_error().decode()
        raise IolbError(int(code), text)
    return code


def make_shape(N, C, H, W, K, R=3, S=3, stride=1, pad=1, algo=DIRECT):
    return Shape(N, C, H, W, K, R, S, stride, pad, algo)


def iolb_tune(shape, lds_bytes=0, vgpr_budget=0):
    """Tile the analytical tuner picks for `shape` (a Shape); returns a dict."""
    out = TileConfig()
    _check(lib().iolb_tune(ctypes.byref(shape), lds_bytes, vgpr_budget, ctypes.byref(out)))
    return out.as_dict()


def iolb_tune_bound(shape, lds_bytes=0, vgpr_budget=0):
    """Tile of least reading volume inside the optimality box (the paper's objective alone); returns a dict."""
    out = TileConfig()
    _check(lib().iolb_tune_bound(ctypes.byref(shape), lds_bytes, vgpr_budget, ctypes.byref(out)))
    return out.as_dict()


def iolb_enumerate(shape, lds_bytes=0, vgpr_budget=0, use_box=True):
    """Every feasible tile, best first, as a list of dicts."""
    L = lib()
    n = _check(L.iolb_enumerate(ctypes.byref(shape), lds_bytes, vgpr_budget, int(use_box), None, 0))
    arr = (TileConfig * max(n, 1))()
    _check(L.iolb_enumerate(ctypes.byref(shape), lds_bytes, vgpr_budget, int(use_box), arr, n))
    return [arr[j].as_dict() for j in range(n)]


def iolb_bounds(shape, Sf):
    out = BoundsOut()
    _check(lib().iolb_bounds(ctypes.byref(shape), int(Sf), ctypes.byref(out)))
    return out.as_dict()


def iolb_winograd_matrices(m):
    """(A, L, B) the Winograd kernels use for F(m x m, 3 x 3), as nested lists of floats."""
    n = m + 2
    A = (ctypes.c_float * (max(m, 1) * n))()
    Lm = (ctypes.c_float * (n * 3))()
    Bm = (ctypes.c_float * (n * n))()
    _check(lib().iolb_winograd_matrices(m, A, Lm, Bm))
    return ([[A[i * n + j] for j in range(n)] for i in range(m)],
            [[Lm[i * 3 + j] for j in range(3)] for i in range(n)],
            [[Bm[i * n + j] for j in range(n)] for i in range(n)])


def _use_current_stream():
    import torch
    _check(lib().iolb_set_stream(ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)))


def _dev_f32(t, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(name + " must be a contiguous float32 tensor on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def conv_direct(x, w, stride=1, pad=0, y=None, cfg=None):
    """y = direct convolution of x [N][C][H][W] with w [K][C][R][S] on the current stream.  pad: zeros per
    side, or (pad_h, pad_w) for a padding of its own per axis (tuned tile only)."""
    import torch
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    if isinstance(pad, (tuple, list)):
        ph, pw = pad
        if cfg is not None:
            raise ValueError("cfg is available with one padding for both axes only")
        if stride < 1 or ph < 0 or pw < 0 or H + 2 * ph < R or W + 2 * pw < S:
            raise IolbError(-1, "invalid argument")
        shape = (N, K, (H + 2 * ph - R) // stride + 1, (W + 2 * pw - S) // stride + 1)
        if y is None:
            y = torch.empty(shape, dtype=torch.float32, device=x.device)
        elif tuple(y.shape) != shape:
            raise ValueError("y has the wrong shape")
        _use_current_stream()
        _check(lib().conv_direct_pad2(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, R, S,
                                      stride, ph, pw))
        return y
    valid = stride >= 1 and pad >= 0 and H + 2 * pad >= R and W + 2 * pad >= S
    if valid:
        shape = (N, K, (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1)
        if y is None:
            y = torch.empty(shape, dtype=torch.float32, device=x.device)
        elif tuple(y.shape) != shape:
            raise ValueError("y has the wrong shape")
    elif y is None:
        raise IolbError(-1, "invalid argument")
    _use_current_stream()
    args = (_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, R, S, stride, pad)
    if cfg is None:
        _check(lib().conv_direct(*args))
    else:
        c = cfg if isinstance(cfg, TileConfig) else TileConfig.from_dict(cfg)
        _check(lib().conv_direct_cfg(*args, ctypes.byref(c)))
    return y


def conv_direct_layout(x, w, stride=1, pad=0, layout=LAYOUT_HWC, y=None, cfg=None):
    """Direct convolution with the tensor layout given: LAYOUT_CHW as conv_direct; LAYOUT_HWC takes
    x [N][H][W][C] and returns y [N][P][Q][K]; LAYOUT_CWH takes x [N][C][W][H] and returns y [N][K][Q][P].
    w is [K][C][R][S] for all."""
    import torch
    if layout == LAYOUT_HWC:
        N, H, W, C = x.shape
    elif layout == LAYOUT_CWH:
        N, C, W, H = x.shape
    else:
        N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    valid = stride >= 1 and pad >= 0 and H + 2 * pad >= R and W + 2 * pad >= S
    if valid:
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        shape = (N, P, Q, K) if layout == LAYOUT_HWC else (N, K, Q, P) if layout == LAYOUT_CWH else (N, K, P, Q)
        if y is None:
            y = torch.empty(shape, dtype=torch.float32, device=x.device)
        elif tuple(y.shape) != shape:
            raise ValueError("y has the wrong shape")
    elif y is None:
        raise IolbError(-1, "invalid argument")
    _use_current_stream()
    c = None
    if cfg is not None:
        c = ctypes.byref(cfg if isinstance(cfg, TileConfig) else TileConfig.from_dict(cfg))
    _check(lib().conv_direct_layout(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, R, S,
                                    stride, pad, int(layout), c))
    return y


def conv_direct_noalloc(x, w, stride, pad, y):
    """conv_direct through the entry point that allocates nothing: y must be given (N, K, P, Q), the re-laid-out
    weights go into the library's fixed scratch array."""
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    _use_current_stream()
    _check(lib().conv_direct_noalloc(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, R, S, stride, pad))
    return y


def conv_winograd(x, w, m, y=None, cfg=None, workspace=None, pad=1):
    """y = Winograd F(m x m, 3 x 3) convolution (stride 1, pad 1 unless `pad` says otherwise) on the current
    stream.  Another padding runs with the tuned tile and the library's workspace only."""
    import torch
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C or R != 3 or S != 3:
        raise ValueError("Winograd path needs 3x3 kernels with matching channels")
    if pad != 1:
        if cfg is not None or workspace is not None:
            raise ValueError("cfg and workspace are available for pad = 1 only")
        if pad < 0 or H + 2 * pad < 3 or W + 2 * pad < 3:
            raise IolbError(-1, "invalid argument")
        shape = (N, K, H + 2 * pad - 2, W + 2 * pad - 2)
        if y is None:
            y = torch.empty(shape, dtype=torch.float32, device=x.device)
        elif tuple(y.shape) != shape:
            raise ValueError("y has the wrong shape")
        _use_current_stream()
        _check(lib().conv_winograd_pad(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, m, pad))
        return y
    if y is None:
        y = torch.empty((N, K, H, W), dtype=torch.float32, device=x.device)
    elif tuple(y.shape) != (N, K, H, W):
        raise ValueError("y has the wrong shape")
    _use_current_stream()
    L = lib()
    if cfg is None and workspace is None:
        _check(L.conv_winograd(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, m))
        return y
    need = L.conv_winograd_workspace_bytes(N, C, H, W, K, m)
    if need == 0:
        raise IolbError(-2, "unsupported Winograd layer")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    c = None
    if cfg is not None:
        c = ctypes.byref(cfg if isinstance(cfg, TileConfig) else TileConfig.from_dict(cfg))
    _check(L.conv_winograd_ws(_dev_f32(x, "x"), _dev_f32(w, "w"), _dev_f32(y, "y"), N, C, H, W, K, m,
                              ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(), c))
    return y


def winograd_transform_kernels(w, m):
    """U = L g L^T for w [K][C][3][3], in a new device buffer the Winograd calls can reuse (see
    conv_winograd_pre); returns (U, C, K)."""
    import torch
    K, C, R, S = w.shape
    if R != 3 or S != 3:
        raise ValueError("Winograd path needs 3x3 kernels")
    need = lib().conv_winograd_kernel_bytes(C, K, m)
    if need == 0:
        raise IolbError(-2, "unsupported Winograd kernel set")
    U = torch.empty(need // 4, dtype=torch.float32, device=w.device)
    _use_current_stream()
    _check(lib().conv_winograd_transform_kernels(_dev_f32(w, "w"), ctypes.c_void_p(U.data_ptr()), C, K, m))
    return U, C, K


def conv_winograd_pre(x, U, K, m, y=None, cfg=None, workspace=None):
    """conv_winograd with kernels transformed beforehand by winograd_transform_kernels."""
    import torch
    N, C, H, W = x.shape
    if y is None:
        y = torch.empty((N, K, H, W), dtype=torch.float32, device=x.device)
    elif tuple(y.shape) != (N, K, H, W):
        raise ValueError("y has the wrong shape")
    L = lib()
    need = L.conv_winograd_workspace_bytes(N, C, H, W, K, m)
    if need == 0:
        raise IolbError(-2, "unsupported Winograd layer")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    c = None
    if cfg is not None:
        c = ctypes.byref(cfg if isinstance(cfg, TileConfig) else TileConfig.from_dict(cfg))
    _use_current_stream()
    _check(L.conv_winograd_pre(_dev_f32(x, "x"), _dev_f32(U, "U"), _dev_f32(y, "y"), N, C, H, W, K, m,
                               ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(), c))
    return y


def winograd_workspace_bytes(N, C, H, W, K, m):
    return int(lib().conv_winograd_workspace_bytes(N, C, H, W, K, m))


def timing_enable(on=True):
    _check(lib().iolb_timing_enable(int(on)))


TIME_DIRECT, TIME_WINO_PRODUCT, TIME_WINO_FUSED = 0, 1, 2


def timing_read(kind):
    """(launches, total_ms) of the main kernels of `kind` timed since the last read."""
    n = ctypes.c_int(0)
    ms = ctypes.c_float(0)
    _check(lib().iolb_timing_read(kind, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


def probe_hbm_copy(src, dst, reps=5):
    """Average milliseconds of one streaming copy of src into dst (float32 GPU tensors of equal size)."""
    if src.numel() != dst.numel():
        raise ValueError("src and dst differ in size")
    _use_current_stream()
    ms = ctypes.c_float(0)
    _check(lib().iolb_probe_hbm_copy(_dev_f32(src, "src"), _dev_f32(dst, "dst"), src.numel() * 4, reps, ctypes.byref(ms)))
    return ms.value


def probe_mfma_sink_bytes():
    return lib().iolb_probe_mfma_sink_bytes()


def probe_mfma_f32(sink, iters=20000, reps=3):
    """(average milliseconds, flop) of one launch of the register-only fp32 MFMA loop."""
    if sink.numel() * 4 < probe_mfma_sink_bytes():
        raise ValueError("sink is too small")
    _use_current_stream()
    ms = ctypes.c_float(0)
    flop = ctypes.c_double(0)
    _check(lib().iolb_probe_mfma_f32(_dev_f32(sink, "sink"), iters, reps, ctypes.byref(ms), ctypes.byref(flop)))
    return ms.value, flop.value


PROBE_ROLE_MFMA, PROBE_ROLE_VALU = 0, 1


def probe_pipeline_share(roles, iters=2000):
    """(milliseconds, [average clock ticks of a wave of each slot]) of one launch in which every SIMD holds
    len(roles) waves, slot s running roles[s] (PROBE_ROLE_MFMA / PROBE_ROLE_VALU)."""
    import torch
    _use_current_stream()
    scratch = torch.zeros(lib().iolb_probe_share_scratch_bytes() // 4 + 1, dtype=torch.float32, device="cuda")
    arr = (ctypes.c_int * len(roles))(*roles)
    ms = ctypes.c_float(0)
    ticks = (ctypes.c_double * len(roles))()
    _check(lib().iolb_probe_pipeline_share(_dev_f32(scratch, "scratch"), len(roles), arr, iters, ctypes.byref(ms), ticks))
    return ms.value, list(ticks)


def release_workspace():
    _check(lib().iolb_release_workspace())
