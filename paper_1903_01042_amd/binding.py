"""Thin ctypes binding of libcodenet.so: same names as the C ABI, argument
marshalling only.  PyTorch supplies device memory and the current stream.

The library must be built first (`python -m paper_1903_01042_amd.build`);
loading fails loudly if it is missing -- there is no fallback path.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcodenet.so")

MAX_T, MAX_R, MAX_L, MAX_FAULTS = 4, 8, 40, 64
F32, BF16_F32ACC = 0, 1
FWD, BWD, WEIGHT, CHECK = 0, 1, 2, 3
CLEAN, CORRECTED, UNCORRECTABLE, DISAGREE = 0, 1, 2, 3
CHECK_EVALUATION, CHECK_LIST = 0, 1
DENSE_REL, SPARSE_ABS = 0, 1
EPI_NONE, EPI_RELU, EPI_MASK_POS, EPI_MUL = 0, 1, 2, 3
E_NULL, E_SHAPE, E_BATCH, E_ORDER, E_CODE, E_FAULT, E_HIP, E_DTYPE, E_ALLOC = range(-1, -10, -1)

EXPORTS = ["codenet_encode", "codenet_layer_geometry", "codenet_forward", "codenet_backward",
           "codenet_forward_ld", "codenet_backward_ld",
           "codenet_inject", "codenet_inject_noalloc", "codenet_detect_decode", "codenet_detect_decode_act",
           "codenet_detect_decode_verified", "codenet_output_modified", "codenet_update", "codenet_regenerate", "codenet_export_coded",
           "codenet_export_weights", "codenet_destroy", "codenet_timestamp", "codenet_profile_stamps", "codenet_strerror"]


class Desc(ctypes.Structure):
    _fields_ = [("n_out", ctypes.c_int), ("n_in", ctypes.c_int), ("m", ctypes.c_int), ("n", ctypes.c_int),
                ("r_rows", ctypes.c_int), ("r_cols", ctypes.c_int),
                ("P_r", ctypes.POINTER(ctypes.c_double)), ("P_c", ctypes.POINTER(ctypes.c_double)),
                ("dtype", ctypes.c_int), ("max_batch", ctypes.c_int),
                ("tau_detect", ctypes.c_double), ("tau_resid", ctypes.c_double)]


class Report(ctypes.Structure):
    _fields_ = [("verdict", ctypes.c_int), ("n_located", ctypes.c_int), ("located", ctypes.c_int * MAX_T),
                ("syn_rel", ctypes.c_float * MAX_R), ("resid_rel", ctypes.c_float)]


class Fault(ctypes.Structure):
    _fields_ = [("phase", ctypes.c_int), ("bi", ctypes.c_int), ("bj", ctypes.c_int), ("mode", ctypes.c_int),
                ("seed", ctypes.c_uint64), ("step", ctypes.c_uint64),
                ("lo", ctypes.c_float), ("hi", ctypes.c_float), ("density", ctypes.c_float),
                ("reserved", ctypes.c_int)]


REPORT_BYTES = ctypes.sizeof(Report)
_lib = None


def load_library(path=LIB_PATH):
    """dlopen the C-ABI library and declare its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch owns the device memory and streams handed to the library: load its
    # HIP runtime first so that both use the one runtime instance.
    import torch  # noqa: F401
    if not os.path.exists(path):
        raise RuntimeError("libcodenet.so is not built: run `python -m paper_1903_01042_amd.build` "
                           "(expected at %s)" % path)
    lib = ctypes.CDLL(path)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    pi = ctypes.POINTER(ctypes.c_int)
    lib.codenet_encode.argtypes = [ctypes.POINTER(Desc), vp, vp, ctypes.POINTER(vp)]
    lib.codenet_layer_geometry.argtypes = [vp, pi, pi, pi, pi]
    lib.codenet_forward.argtypes = [vp, vp, ci, vp, vp]
    lib.codenet_backward.argtypes = [vp, vp, ci, vp, vp]
    lib.codenet_forward_ld.argtypes = [vp, vp, ctypes.c_long, ci, vp, vp]
    lib.codenet_backward_ld.argtypes = [vp, vp, ctypes.c_long, ci, vp, vp]
    lib.codenet_inject.argtypes = [vp, ctypes.POINTER(Fault), ci, vp, ci, vp]
    lib.codenet_inject_noalloc.argtypes = [vp, ctypes.POINTER(Fault), ci, vp, ci, vp]
    lib.codenet_detect_decode.argtypes = [vp, ci, vp, ci, vp, vp, vp]
    lib.codenet_detect_decode_act.argtypes = [vp, ci, vp, ci, vp, vp, ci, vp, vp]
    lib.codenet_detect_decode_verified.argtypes = [vp, ci, vp, ci, vp, vp, ci, vp, vp]
    lib.codenet_output_modified.argtypes = [vp, ci]
    lib.codenet_update.argtypes = [vp, cf, vp]
    lib.codenet_regenerate.argtypes = [vp, ci, vp, vp]
    lib.codenet_export_coded.argtypes = [vp, vp, vp]
    lib.codenet_export_weights.argtypes = [vp, vp, vp]
    lib.codenet_destroy.argtypes = [vp]
    lib.codenet_timestamp.argtypes = [vp, vp, pi]
    lib.codenet_profile_stamps.argtypes = [vp, vp]
    lib.codenet_strerror.argtypes = [ci]
    lib.codenet_strerror.restype = ctypes.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def timestamp(dst, index=0):
    """Enqueue a device time stamp into element `index` of the int64 CUDA tensor `dst` on the current
    stream; returns the clock rate in ticks per microsecond."""
    rate = ctypes.c_int(0)
    _check(load_library().codenet_timestamp(ctypes.c_void_p(dst.data_ptr() + 8 * int(index)), _stream(),
                                            ctypes.byref(rate)), "codenet_timestamp")
    return int(rate.value)


class CodenetError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = load_library().codenet_strerror(code).decode()
        super().__init__("%s failed: %s (%d)" % (where, msg, code))


def _check(code, where):
    if code != 0:
        raise CodenetError(code, where)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_f32(t, shape, name):
    import torch
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError("%s must be a contiguous float32 CUDA tensor of shape %s, got %s %s"
                         % (name, tuple(shape), t.dtype, tuple(t.shape)))
    return t


def pack_faults(faults):
    arr = (Fault * max(1, len(faults)))()
    for k, f in enumerate(faults):
        arr[k] = Fault(int(f["phase"]), int(f["bi"]), int(f["bj"]), int(f.get("mode", DENSE_REL)),
                       int(f["seed"]), int(f["step"]), float(f["lo"]), float(f["hi"]),
                       float(f.get("density", 0.0)), 0)
    return arr


class CodedLayer:
    """Owns one `codenet_layer*`.  Methods are the C calls with tensors for pointers."""

    def __init__(self, W, P_r, P_c, dtype=F32, max_batch=1, tau_detect=1e-3, tau_resid=2e-3):
        import torch
        self._h = ctypes.c_void_p(0)
        lib = load_library()
        if not (W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()):
            raise ValueError("W must be a contiguous float32 CUDA matrix")
        self.n_out, self.n_in = int(W.shape[0]), int(W.shape[1])
        P_r = np.ascontiguousarray(np.asarray(P_r, dtype=np.float64))
        P_c = np.ascontiguousarray(np.asarray(P_c, dtype=np.float64))
        self.m, self.n = int(P_r.shape[0]), int(P_c.shape[0])
        self.r_rows = int(P_r.shape[1]) if P_r.ndim == 2 else 0
        self.r_cols = int(P_c.shape[1]) if P_c.ndim == 2 else 0
        d = Desc(self.n_out, self.n_in, self.m, self.n, self.r_rows, self.r_cols,
                 P_r.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if self.r_rows else None,
                 P_c.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if self.r_cols else None,
                 int(dtype), int(max_batch), float(tau_detect), float(tau_resid))
        h = ctypes.c_void_p(0)
        _check(lib.codenet_encode(ctypes.byref(d), _ptr(W), _stream(), ctypes.byref(h)), "codenet_encode")
        self._h = h
        self.device = W.device
        self.max_batch = int(max_batch)
        g = [ctypes.c_int(0) for _ in range(4)]
        _check(lib.codenet_layer_geometry(h, *[ctypes.byref(x) for x in g]), "codenet_layer_geometry")
        self.B_r, self.B_c, self.coded_rows, self.coded_cols = (x.value for x in g)

    # ---- the six calls -----------------------------------------------------------------
    @staticmethod
    def _rows(t, width, name):
        """A float32 CUDA matrix [b][>= width] whose rows may be a part of wider rows (a column slice
        of a contiguous tensor): returns (b, row pitch in elements)."""
        import torch
        ok = (t.is_cuda and t.dtype == torch.float32 and t.dim() == 2 and int(t.shape[1]) == width
              and t.stride(1) == 1 and t.stride(0) >= width)
        if not ok:
            raise ValueError("%s must be a float32 CUDA matrix with %d unit-stride columns, got %s %s strides %s"
                             % (name, width, t.dtype, tuple(t.shape), tuple(t.stride())))
        return int(t.shape[0]), int(t.stride(0))

    def forward(self, X, S_coded=None):
        """X: [b][n_in]; its rows may be a part of wider rows (a column slice of another tensor, e.g. of the
        coded buffer in which another layer's check left its decoded output): codenet_forward_ld."""
        import torch
        b, ldx = self._rows(X, self.n_in, "X")
        if S_coded is None:
            S_coded = torch.empty((b, self.coded_rows), dtype=torch.float32, device=self.device)
        _dev_f32(S_coded, (b, self.coded_rows), "S_coded")
        if ldx == self.n_in:
            _check(load_library().codenet_forward(self._h, _ptr(X), b, _ptr(S_coded), _stream()), "codenet_forward")
        else:
            _check(load_library().codenet_forward_ld(self._h, _ptr(X), ldx, b, _ptr(S_coded), _stream()), "codenet_forward_ld")
        return S_coded

    def backward(self, D, C_coded=None):
        import torch
        b, ldd = self._rows(D, self.n_out, "Delta")
        if C_coded is None:
            C_coded = torch.empty((b, self.coded_cols), dtype=torch.float32, device=self.device)
        _dev_f32(C_coded, (b, self.coded_cols), "C_coded")
        if ldd == self.n_out:
            _check(load_library().codenet_backward(self._h, _ptr(D), b, _ptr(C_coded), _stream()), "codenet_backward")
        else:
            _check(load_library().codenet_backward_ld(self._h, _ptr(D), ldd, b, _ptr(C_coded), _stream()), "codenet_backward_ld")
        return C_coded

    def inject(self, faults, coded_out=None, noalloc=False):
        """noalloc: through codenet_inject_noalloc (the library's fixed scratch array instead of the
        layer's buffer)."""
        if not faults:
            return
        phase = int(faults[0]["phase"])
        b = 0
        if phase == CHECK:
            coded_out = None
        elif phase != WEIGHT:
            width = self.coded_rows if phase == FWD else self.coded_cols
            b = int(coded_out.shape[0])
            _dev_f32(coded_out, (b, width), "coded_out")
        arr = pack_faults(faults)
        if noalloc:
            _check(load_library().codenet_inject_noalloc(self._h, arr, len(faults), _ptr(coded_out), b, _stream()),
                   "codenet_inject_noalloc")
            return
        _check(load_library().codenet_inject(self._h, arr, len(faults), _ptr(coded_out), b, _stream()),
               "codenet_inject")

    def detect_decode(self, phase, coded_out, decoded=None, report=None, want_decoded=True, epilogue=0, aux=None,
                      verified=False):
        """report: optional uint8 CUDA (or pinned) tensor of REPORT_BYTES bytes.
        epilogue / aux: EPI_* elementwise step applied to the decoded output (aux shaped like it).
        verified: the check with the verification steps of Error Model 2 (needs a report)."""
        import torch
        width, n_logical = (self.coded_rows, self.n_out) if phase == FWD else (self.coded_cols, self.n_in)
        b = int(coded_out.shape[0])
        _dev_f32(coded_out, (b, width), "coded_out")
        if decoded is None and want_decoded:
            decoded = torch.empty((b, n_logical), dtype=torch.float32, device=self.device)
        if decoded is not None and decoded.data_ptr() != coded_out.data_ptr():
            _dev_f32(decoded, (b, n_logical), "decoded")
        if report is not None and (report.dtype != torch.uint8 or report.numel() < REPORT_BYTES):
            raise ValueError("report must be a uint8 tensor of at least %d bytes" % REPORT_BYTES)
        if aux is not None:
            _dev_f32(aux, (b, n_logical), "aux")
        if verified:
            _check(load_library().codenet_detect_decode_verified(self._h, int(phase), _ptr(coded_out), b,
                                                                 _ptr(decoded), _ptr(report), int(epilogue),
                                                                 _ptr(aux), _stream()),
                   "codenet_detect_decode_verified")
            return decoded
        if epilogue:
            _check(load_library().codenet_detect_decode_act(self._h, int(phase), _ptr(coded_out), b, _ptr(decoded),
                                                            _ptr(report), int(epilogue), _ptr(aux), _stream()),
                   "codenet_detect_decode_act")
            return decoded
        _check(load_library().codenet_detect_decode(self._h, int(phase), _ptr(coded_out), b, _ptr(decoded),
                                                    _ptr(report), _stream()), "codenet_detect_decode")
        return decoded

    def output_modified(self, phase):
        _check(load_library().codenet_output_modified(self._h, int(phase)), "codenet_output_modified")

    def update(self, eta):
        _check(load_library().codenet_update(self._h, float(eta), _stream()), "codenet_update")

    def regenerate(self, phase, report):
        """Rebuild the stored blocks of the block-rows (FWD) / block-columns (BWD) that the device-side
        `report` of that phase's detect_decode lists as located; a no-op for any other verdict."""
        import torch
        if report is None or report.dtype != torch.uint8 or report.numel() < REPORT_BYTES or not report.is_cuda:
            raise ValueError("report must be the uint8 CUDA tensor that detect_decode filled")
        _check(load_library().codenet_regenerate(self._h, int(phase), _ptr(report), _stream()), "codenet_regenerate")

    # ---- inspection ----------------------------------------------------------------------
    def export_coded(self):
        import torch
        out = torch.empty((self.coded_rows, self.coded_cols), dtype=torch.float32, device=self.device)
        _check(load_library().codenet_export_coded(self._h, _ptr(out), _stream()), "codenet_export_coded")
        return out

    def export_weights(self):
        import torch
        out = torch.empty((self.n_out, self.n_in), dtype=torch.float32, device=self.device)
        _check(load_library().codenet_export_weights(self._h, _ptr(out), _stream()), "codenet_export_weights")
        return out

    def new_report(self):
        import torch
        return torch.zeros(REPORT_BYTES, dtype=torch.uint8, device=self.device)

    @staticmethod
    def read_report(report):
        """Synchronising read of a report tensor into a dict."""
        raw = bytes(report.cpu().numpy().tobytes()[:REPORT_BYTES])
        r = Report.from_buffer_copy(raw)
        return dict(verdict=r.verdict, n_located=r.n_located,
                    located=[int(v) for v in r.located[: r.n_located]],
                    syn_rel=[float(v) for v in r.syn_rel], resid_rel=float(r.resid_rel))

    def destroy(self):
        if self._h:
            load_library().codenet_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
