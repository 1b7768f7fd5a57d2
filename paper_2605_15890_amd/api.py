"""Thin ctypes binding of include/agc.h: same names, argument marshalling only.

Every step of the path runs in the HIP kernels of libagc.so; torch is used for device
memory and for the current stream.  `load()` raises if the library has not been built: there
is no fallback of any kind.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libagc.so")

AGC_OK = 0
AGC_EINVAL, AGC_ESHAPE, AGC_EBITS, AGC_EALIGN, AGC_ENOMEM, AGC_EHIP, AGC_ESTATE = -1, -2, -3, -4, -5, -6, -7
AGC_SCALE_L2, AGC_SCALE_MAXABS = 0, 1
AGC_MAX_WORKERS, AGC_MAX_BITS, AGC_NUM_KERNELS, AGC_MAX_LAYERS = 256, 16, 4, 256
KERNEL_NAMES = ("scale_pass", "scale_finalize", "quantize", "decode")

EXPORTS = [
    "agc_create", "agc_destroy", "agc_set_code", "agc_code_path", "agc_code_bytes", "agc_last_error",
    "agc_encode_quantize", "agc_decode", "agc_step", "agc_profile_enable", "agc_profile_read",
    "agc_scales_per_worker", "agc_set_layers", "agc_decode2", "agc_decode_noalloc", "agc_adam_update", "agc_second_moment_decoder",
    "agc_calibration_copy", "agc_debug_stream_rows", "agc_ls_workspace_floats", "agc_ls_partial_gradients", "agc_gd_update",
    "agc_phi_coef_balanced", "agc_alloc_bits", "agc_alloc_bits_dp", "agc_alloc_objective",
    "agc_build_code", "agc_build_cyclic_code", "agc_build_cyclic_code_opt", "agc_check_unbiased",
]


class AgcOpts(C.Structure):
    _fields_ = [("scale_mode", C.c_int), ("allow_1bit", C.c_int), ("force_generic", C.c_int),
                ("bucket", C.c_int), ("unfused_step", C.c_int), ("reserved", C.c_int * 3)]


class AgcError(RuntimeError):
    def __init__(self, status, message=""):
        super().__init__(f"agc status {status}: {message}")
        self.status = status


_lib = None
_vp, _u8p, _i32p, _f32p, _f64p = (C.c_void_p, C.POINTER(C.c_uint8), C.POINTER(C.c_int32),
                                  C.POINTER(C.c_float), C.POINTER(C.c_double))


def load():
    """Loads libagc.so (built by `python -m paper_2605_15890_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_15890_amd.build`; "
                           "there is no fallback path")
    # The library needs the HIP runtime (libamdhip64.so.7).  PyTorch ships its own copy and the
    # device memory and streams this binding passes down come from that copy, so it has to be
    # in the process first: the loader then binds libagc.so to it by soname instead of pulling
    # a second runtime from the system ROCm directory.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(LIB_PATH)
    L.agc_create.argtypes = [C.POINTER(_vp), C.c_int, C.c_int, C.c_int64, C.POINTER(AgcOpts)]
    L.agc_create.restype = C.c_int
    L.agc_destroy.argtypes = [_vp]
    L.agc_destroy.restype = None
    L.agc_set_code.argtypes = [_vp, _i32p, _i32p, _f32p]
    L.agc_set_code.restype = C.c_int
    L.agc_code_path.argtypes = [_vp]
    L.agc_code_path.restype = C.c_int
    L.agc_code_bytes.argtypes = [C.c_int64, C.c_int]
    L.agc_code_bytes.restype = C.c_int64
    L.agc_last_error.argtypes = [_vp]
    L.agc_last_error.restype = C.c_char_p
    L.agc_encode_quantize.argtypes = [_vp, _vp, C.c_int64, _u8p, C.c_uint64, C.c_uint64,
                                      C.POINTER(_vp), _vp, _vp]
    L.agc_encode_quantize.restype = C.c_int
    L.agc_decode.argtypes = [_vp, C.POINTER(_vp), _vp, _u8p, _f32p, _u8p, _vp, _vp]
    L.agc_decode.restype = C.c_int
    L.agc_scales_per_worker.argtypes = [_vp]
    L.agc_scales_per_worker.restype = C.c_int64
    L.agc_set_layers.argtypes = [_vp, C.c_int, C.POINTER(C.c_int64)]
    L.agc_set_layers.restype = C.c_int
    L.agc_decode2.argtypes = [_vp, C.POINTER(_vp), _vp, _u8p, _f32p, _f32p, _u8p, _vp, _vp, _vp]
    L.agc_decode2.restype = C.c_int
    L.agc_decode_noalloc.argtypes = [C.c_int, C.c_int64, C.c_int, C.POINTER(_vp), _vp, _u8p, _f32p, _u8p, _vp, _vp]
    L.agc_decode_noalloc.restype = C.c_int
    L.agc_adam_update.argtypes = [_vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float, C.c_float, C.c_float,
                                  C.c_int64, C.c_int64, _vp]
    L.agc_adam_update.restype = C.c_int
    L.agc_second_moment_decoder.argtypes = [C.c_int, C.c_int, _i32p, _i32p, _f32p, _f64p, _u8p, C.c_double,
                                            C.c_double, _f32p]
    L.agc_second_moment_decoder.restype = C.c_int
    L.agc_step.argtypes = [_vp, _vp, C.c_int64, _u8p, _f32p, _u8p, C.c_uint64, C.c_uint64,
                           C.POINTER(_vp), _vp, _vp, _vp]
    L.agc_step.restype = C.c_int
    L.agc_ls_workspace_floats.argtypes = [C.c_int64, C.c_int, C.c_int]
    L.agc_ls_workspace_floats.restype = C.c_int64
    L.agc_ls_partial_gradients.argtypes = [_vp, C.c_int64, C.c_int, _vp, _vp, C.c_int, _vp, C.c_int64, _vp,
                                           _vp, _vp]
    L.agc_ls_partial_gradients.restype = C.c_int
    L.agc_gd_update.argtypes = [_vp, _vp, C.c_float, C.c_int64, _vp]
    L.agc_gd_update.restype = C.c_int
    L.agc_calibration_copy.argtypes = [_vp, _vp, C.c_int64, _vp]
    L.agc_calibration_copy.restype = C.c_int
    L.agc_debug_stream_rows.argtypes = [_vp, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _vp, _vp]
    L.agc_debug_stream_rows.restype = C.c_int
    L.agc_profile_enable.argtypes = [_vp, C.c_int]
    L.agc_profile_enable.restype = C.c_int
    L.agc_profile_read.argtypes = [_vp, _f64p, C.POINTER(C.c_int64)]
    L.agc_profile_read.restype = C.c_int
    L.agc_phi_coef_balanced.argtypes = [C.c_int, _f64p, C.c_int]
    L.agc_phi_coef_balanced.restype = C.c_double
    for name in ("agc_alloc_bits", "agc_alloc_bits_dp"):
        fn = getattr(L, name)
        fn.argtypes = [C.c_int, _f64p, C.c_double, C.c_int, C.c_int, C.c_int, _u8p]
        fn.restype = C.c_int
    L.agc_alloc_objective.argtypes = [C.c_int, _f64p, C.c_double, _u8p]
    L.agc_alloc_objective.restype = C.c_double
    L.agc_build_code.argtypes = [C.c_int, C.c_int, _f64p, _u8p, C.c_double, _i32p, _i32p, _f32p,
                                 _f32p, C.c_int, C.POINTER(C.c_int)]
    L.agc_build_code.restype = C.c_int
    L.agc_build_cyclic_code.argtypes = [C.c_int, C.c_int, C.c_int, _f64p, _u8p, C.c_double, _i32p,
                                        _i32p, _f32p, _f32p]
    L.agc_build_cyclic_code.restype = C.c_int
    L.agc_build_cyclic_code_opt.argtypes = [C.c_int, C.c_int, C.c_int, _f64p, _u8p, C.c_double, _i32p,
                                            _i32p, _f32p, _f32p, _f64p, C.POINTER(C.c_int)]
    L.agc_build_cyclic_code_opt.restype = C.c_int
    L.agc_check_unbiased.argtypes = [C.c_int, C.c_int, _i32p, _i32p, _f32p, _f32p, _f64p,
                                     C.c_double, _f64p]
    L.agc_check_unbiased.restype = C.c_int
    _lib = L
    return L


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a, ptype):
    return a.ctypes.data_as(ptype)


# --------------------------------------------------------------------------- host routines
def agc_code_bytes(d, bits):
    return int(load().agc_code_bytes(int(d), int(bits)))


def agc_phi_coef_balanced(p, z_total):
    p = _np(p, np.float64)
    return float(load().agc_phi_coef_balanced(len(p), _ptr(p, _f64p), int(z_total)))


def _alloc(fn, p, phi_coef, z_total, z_min, z_max):
    p = _np(p, np.float64)
    out = np.zeros(len(p), dtype=np.uint8)
    st = fn(len(p), _ptr(p, _f64p), float(phi_coef), int(z_total), int(z_min), int(z_max), _ptr(out, _u8p))
    if st != AGC_OK:
        raise AgcError(st, "bit allocation")
    return out


def agc_alloc_bits(p, phi_coef, z_total, z_min=2, z_max=8):
    return _alloc(load().agc_alloc_bits, p, phi_coef, z_total, z_min, z_max)


def agc_alloc_bits_dp(p, phi_coef, z_total, z_min=2, z_max=8):
    return _alloc(load().agc_alloc_bits_dp, p, phi_coef, z_total, z_min, z_max)


def agc_alloc_objective(p, phi_coef, bits):
    p = _np(p, np.float64)
    bits = _np(bits, np.uint8)
    return float(load().agc_alloc_objective(len(p), _ptr(p, _f64p), float(phi_coef), _ptr(bits, _u8p)))


def agc_build_code(n, k, p, bits, phi_coef):
    """Returns (row_ptr, col, val, w) of the optimally structured interval code."""
    p = _np(p, np.float64)
    bits = _np(bits, np.uint8)
    cap = n + k
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col = np.zeros(cap, dtype=np.int32)
    val = np.zeros(cap, dtype=np.float32)
    w = np.zeros(n, dtype=np.float32)
    nnz = C.c_int()
    st = load().agc_build_code(n, k, _ptr(p, _f64p), _ptr(bits, _u8p), float(phi_coef), _ptr(row_ptr, _i32p),
                               _ptr(col, _i32p), _ptr(val, _f32p), _ptr(w, _f32p), cap, C.byref(nnz))
    if st != AGC_OK:
        raise AgcError(st, "agc_build_code")
    return row_ptr, col[:nnz.value].copy(), val[:nnz.value].copy(), w


def agc_build_cyclic_code(n, k, s, p, bits, phi_coef):
    p = _np(p, np.float64)
    bits = _np(bits, np.uint8)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col = np.zeros(n * s, dtype=np.int32)
    val = np.zeros(n * s, dtype=np.float32)
    w = np.zeros(n, dtype=np.float32)
    st = load().agc_build_cyclic_code(n, k, s, _ptr(p, _f64p), _ptr(bits, _u8p), float(phi_coef),
                                      _ptr(row_ptr, _i32p), _ptr(col, _i32p), _ptr(val, _f32p), _ptr(w, _f32p))
    if st != AGC_OK:
        raise AgcError(st, "agc_build_cyclic_code")
    return row_ptr, col, val, w


def agc_build_cyclic_code_opt(n, k, s, p, bits, phi_coef):
    """Optimal weights on the cyclic support.  Returns (row_ptr, col, val, w, objective, reaches_bound)."""
    p = _np(p, np.float64)
    bits = _np(bits, np.uint8)
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col = np.zeros(n * s, dtype=np.int32)
    val = np.zeros(n * s, dtype=np.float32)
    w = np.zeros(n, dtype=np.float32)
    obj, reach = C.c_double(), C.c_int()
    st = load().agc_build_cyclic_code_opt(n, k, s, _ptr(p, _f64p), _ptr(bits, _u8p), float(phi_coef),
                                          _ptr(row_ptr, _i32p), _ptr(col, _i32p), _ptr(val, _f32p), _ptr(w, _f32p),
                                          C.byref(obj), C.byref(reach))
    if st != AGC_OK:
        raise AgcError(st, "agc_build_cyclic_code_opt")
    return row_ptr, col, val, w, float(obj.value), bool(reach.value)


def agc_check_unbiased(k, row_ptr, col, val, w, p, tol=1e-5):
    """Returns (holds: bool, residual)."""
    row_ptr, col, val = _np(row_ptr, np.int32), _np(col, np.int32), _np(val, np.float32)
    w, p = _np(w, np.float32), _np(p, np.float64)
    res = C.c_double()
    st = load().agc_check_unbiased(len(row_ptr) - 1, int(k), _ptr(row_ptr, _i32p), _ptr(col, _i32p),
                                   _ptr(val, _f32p), _ptr(w, _f32p), _ptr(p, _f64p), float(tol), C.byref(res))
    if st not in (AGC_OK, AGC_EINVAL):
        raise AgcError(st, "agc_check_unbiased")
    return st == AGC_OK, float(res.value)


def agc_second_moment_decoder(k, row_ptr, col, val, p, bits, phi_coef, lam):
    """Second decoding vector v* of the two-track decode (float32, n entries)."""
    row_ptr, col, val = _np(row_ptr, np.int32), _np(col, np.int32), _np(val, np.float32)
    p, bits = _np(p, np.float64), _np(bits, np.uint8)
    n = len(row_ptr) - 1
    v = np.zeros(n, dtype=np.float32)
    st = load().agc_second_moment_decoder(n, int(k), _ptr(row_ptr, _i32p), _ptr(col, _i32p), _ptr(val, _f32p),
                                          _ptr(p, _f64p), _ptr(bits, _u8p), float(phi_coef), float(lam),
                                          _ptr(v, _f32p))
    if st != AGC_OK:
        raise AgcError(st, "agc_second_moment_decoder")
    return v


# --------------------------------------------------------------------------- hot path
def _stream_handle(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(int(stream))


class Context:
    """Owns an agc_ctx and, for convenience, torch buffers for codes / scales / g_hat."""

    def __init__(self, n, k, d, scale_mode=AGC_SCALE_MAXABS, allow_1bit=False, force_generic=False, bucket=0,
                 unfused_step=False):
        self.lib = load()
        self.n, self.k, self.d, self.bucket = int(n), int(k), int(d), int(bucket)
        opts = AgcOpts(int(scale_mode), int(bool(allow_1bit)), int(bool(force_generic)), int(bucket),
                       int(bool(unfused_step)), (C.c_int * 3)())
        h = _vp()
        st = self.lib.agc_create(C.byref(h), self.n, self.k, self.d, C.byref(opts))
        if st != AGC_OK:
            raise AgcError(st, "agc_create: " + self.lib.agc_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.agc_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def _check(self, st):
        if st != AGC_OK:
            raise AgcError(st, self.lib.agc_last_error(self.h).decode())

    def status_of(self, st):
        return st

    def agc_set_code(self, row_ptr, col, val):
        row_ptr, col, val = _np(row_ptr, np.int32), _np(col, np.int32), _np(val, np.float32)
        self._check(self.lib.agc_set_code(self.h, _ptr(row_ptr, _i32p), _ptr(col, _i32p), _ptr(val, _f32p)))

    def agc_set_layers(self, layer_end):
        """Layer-wise max-abs scales: layer_end = ascending ends of the layers (all but the last multiples
        of 256, the last equal to d); an empty sequence returns to one scale per vector."""
        ends = np.ascontiguousarray(np.asarray(layer_end, dtype=np.int64))
        ptr = ends.ctypes.data_as(C.POINTER(C.c_int64)) if ends.size else None
        self._check(self.lib.agc_set_layers(self.h, int(ends.size), ptr))

    def agc_code_path(self):
        return int(self.lib.agc_code_path(self.h))

    def agc_scales_per_worker(self):
        return int(self.lib.agc_scales_per_worker(self.h))

    # ---- buffers (torch: device memory only)
    def alloc_outputs(self, bits, device="cuda"):
        import torch
        bits = _np(bits, np.uint8)
        codes = [torch.empty(agc_code_bytes(self.d, int(b)), dtype=torch.uint8, device=device) for b in bits]
        per = self.agc_scales_per_worker()
        scales = torch.empty((self.n, per) if per > 1 or self.bucket else self.n, dtype=torch.float32, device=device)
        ghat = torch.empty(self.d, dtype=torch.float32, device=device)
        return codes, scales, ghat

    @staticmethod
    def _code_ptrs(codes):
        arr = (_vp * len(codes))()
        for i, t in enumerate(codes):
            arr[i] = t.data_ptr()
        return arr

    def _check_buffers(self, codes, bits, scales=None, ghat=None):
        """The C ABI sees bare pointers; the binding knows the tensors and refuses buffers that
        are too small for the geometry the kernels will write or read."""
        if len(codes) != self.n or len(bits) != self.n:
            raise AgcError(AGC_ESHAPE, f"expected {self.n} streams and bit-widths")
        for i, t in enumerate(codes):
            need = agc_code_bytes(self.d, int(bits[i]))
            if need and t.numel() * t.element_size() < need:
                raise AgcError(AGC_ESHAPE, f"codes[{i}] holds {t.numel() * t.element_size()} bytes, "
                                           f"{need} needed for d={self.d}, bits={int(bits[i])}")
        if scales is not None and scales.numel() < self.n * self.agc_scales_per_worker():
            raise AgcError(AGC_ESHAPE, "scales tensor too small")
        if ghat is not None and ghat.numel() < self.d:
            raise AgcError(AGC_ESHAPE, "ghat tensor too small")

    def _check_gradients(self, G):
        if G.dim() != 2 or G.shape[0] < self.k or G.shape[1] < self.d or G.stride(1) != 1:
            raise AgcError(AGC_ESHAPE, f"G must be a ({self.k}, {self.d}) row-major view, got {tuple(G.shape)}")
        # the kernels read whole groups of four coordinates: the storage behind the view must reach
        # to the end of the last row's last group
        need = G.storage_offset() + (self.k - 1) * G.stride(0) + (self.d + 3) // 4 * 4
        if G.untyped_storage().nbytes() // G.element_size() < need:
            raise AgcError(AGC_ESHAPE, "the storage behind G ends before the last row's last 16-byte group")

    def agc_encode_quantize(self, G, bits, seed, step, codes, scales, stream=None, check=True):
        bits = _np(bits, np.uint8)
        self._check_gradients(G)
        self._check_buffers(codes, bits, scales)
        st = self.lib.agc_encode_quantize(self.h, C.c_void_p(G.data_ptr()), G.stride(0), _ptr(bits, _u8p),
                                          int(seed), int(step), self._code_ptrs(codes),
                                          C.c_void_p(scales.data_ptr()), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def agc_decode(self, codes, scales, bits, w, mask, ghat, stream=None, check=True):
        bits, w, mask = _np(bits, np.uint8), _np(w, np.float32), _np(mask, np.uint8)
        self._check_buffers(codes, bits, scales, ghat)
        st = self.lib.agc_decode(self.h, self._code_ptrs(codes), C.c_void_p(scales.data_ptr()),
                                 _ptr(bits, _u8p), _ptr(w, _f32p), _ptr(mask, _u8p),
                                 C.c_void_p(ghat.data_ptr()), _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def agc_decode2(self, codes, scales, bits, w, v, mask, ghat, ghat2, stream=None, check=True):
        bits, w, v, mask = _np(bits, np.uint8), _np(w, np.float32), _np(v, np.float32), _np(mask, np.uint8)
        self._check_buffers(codes, bits, scales, ghat)
        self._check_buffers(codes, bits, None, ghat2)
        st = self.lib.agc_decode2(self.h, self._code_ptrs(codes), C.c_void_p(scales.data_ptr()),
                                  _ptr(bits, _u8p), _ptr(w, _f32p), _ptr(v, _f32p), _ptr(mask, _u8p),
                                  C.c_void_p(ghat.data_ptr()), C.c_void_p(ghat2.data_ptr()),
                                  _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def agc_step(self, G, bits, w, mask, seed, step, codes, scales, ghat, stream=None, check=True):
        bits, w, mask = _np(bits, np.uint8), _np(w, np.float32), _np(mask, np.uint8)
        self._check_gradients(G)
        self._check_buffers(codes, bits, scales, ghat)
        st = self.lib.agc_step(self.h, C.c_void_p(G.data_ptr()), G.stride(0), _ptr(bits, _u8p), _ptr(w, _f32p),
                               _ptr(mask, _u8p), int(seed), int(step), self._code_ptrs(codes),
                               C.c_void_p(scales.data_ptr()), C.c_void_p(ghat.data_ptr()),
                               _stream_handle(stream))
        if check:
            self._check(st)
        return st

    def agc_profile_enable(self, on=True):
        self._check(self.lib.agc_profile_enable(self.h, int(bool(on))))

    def agc_profile_read(self):
        ms = (C.c_double * AGC_NUM_KERNELS)()
        cnt = (C.c_int64 * AGC_NUM_KERNELS)()
        self._check(self.lib.agc_profile_read(self.h, ms, cnt))
        return {KERNEL_NAMES[j]: (float(ms[j]), int(cnt[j])) for j in range(AGC_NUM_KERNELS)}


def agc_ls_workspace_floats(n_rows, n_feat, k_parts):
    return int(load().agc_ls_workspace_floats(int(n_rows), int(n_feat), int(k_parts)))


def agc_ls_partial_gradients(X, y, beta, k_parts, G, resid, workspace, stream=None, check=True):
    """X: (n_rows, n_feat) torch.bfloat16 on the GPU; G: (k_parts, n_feat) float32 view."""
    n_rows, n_feat = int(X.shape[0]), int(X.shape[1])
    need_ws = agc_ls_workspace_floats(n_rows, n_feat, k_parts)
    if (X.dim() != 2 or not X.is_contiguous() or X.element_size() != 2 or y.numel() < n_rows or beta.numel() < n_feat
            or resid.numel() < n_rows or G.dim() != 2 or G.shape[0] < k_parts or G.shape[1] < n_feat
            or G.stride(1) != 1 or workspace.numel() < need_ws):
        raise AgcError(AGC_ESHAPE, "agc_ls_partial_gradients: a tensor is smaller than the shapes require")
    st = load().agc_ls_partial_gradients(C.c_void_p(X.data_ptr()), X.shape[0], X.shape[1],
                                         C.c_void_p(y.data_ptr()), C.c_void_p(beta.data_ptr()), int(k_parts),
                                         C.c_void_p(G.data_ptr()), G.stride(0), C.c_void_p(resid.data_ptr()),
                                         C.c_void_p(workspace.data_ptr()), _stream_handle(stream))
    if check and st != AGC_OK:
        raise AgcError(st, "agc_ls_partial_gradients")
    return st


def agc_gd_update(beta, ghat, lr, stream=None):
    st = load().agc_gd_update(C.c_void_p(beta.data_ptr()), C.c_void_p(ghat.data_ptr()), float(lr),
                              beta.numel(), _stream_handle(stream))
    if st != AGC_OK:
        raise AgcError(st, "agc_gd_update")


def agc_adam_update(beta, m1, m2, ghat, ghat2, lr, beta1, beta2, eps, t, stream=None):
    st = load().agc_adam_update(C.c_void_p(beta.data_ptr()), C.c_void_p(m1.data_ptr()), C.c_void_p(m2.data_ptr()),
                                C.c_void_p(ghat.data_ptr()), C.c_void_p(ghat2.data_ptr()), float(lr),
                                float(beta1), float(beta2), float(eps), int(t), beta.numel(),
                                _stream_handle(stream))
    if st != AGC_OK:
        raise AgcError(st, "agc_adam_update")


def agc_decode_noalloc(n, d, bucket, codes, scales, bits, w, mask, ghat, stream=None, check=True):
    """Context-free decode for callers that cannot allocate: same outputs as Context.agc_decode."""
    bits, w, mask = _np(bits, np.uint8), _np(w, np.float32), _np(mask, np.uint8)
    L = load()
    if len(codes) != n or len(bits) != n or len(w) != n or len(mask) != n:
        raise AgcError(AGC_ESHAPE, f"expected {n} streams, bit-widths, weights and mask entries")
    if n <= AGC_MAX_WORKERS:   # sizes the library would refuse are left for it to refuse
        for i, t in enumerate(codes):
            need = agc_code_bytes(d, int(bits[i]))
            if need and t.numel() * t.element_size() < need:
                raise AgcError(AGC_ESHAPE, f"codes[{i}] is smaller than d={d}, bits={int(bits[i])} require")
        per = (int(d) + 255) // 256 if bucket == 256 else 1
        if scales.numel() < n * per or ghat.numel() < d:
            raise AgcError(AGC_ESHAPE, "scales or ghat tensor too small")
    st = L.agc_decode_noalloc(int(n), int(d), int(bucket), Context._code_ptrs(codes),
                              C.c_void_p(scales.data_ptr()), _ptr(bits, _u8p), _ptr(w, _f32p), _ptr(mask, _u8p),
                              C.c_void_p(ghat.data_ptr()), _stream_handle(stream))
    if check and st != AGC_OK:
        raise AgcError(st, L.agc_last_error(None).decode())
    return st


def agc_calibration_copy(dst, src, nbytes, stream=None):
    """Plain copy of nbytes between two torch tensors (counter calibration)."""
    st = load().agc_calibration_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), int(nbytes),
                                     _stream_handle(stream))
    if st != AGC_OK:
        raise AgcError(st, "agc_calibration_copy")


def agc_debug_stream_rows(G, piece_bytes, out, wg_flush=False, blocks_per_wave=1, waves_per_simd=0, fma_per_row=0,
                          stream=None):
    """The bare access pattern of the streaming passes over G (k x d view); piece_bytes = 0 reads only;
    wg_flush: pieces leave per workgroup after a barrier (the quantize pass's form) instead of per wave;
    blocks_per_wave = 2 (reads only): the two-block walk of the max-abs scale pass; waves_per_simd = 4: built
    for the quantize pass's occupancy; fma_per_row: dummy dependent multiply-adds per row and lane."""
    k, d = int(G.shape[0]), int(G.shape[1])
    need = max(16, k * (d // 256) * int(piece_bytes))
    if G.dim() != 2 or G.stride(1) != 1 or out.numel() * out.element_size() < need:
        raise AgcError(AGC_ESHAPE, f"agc_debug_stream_rows: out must hold {need} bytes")
    st = load().agc_debug_stream_rows(C.c_void_p(G.data_ptr()), G.stride(0), k, d, int(piece_bytes),
                                      int(bool(wg_flush)), int(blocks_per_wave), int(waves_per_simd), int(fma_per_row),
                                      C.c_void_p(out.data_ptr()), _stream_handle(stream))
    if st != AGC_OK:
        raise AgcError(st, "agc_debug_stream_rows")


def padded_rows(k, d, device="cuda"):
    """A k x d float32 view whose row stride is a multiple of 4 elements and whose base is
    16-byte aligned, as agc_encode_quantize requires."""
    import torch
    ld = (d + 3) // 4 * 4
    return torch.zeros((k, ld), dtype=torch.float32, device=device)[:, :d]
