"""ctypes front-end of the C oracle (oracle/agc_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  It never imports the product package.
All arrays are host numpy arrays.
"""
import ctypes as C
import os
import numpy as np

from . import build as _build

_lib = None

_u8p = C.POINTER(C.c_uint8)
_u32p = C.POINTER(C.c_uint32)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


def lib():
    global _lib
    if _lib is None:
        # AGC_ORACLE_LIB: another build of the same source (the sanitizer leg of the tests)
        _lib = C.CDLL(os.environ.get("AGC_ORACLE_LIB") or _build.build())
        L = _lib
        L.agc_oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.agc_oracle_philox4x32_10.restype = None
        L.agc_oracle_draw.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, _u32p, _u32p]
        L.agc_oracle_draw.restype = None
        L.agc_oracle_encode_range.argtypes = [_f32p, C.c_int64, _i32p, _i32p, _f32p, C.c_int,
                                              C.c_int64, C.c_int64, _f32p]
        L.agc_oracle_encode_range.restype = None
        L.agc_oracle_scale_maxabs.argtypes = [_f32p, C.c_int64]
        L.agc_oracle_scale_maxabs.restype = C.c_float
        L.agc_oracle_scale_l2.argtypes = [_f32p, C.c_int64]
        L.agc_oracle_scale_l2.restype = C.c_float
        L.agc_oracle_sumsq_tree.argtypes = [_f32p, C.c_int64]
        L.agc_oracle_sumsq_tree.restype = C.c_double
        L.agc_oracle_levels.argtypes = [C.c_int]
        L.agc_oracle_levels.restype = C.c_int
        L.agc_oracle_inv16.argtypes = [C.c_float, C.c_int]
        L.agc_oracle_inv16.restype = C.c_float
        L.agc_oracle_grid_pos.argtypes = [C.c_float, C.c_float, C.c_int]
        L.agc_oracle_grid_pos.restype = C.c_float
        L.agc_oracle_quantize_one.argtypes = [C.c_float, C.c_float, C.c_int, C.c_uint32, C.c_uint32]
        L.agc_oracle_quantize_one.restype = C.c_uint32
        L.agc_oracle_quantize_prob.argtypes = [C.c_float, C.c_float, C.c_int, _u32p,
                                               C.POINTER(C.c_double)]
        L.agc_oracle_quantize_prob.restype = None
        L.agc_oracle_code_bytes.argtypes = [C.c_int64, C.c_int]
        L.agc_oracle_code_bytes.restype = C.c_int64
        L.agc_oracle_pack.argtypes = [_u32p, C.c_int64, C.c_int, _u8p]
        L.agc_oracle_pack.restype = None
        L.agc_oracle_unpack.argtypes = [_u8p, C.c_int64, C.c_int, _u32p]
        L.agc_oracle_unpack.restype = None
        L.agc_oracle_unpack_range.argtypes = [_u8p, C.c_int, C.c_int64, C.c_int64, _u32p]
        L.agc_oracle_unpack_range.restype = None
        L.agc_oracle_code_value.argtypes = [C.c_uint32, C.c_int]
        L.agc_oracle_code_value.restype = C.c_float
        L.agc_oracle_coef.argtypes = [C.c_float, C.c_float, C.c_int]
        L.agc_oracle_coef.restype = C.c_float
        L.agc_oracle_decode_range.argtypes = [C.c_int, C.POINTER(_u8p), _f32p, _u8p, _f32p, _u8p,
                                              C.c_int64, C.c_int64, _f32p]
        L.agc_oracle_decode_range.restype = None
        L.agc_oracle_scales.argtypes = [C.c_int, C.c_int64, _f32p, C.c_int64, _i32p, _i32p, _f32p,
                                        C.c_int, _f32p]
        L.agc_oracle_scales.restype = None
        L.agc_oracle_codes_range.argtypes = [_f32p, C.c_int64, _i32p, _i32p, _f32p, C.c_int, C.c_int,
                                             C.c_float, C.c_uint64, C.c_uint64, C.c_int64,
                                             C.c_int64, _u32p]
        L.agc_oracle_codes_range.restype = None
        L.agc_oracle_encode_quantize.argtypes = [C.c_int, C.c_int64, _f32p, C.c_int64, _i32p, _i32p,
                                                 _f32p, _u8p, C.c_uint64, C.c_uint64, C.c_int,
                                                 _f32p, C.POINTER(_u8p), _f32p]
        L.agc_oracle_encode_quantize.restype = None
        L.agc_oracle_bucket_scale.argtypes = [_f32p, C.c_int64, C.c_int64, C.c_int]
        L.agc_oracle_bucket_scale.restype = C.c_float
        L.agc_oracle_inv16_bucket.argtypes = [C.c_float, C.c_int]
        L.agc_oracle_inv16_bucket.restype = C.c_float
        L.agc_oracle_wl_bucket.argtypes = [C.c_float, C.c_int]
        L.agc_oracle_wl_bucket.restype = C.c_float
        L.agc_oracle_codes_bucket_range.argtypes = [_f32p, C.c_int64, _i32p, _i32p, _f32p, C.c_int, C.c_int,
                                                    C.c_int, C.c_uint64, C.c_uint64, C.c_int64, C.c_int64,
                                                    C.c_int64, _u32p, _f32p]
        L.agc_oracle_codes_bucket_range.restype = None
        L.agc_oracle_encode_quantize_bucket.argtypes = [C.c_int, C.c_int64, _f32p, C.c_int64, _i32p, _i32p,
                                                        _f32p, _u8p, C.c_uint64, C.c_uint64, C.c_int,
                                                        C.POINTER(_u8p), _f32p]
        L.agc_oracle_encode_quantize_bucket.restype = None
        L.agc_oracle_decode_bucket_range.argtypes = [C.c_int, C.POINTER(_u8p), _f32p, C.c_int64, _u8p, _f32p,
                                                     _u8p, C.c_int64, C.c_int64, _f32p]
        L.agc_oracle_decode_bucket_range.restype = None
        L.agc_oracle_step_bucket.argtypes = [C.c_int, C.c_int64, _f32p, C.c_int64, _i32p, _i32p, _f32p,
                                             _u8p, _f32p, _u8p, C.c_uint64, C.c_uint64, C.c_int,
                                             C.POINTER(_u8p), _f32p, _f32p]
        L.agc_oracle_step_bucket.restype = None
        L.agc_oracle_step.argtypes = [C.c_int, C.c_int64, _f32p, C.c_int64, _i32p, _i32p, _f32p,
                                      _u8p, _f32p, _u8p, C.c_uint64, C.c_uint64, C.c_int,
                                      C.POINTER(_u8p), _f32p, _f32p]
        L.agc_oracle_step.restype = None
        L.agc_oracle_worker_moments.argtypes = [_f32p, C.c_int64, _i32p, _i32p, _f32p, C.c_int, C.c_int, C.c_float,
                                                C.c_int64, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.agc_oracle_worker_moments.restype = C.c_int
        L.agc_oracle_set_threads.argtypes = [C.c_int]
        L.agc_oracle_set_threads.restype = None
        L.agc_oracle_threads.argtypes = []
        L.agc_oracle_threads.restype = C.c_int
    return _lib


SCALE_L2 = 0
SCALE_MAXABS = 1


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(_u8p)


def _u32(a):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    return a, a.ctypes.data_as(_u32p)


# ------------------------------------------------------------------ bucket-wise scales
BUCKET = 256


def num_buckets(d):
    return (int(d) + BUCKET - 1) // BUCKET


def bucket_scale(f, u, scale_mode):
    f, fp = _f32(f)
    return float(lib().agc_oracle_bucket_scale(fp, f.size, int(u), int(scale_mode)))


def inv16_bucket(scale, bits):
    return float(lib().agc_oracle_inv16_bucket(float(scale), int(bits)))


def wl_bucket(w, bits):
    return float(lib().agc_oracle_wl_bucket(float(w), int(bits)))


def codes_bucket_range(G, csr, i, bits_i, scale_mode, seed, step, m0, m1):
    """Unpacked codes of worker i on [m0, m1) (m0 a multiple of 256) and the scales of the
    buckets that cover the range."""
    G, gp = _f32(G)
    d = G.shape[1]
    assert m0 % BUCKET == 0
    rp, cp, vp = csr.ptrs()
    out = np.zeros(m1 - m0, dtype=np.uint32)
    sc = np.zeros(num_buckets(m1) - m0 // BUCKET, dtype=np.float32)
    lib().agc_oracle_codes_bucket_range(gp, G.strides[0] // 4, rp, cp, vp, int(i), int(bits_i),
                                        int(scale_mode), int(seed), int(step), d, int(m0), int(m1),
                                        out.ctypes.data_as(_u32p), sc.ctypes.data_as(_f32p))
    return out, sc


def decode_bucket(streams, scales, bits, w, mask, d, m0=0, m1=None):
    """scales: (n, num_buckets(d)) float32."""
    m1 = d if m1 is None else m1
    n = len(streams)
    sp, keep = _stream_ptrs(streams)
    sc, scp = _f32(scales)
    assert sc.shape == (n, num_buckets(d))
    b, bp = _u8(bits)
    ww, wp = _f32(w)
    mk, mp = _u8(mask)
    out = np.zeros(m1 - m0, dtype=np.float32)
    lib().agc_oracle_decode_bucket_range(n, sp, scp, num_buckets(d), bp, wp, mp, int(m0), int(m1),
                                         out.ctypes.data_as(_f32p))
    return out


def step_bucket(G, csr, bits, w, mask, seed, step_, scale_mode):
    """One whole pass with one scale per 256-coordinate bucket.  Returns (streams, scales (n, nb), ghat)."""
    G, gp = _f32(G)
    d = G.shape[1]
    rp, cp, vp = csr.ptrs()
    b, bp = _u8(bits)
    ww, wp = _f32(w)
    mk, mp = _u8(mask)
    streams = [np.zeros(code_bytes(d, int(bi)), dtype=np.uint8) for bi in b]
    sp, keep = _stream_ptrs(streams)
    sc_out = np.zeros((csr.n, num_buckets(d)), dtype=np.float32)
    ghat = np.zeros(d, dtype=np.float32)
    lib().agc_oracle_step_bucket(csr.n, d, gp, G.strides[0] // 4, rp, cp, vp, bp, wp, mp, int(seed),
                                 int(step_), int(scale_mode), sp, sc_out.ctypes.data_as(_f32p),
                                 ghat.ctypes.data_as(_f32p))
    return streams, sc_out, ghat


def threads():
    return int(lib().agc_oracle_threads())


def set_threads(count):
    lib().agc_oracle_set_threads(int(count))


def philox4x32_10(ctr, key):
    c, cp = _u32(ctr)
    k, kp = _u32(key)
    out = np.zeros(4, dtype=np.uint32)
    lib().agc_oracle_philox4x32_10(cp, kp, out.ctypes.data_as(_u32p))
    return out


def draw(seed, step, worker, m):
    u16 = C.c_uint32()
    r2 = C.c_uint32()
    lib().agc_oracle_draw(int(seed), int(step), int(worker), int(m), C.byref(u16), C.byref(r2))
    return int(u16.value), int(r2.value)


class Csr:
    """Code matrix B (n x k) as CSR rows; column order in a row is the summation order."""

    def __init__(self, row_ptr, col, val, k):
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
        self.col = np.ascontiguousarray(col, dtype=np.int32)
        self.val = np.ascontiguousarray(val, dtype=np.float32)
        self.n = len(self.row_ptr) - 1
        self.k = int(k)

    @staticmethod
    def from_dense(B):
        B = np.asarray(B)
        n, k = B.shape
        row_ptr, col, val = [0], [], []
        for i in range(n):
            for j in range(k):
                if B[i, j] != 0:
                    col.append(j)
                    val.append(B[i, j])
            row_ptr.append(len(col))
        return Csr(row_ptr, col, val, k)

    def dense(self):
        B = np.zeros((self.n, self.k), dtype=np.float64)
        for i in range(self.n):
            for e in range(self.row_ptr[i], self.row_ptr[i + 1]):
                B[i, self.col[e]] += float(self.val[e])
        return B

    def ptrs(self):
        return (self.row_ptr.ctypes.data_as(_i32p), self.col.ctypes.data_as(_i32p),
                self.val.ctypes.data_as(_f32p))


def encode(G, csr, i, m0=0, m1=None):
    G, gp = _f32(G)
    d = G.shape[1]
    m1 = d if m1 is None else m1
    out = np.zeros(m1 - m0, dtype=np.float32)
    rp, cp, vp = csr.ptrs()
    lib().agc_oracle_encode_range(gp, G.strides[0] // 4, rp, cp, vp, int(i), int(m0), int(m1),
                                  out.ctypes.data_as(_f32p))
    return out


def scale_maxabs(f):
    f, fp = _f32(f)
    return np.float32(lib().agc_oracle_scale_maxabs(fp, f.size))


def scale_l2(f):
    f, fp = _f32(f)
    return np.float32(lib().agc_oracle_scale_l2(fp, f.size))


def sumsq_tree(f):
    f, fp = _f32(f)
    return float(lib().agc_oracle_sumsq_tree(fp, f.size))


def levels(bits):
    return int(lib().agc_oracle_levels(int(bits)))


def inv16(scale, bits):
    return np.float32(lib().agc_oracle_inv16(float(np.float32(scale)), int(bits)))


def grid_pos(f, inv16_, bits):
    return np.float32(lib().agc_oracle_grid_pos(float(np.float32(f)), float(np.float32(inv16_)),
                                                int(bits)))


def quantize_one(f, inv16_, bits, u16, r2):
    return int(lib().agc_oracle_quantize_one(float(np.float32(f)), float(np.float32(inv16_)),
                                             int(bits), int(u16), int(r2)))


def quantize_prob(f, inv16_, bits):
    lo = C.c_uint32()
    p = C.c_double()
    lib().agc_oracle_quantize_prob(float(np.float32(f)), float(np.float32(inv16_)), int(bits),
                                   C.byref(lo), C.byref(p))
    return int(lo.value), float(p.value)


def code_bytes(d, bits):
    return int(lib().agc_oracle_code_bytes(int(d), int(bits)))


def pack(codes, bits):
    codes, cp = _u32(codes)
    out = np.zeros(code_bytes(codes.size, bits), dtype=np.uint8)
    lib().agc_oracle_pack(cp, codes.size, int(bits), out.ctypes.data_as(_u8p))
    return out


def unpack(stream, d, bits):
    stream, sp = _u8(stream)
    out = np.zeros(d, dtype=np.uint32)
    lib().agc_oracle_unpack(sp, int(d), int(bits), out.ctypes.data_as(_u32p))
    return out


def unpack_range(stream, bits, m0, m1):
    stream, sp = _u8(stream)
    out = np.zeros(m1 - m0, dtype=np.uint32)
    lib().agc_oracle_unpack_range(sp, int(bits), int(m0), int(m1), out.ctypes.data_as(_u32p))
    return out


def code_value(code, bits):
    return np.float32(lib().agc_oracle_code_value(int(code), int(bits)))


def coef(w, scale, bits):
    return np.float32(lib().agc_oracle_coef(float(np.float32(w)), float(np.float32(scale)),
                                            int(bits)))


def _stream_ptrs(streams):
    arr = (_u8p * len(streams))()
    keep = []
    for i, s in enumerate(streams):
        assert s.dtype == np.uint8 and s.flags.c_contiguous
        keep.append(s)
        arr[i] = s.ctypes.data_as(_u8p)
    return arr, keep


def decode(streams, scales, bits, w, mask, d, m0=0, m1=None):
    m1 = d if m1 is None else m1
    n = len(streams)
    sp, keep = _stream_ptrs(streams)
    sc, scp = _f32(scales)
    b, bp = _u8(bits)
    ww, wp = _f32(w)
    mk, mp = _u8(mask)
    out = np.zeros(m1 - m0, dtype=np.float32)
    lib().agc_oracle_decode_range(n, sp, scp, bp, wp, mp, int(m0), int(m1),
                                  out.ctypes.data_as(_f32p))
    return out


def scales(G, csr, scale_mode):
    G, gp = _f32(G)
    rp, cp, vp = csr.ptrs()
    out = np.zeros(csr.n, dtype=np.float32)
    lib().agc_oracle_scales(csr.n, G.shape[1], gp, G.strides[0] // 4, rp, cp, vp, int(scale_mode),
                            out.ctypes.data_as(_f32p))
    return out


def codes_range(G, csr, i, bits_i, scale_i, seed, step, m0, m1):
    G, gp = _f32(G)
    rp, cp, vp = csr.ptrs()
    out = np.zeros(m1 - m0, dtype=np.uint32)
    lib().agc_oracle_codes_range(gp, G.strides[0] // 4, rp, cp, vp, int(i), int(bits_i),
                                 float(np.float32(scale_i)), int(seed), int(step), int(m0), int(m1),
                                 out.ctypes.data_as(_u32p))
    return out


def worker_moments(G, csr, i, bits_i, scale_i):
    """(sum_m f_i[m]^2, sum_m Var[Q_i(f_i)_m]) in binary64 over all coordinates (b >= 2)."""
    G, gp = _f32(G)
    rp, cp, vp = csr.ptrs()
    ss, vq = C.c_double(), C.c_double()
    rc = lib().agc_oracle_worker_moments(gp, G.strides[0] // 4, rp, cp, vp, int(i), int(bits_i),
                                         float(np.float32(scale_i)), G.shape[1], C.byref(ss), C.byref(vq))
    if rc != 0:
        raise ValueError("worker_moments covers b >= 2 only")
    return float(ss.value), float(vq.value)


def encode_quantize(G, csr, bits, seed, step, scale_mode, scales_in=None):
    """Returns (streams: list of uint8 arrays, scales: float32[n])."""
    G, gp = _f32(G)
    d = G.shape[1]
    rp, cp, vp = csr.ptrs()
    b, bp = _u8(bits)
    streams = [np.zeros(code_bytes(d, int(bi)), dtype=np.uint8) for bi in b]
    sp, keep = _stream_ptrs(streams)
    sc_out = np.zeros(csr.n, dtype=np.float32)
    if scales_in is None:
        sin_p = None
    else:
        sin, sin_p = _f32(scales_in)
    lib().agc_oracle_encode_quantize(csr.n, d, gp, G.strides[0] // 4, rp, cp, vp, bp, int(seed),
                                     int(step), int(scale_mode), sin_p, sp,
                                     sc_out.ctypes.data_as(_f32p))
    return streams, sc_out


def step(G, csr, bits, w, mask, seed, step_, scale_mode):
    """One whole pass.  Returns (streams, scales, ghat)."""
    G, gp = _f32(G)
    d = G.shape[1]
    rp, cp, vp = csr.ptrs()
    b, bp = _u8(bits)
    ww, wp = _f32(w)
    mk, mp = _u8(mask)
    streams = [np.zeros(code_bytes(d, int(bi)), dtype=np.uint8) for bi in b]
    sp, keep = _stream_ptrs(streams)
    sc_out = np.zeros(csr.n, dtype=np.float32)
    ghat = np.zeros(d, dtype=np.float32)
    lib().agc_oracle_step(csr.n, d, gp, G.strides[0] // 4, rp, cp, vp, bp, wp, mp, int(seed),
                          int(step_), int(scale_mode), sp, sc_out.ctypes.data_as(_f32p),
                          ghat.ctypes.data_as(_f32p))
    return streams, sc_out, ghat


# ------------------------------------------------------------------ layer-wise scales
# Sec. II-B applies the quantizer "at layer-wise or bucket-wise granularity": the coded vector is
# cut into consecutive layers and each layer is quantized as a vector of its own, with its own
# scale; the draws stay those of the coordinate's place in the whole vector.  Written out with
# the per-vector routines above: nothing here has arithmetic of its own.
def layer_ranges(ends, d):
    ends = [int(e) for e in ends]
    assert ends and ends[-1] == int(d) and all(b > a for a, b in zip([0] + ends[:-1], ends))
    return list(zip([0] + ends[:-1], ends))


def scales_layers(G, csr, ends, scale_mode=1):
    """(n, n_layers) float32: the scale of f_i inside every layer - its largest magnitude
    (scale_mode 1), or its Euclidean norm with the summation tree started at the layer's first
    coordinate (scale_mode 0): the layer taken as a vector of its own."""
    G, _ = _f32(G)
    ranges = layer_ranges(ends, G.shape[1])
    one = scale_maxabs if int(scale_mode) == 1 else scale_l2
    out = np.zeros((csr.n, len(ranges)), dtype=np.float32)
    for i in range(csr.n):
        for l, (m0, m1) in enumerate(ranges):
            out[i, l] = one(encode(G, csr, i, m0, m1))
    return out


def encode_quantize_layers(G, csr, bits, seed, step_, ends, scales_in=None, scale_mode=1):
    """Streams and (n, n_layers) scales: layer l of worker i is quantized with scale [i, l]."""
    G, _ = _f32(G)
    d = G.shape[1]
    ranges = layer_ranges(ends, d)
    sc = scales_layers(G, csr, ends, scale_mode) if scales_in is None else np.asarray(scales_in, dtype=np.float32)
    streams = []
    for i in range(csr.n):
        codes = np.concatenate([codes_range(G, csr, i, int(bits[i]), sc[i, l], seed, step_, m0, m1)
                                for l, (m0, m1) in enumerate(ranges)])
        streams.append(pack(codes, int(bits[i])))
    return streams, sc


def decode_layers(streams, scales, bits, w, mask, d, ends):
    """scales: (n, n_layers).  Every layer is decoded with its own column of scales."""
    scales = np.asarray(scales, dtype=np.float32)
    return np.concatenate([decode(streams, np.ascontiguousarray(scales[:, l]), bits, w, mask, d, m0, m1)
                           for l, (m0, m1) in enumerate(layer_ranges(ends, d))])


def step_layers(G, csr, bits, w, mask, seed, step_, ends, scale_mode=1):
    """One whole pass with layer-wise scales.  Returns (streams, scales (n, n_layers), ghat)."""
    G, _ = _f32(G)
    streams, sc = encode_quantize_layers(G, csr, bits, seed, step_, ends, scale_mode=scale_mode)
    return streams, sc, decode_layers(streams, sc, bits, w, mask, G.shape[1], ends)
