"""CPU-only checks of the built library: it loads, exports every symbol the header declares,
and its host-side design routines agree with the oracle's binary64 versions."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import agc_oracle as O
from oracle import design as D
from paper_2605_15890_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for header in ("agc.h", "agc_debug.h"):        # the method's ABI, and the measurement/testing hooks
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(agc_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_method_header_declares_no_measurement_hooks():
    text = open(os.path.join(ROOT, "include", "agc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for name in ("agc_profile_enable", "agc_profile_read", "agc_calibration_copy", "agc_debug_stream_rows"):
        assert name not in text


def test_library_exports_every_declared_symbol():
    lib = api.load()
    names = _declared_symbols()
    assert len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(api.EXPORTS) == names


def test_code_bytes_matches_payload_definition():
    for d in (1, 127, 128, 129, 4096, 25_600_000):
        for b in range(1, 17):
            assert api.agc_code_bytes(d, b) == -(-d // 128) * 16 * b == O.code_bytes(d, b)
    assert api.agc_code_bytes(0, 4) == 0 and api.agc_code_bytes(10, 17) == 0


def test_create_rejects_bad_shapes_without_touching_the_gpu():
    lib = api.load()
    h = ctypes.c_void_p()
    for n, k, d in [(0, 4, 16), (257, 4, 16), (4, 0, 16), (4, 4, 0), (4, 4, (1 << 33) + 1)]:
        assert lib.agc_create(ctypes.byref(h), n, k, d, None) == api.AGC_ESHAPE
        assert not h.value
    assert lib.agc_create(None, 4, 4, 16, None) == api.AGC_EINVAL
    bad = api.AgcOpts(7, 0, 0, 0, 0, (ctypes.c_int * 3)())
    assert lib.agc_create(ctypes.byref(h), 4, 4, 16, ctypes.byref(bad)) == api.AGC_EINVAL
    bad = api.AgcOpts(api.AGC_SCALE_MAXABS, 0, 0, 512, 0, (ctypes.c_int * 3)())     # only 256-coordinate buckets
    assert lib.agc_create(ctypes.byref(h), 4, 4, 16, ctypes.byref(bad)) == api.AGC_EINVAL


def test_noalloc_decode_rejects_sizes_beyond_its_fixed_scratch_without_touching_the_gpu():
    lib = api.load()
    n = api.AGC_MAX_WORKERS + 1
    ptrs = (ctypes.c_void_p * n)()
    bits = np.full(n, 4, np.uint8)
    w = np.ones(n, np.float32)
    mask = np.ones(n, np.uint8)
    args = (ptrs, ctypes.c_void_p(0), bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
            w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
            ctypes.c_void_p(0), ctypes.c_void_p(0))
    assert lib.agc_decode_noalloc(n, 1024, 0, *args) == api.AGC_ESHAPE
    msg = lib.agc_last_error(None).decode()
    assert "257" in msg and "256" in msg, msg
    assert lib.agc_decode_noalloc(0, 1024, 0, *args) == api.AGC_ESHAPE
    assert lib.agc_decode_noalloc(4, 0, 0, *args) == api.AGC_ESHAPE
    assert lib.agc_decode_noalloc(4, 1024, 0, *args) == api.AGC_EINVAL      # null scales / estimate


def test_phi_coef_balanced():
    rng = np.random.default_rng(0)
    p = rng.uniform(0.05, 0.6, 16)
    assert api.agc_phi_coef_balanced(p, 64) == pytest.approx(D.phi_coef_balanced(p, 64), rel=1e-14)


def test_dp_allocator_is_optimal():
    rng = np.random.default_rng(1)
    for _ in range(20):
        n = int(rng.integers(2, 6))
        p = rng.uniform(0.02, 0.7, n)
        z_total = 2 * n + int(rng.integers(0, 9))
        pc = 10 ** rng.uniform(-2, 2)
        bits = api.agc_alloc_bits_dp(p, pc, z_total, 2, 8)
        assert bits.sum() == z_total and bits.min() >= 2 and bits.max() <= 8
        r_bf, f_bf = D.alloc_bruteforce(p, pc, z_total - 2 * n, 6)
        assert api.agc_alloc_objective(p, pc, bits) == pytest.approx(f_bf, rel=1e-12)
        assert D.objective(p, bits.astype(int) - 2, pc) == pytest.approx(f_bf, rel=1e-12)


def test_low_complexity_allocator_near_optimal_and_feasible():
    rng = np.random.default_rng(2)
    worst = 1.0
    for trial in range(40):
        n = int(rng.integers(3, 65))
        p = rng.uniform(0.05, 0.6, n)
        z_total = 2 * n + int(rng.integers(1, 4 * n))
        pc = api.agc_phi_coef_balanced(p, z_total) if trial % 2 else 10 ** rng.uniform(-1, 2)
        bits = api.agc_alloc_bits(p, pc, z_total, 2, 8)
        assert bits.sum() == z_total and bits.min() >= 2 and bits.max() <= 8
        f = api.agc_alloc_objective(p, pc, bits)
        f_dp = api.agc_alloc_objective(p, pc, api.agc_alloc_bits_dp(p, pc, z_total, 2, 8))
        assert f <= f_dp * (1 + 1e-12)
        worst = min(worst, f / f_dp)
        if n <= 10:   # the oracle's own reading of Algorithm 1 reaches the same utility
            _, f_or = D.alloc_lowcomplexity(p, pc, z_total - 2 * n, 6)
            assert f == pytest.approx(f_or, rel=1e-9)
    assert worst >= 1 - 1e-3


def test_allocator_argument_errors():
    p = np.array([0.1, 0.2])
    with pytest.raises(api.AgcError) as e:
        api.agc_alloc_bits(p, 1.0, 3, 2, 8)          # below n * z_min
    assert e.value.status == api.AGC_EBITS
    with pytest.raises(api.AgcError):
        api.agc_alloc_bits(p, 1.0, 17, 2, 8)         # above n * z_max
    with pytest.raises(api.AgcError):
        api.agc_alloc_bits(p, 1.0, 6, 1, 8)          # z_min below the paper's minimum of 2
    with pytest.raises(api.AgcError):
        api.agc_alloc_bits(np.array([0.1, 1.0]), 1.0, 6, 2, 8)


@pytest.mark.parametrize("n,k", [(3, 3), (5, 8), (8, 5), (64, 64)])
def test_interval_code_matches_oracle(n, k):
    rng = np.random.default_rng(n + k)
    p = rng.uniform(0.05, 0.6, n)
    bits = rng.integers(2, 9, n).astype(np.uint8)
    pc = 0.3
    row_ptr, col, val, w = api.agc_build_code(n, k, p, bits, pc)
    alpha = D.interval_code(D.row_targets(D.c_weights(p, bits, pc), k), k)
    dense = O.Csr(row_ptr, col, val, k).dense()
    keep = alpha > 1e-9          # the library moves segment ends at rounding distance onto the boundary
    assert np.allclose(dense, alpha, atol=1e-6)
    assert np.all(dense[keep] > 0)
    assert len(col) <= n + k - 1                                  # Sec. III-A: at most n + k - 1 entries
    assert np.all(val > 1e-11 * k)                                # no entry at rounding level
    assert np.allclose(dense.astype(np.float64).sum(axis=0), 1.0, atol=2e-7)


@pytest.mark.parametrize("n,k", [(4, 4), (6, 12), (12, 6), (64, 64), (256, 256)])
def test_interval_code_of_equal_workers_has_no_slivers(n, k):
    """Equal workers have equal segments whose ends fall on partition boundaries wherever
    i*k/n is an integer; the running sum misses those by rounding, and the construction must
    not turn the miss into stored entries: exactly as many entries as the exact-arithmetic
    construction has (Sec. III-A), n = k giving the identity."""
    from fractions import Fraction
    p = np.full(n, 0.3)
    bits = np.full(n, 3, np.uint8)
    row_ptr, col, val, w = api.agc_build_code(n, k, p, bits, 0.7)
    exact = 0
    for i in range(n):
        lo, hi = Fraction(i * k, n), Fraction((i + 1) * k, n)
        exact += sum(1 for j in range(k) if min(hi, j + 1) - max(lo, j) > 0)
    assert len(col) == exact
    if n == k:
        assert np.array_equal(col, np.arange(n)) and np.array_equal(val, np.ones(n, np.float32))
    ctx_shape_ok = all(row_ptr[i + 1] - row_ptr[i] <= 8 for i in range(n))
    assert ctx_shape_ok
    assert np.allclose(w, 1 / (1 - p), rtol=1e-6)
    for i in range(n):   # columns ascending inside a row
        c = col[row_ptr[i]:row_ptr[i + 1]]
        assert np.all(np.diff(c) > 0)
    ok, res = api.agc_check_unbiased(k, row_ptr, col, val, w, p, 1e-5)
    assert ok and res < 1e-5
    val_bad = val.copy()
    val_bad[0] *= 1.5
    ok, res = api.agc_check_unbiased(k, row_ptr, col, val_bad, w, p, 1e-5)
    assert not ok and res > 1e-3


def test_cyclic_code_matches_oracle():
    rng = np.random.default_rng(5)
    for n, s in [(4, 2), (16, 3), (64, 4), (5, 5), (6, 1)]:
        p = rng.uniform(0.05, 0.6, n)
        bits = rng.integers(2, 9, n).astype(np.uint8)
        row_ptr, col, val, w = api.agc_build_cyclic_code(n, n, s, p, bits, 0.2)
        alpha, supp = D.cyclic_code(D.c_weights(p, bits, 0.2), n, s)
        assert np.array_equal(row_ptr, np.arange(n + 1) * s)
        assert np.array_equal(col.reshape(n, s), np.array(supp))
        assert np.allclose(val.reshape(n, s), [[alpha[i, j] for j in supp[i]] for i in range(n)], rtol=1e-6)
        ok, res = api.agc_check_unbiased(n, row_ptr, col, val, w, p, 1e-5)
        assert ok
    with pytest.raises(api.AgcError):
        api.agc_build_cyclic_code(4, 5, 2, [0.1] * 4, [2] * 4, 0.2)


def test_second_moment_decoder_matches_oracle_and_beats_unbiased_decoder():
    """Closed form of the two-track decoder (Sec. V): the host routine against the oracle's
    formula (itself pinned by numerical minimisation), and Proposition 3's dominance."""
    rng = np.random.default_rng(23)
    for n, s in [(4, 2), (16, 3), (64, 4)]:
        p = rng.uniform(0.05, 0.6, n)
        bits = rng.integers(2, 9, n).astype(np.uint8)
        row_ptr, col, val, w = api.agc_build_cyclic_code(n, n, s, p, bits, 0.2)
        B = np.zeros((n, n))
        for i in range(n):
            B[i, col[row_ptr[i]:row_ptr[i + 1]]] = val[row_ptr[i]:row_ptr[i + 1]]
        for lam in (0.05, 1.0, 50.0):
            v = api.agc_second_moment_decoder(n, row_ptr, col, val, p, bits, 0.2, lam)
            v_o = D.second_moment_decoder(p, bits, 0.2, B, lam)
            assert np.allclose(v, v_o, rtol=2e-7 * 4, atol=0)
            m_v = D.second_moment_objective(v.astype(np.float64), p, bits, 0.2, B, lam)
            m_w = D.second_moment_objective(w.astype(np.float64), p, bits, 0.2, B, lam)
            assert m_v <= m_w
            var = lambda u: D.second_moment_objective(u, p, bits, 0.2, B, 0.0)      # variance part alone
            assert var(v.astype(np.float64)) <= var(w.astype(np.float64)) * (1 + 1e-6)
    with pytest.raises(api.AgcError):
        api.agc_second_moment_decoder(4, [0, 1, 2, 3, 4], [0, 1, 2, 3], [1, 1, 1, 1], [0.1] * 4, [4] * 4, 0.2, 0.0)


def test_optimal_cyclic_code_matches_the_oracle_optimum():
    """Support-restricted structure problem: the library's column-wise minimisation against the
    oracle's library solver (objective), Theorem 1's value when the support admits it, and the
    unbiasedness condition; never worse than the column-normalised heuristic."""
    rng = np.random.default_rng(41)
    saw_bound, saw_gap = False, False
    for n, s in [(6, 6), (10, 2), (10, 3), (16, 3), (12, 1), (24, 4)]:
        p = rng.uniform(0.02, 0.7, n)
        bits = rng.integers(2, 9, n).astype(np.uint8)
        c = D.c_weights(p, bits, 0.3)
        row_ptr, col, val, w, obj, reach = api.agc_build_cyclic_code_opt(n, n, s, p, bits, 0.3)
        assert np.array_equal(row_ptr, np.arange(n + 1) * s)
        assert np.array_equal(col.reshape(n, s), np.array(D.cyclic_support(n, n, s)))
        ok, res = api.agc_check_unbiased(n, row_ptr, col, val, w, p, 1e-5)
        assert ok, res
        a_o, _ = D.cyclic_code_optimal(c, n, s)
        obj_o = D.csp2_objective(c, a_o)
        assert obj <= obj_o * (1 + 1e-7), (n, s, obj, obj_o)           # at least as good as the library solver
        assert obj >= n * n / np.sum(1 / c) * (1 - 1e-12)              # and never below Theorem 1's value
        alpha = np.zeros((n, n))
        for i in range(n):
            alpha[i, col[row_ptr[i]:row_ptr[i + 1]]] = val[row_ptr[i]:row_ptr[i + 1]]
        assert abs(D.csp2_objective(c, alpha) - obj) <= 1e-5 * obj     # the float32 entries carry that objective
        heur = D.csp2_objective(c, D.cyclic_code(c, n, s)[0])
        assert obj <= heur * (1 + 1e-12)
        feasible, _ = D.cyclic_row_sum_feasible(c, n, s)
        assert reach == feasible
        if reach:
            saw_bound = True
            assert np.allclose(alpha.sum(axis=1), D.row_targets(c, n), rtol=1e-5)
        else:
            saw_gap = True
    assert saw_bound and saw_gap
    with pytest.raises(api.AgcError):
        api.agc_build_cyclic_code_opt(4, 5, 2, [0.1] * 4, [2] * 4, 0.2)


def test_public_headers_compile_as_plain_c_and_as_cpp(tmp_path):
    """The boundary is a C ABI: both headers must be valid C99 (no C++-isms outside the extern "C"
    guards) and valid C++, on their own, with warnings as errors."""
    import shutil
    import subprocess
    inc = os.path.join(ROOT, "include")
    src_c = tmp_path / "use_headers.c"
    src_c.write_text('#include "agc.h"\n#include "agc_debug.h"\n'
                     'static agc_opts o;\nint use(void) { agc_ctx *c = 0; (void)c; return o.bucket + AGC_MAX_LAYERS + AGC_NUM_KERNELS; }\n')
    src_cpp = tmp_path / "use_headers.cpp"
    src_cpp.write_text(src_c.read_text())
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    assert gcc and gxx
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src_c)],
                   check=True)
    subprocess.run([gxx, "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src_cpp)],
                   check=True)
    # each header also stands alone
    for h in ("agc.h", "agc_debug.h"):
        one = tmp_path / ("only_" + h.replace(".h", ".c"))
        one.write_text(f'#include "{h}"\nint main(void) {{ return 0; }}\n')
        subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(one)], check=True)
