"""Exercises every host-side design routine of csrc/agc_host.cpp through a library given on the
command line (the sanitizer leg builds that source with g++ -fsanitize=address,undefined).  Run
as a script in a process of its own: a sanitizer report ends it with a non-zero status."""
import ctypes as C
import sys

import numpy as np


def main(path):
    L = C.CDLL(path)
    f64p, u8p, i32p, f32p = (C.POINTER(C.c_double), C.POINTER(C.c_uint8), C.POINTER(C.c_int32), C.POINTER(C.c_float))
    L.agc_phi_coef_balanced.restype = C.c_double
    L.agc_phi_coef_balanced.argtypes = [C.c_int, f64p, C.c_int]
    L.agc_alloc_objective.restype = C.c_double
    L.agc_alloc_objective.argtypes = [C.c_int, f64p, C.c_double, u8p]
    for fn in (L.agc_alloc_bits, L.agc_alloc_bits_dp):
        fn.argtypes = [C.c_int, f64p, C.c_double, C.c_int, C.c_int, C.c_int, u8p]
    L.agc_build_code.argtypes = [C.c_int, C.c_int, f64p, u8p, C.c_double, i32p, i32p, f32p, f32p, C.c_int, C.POINTER(C.c_int)]
    L.agc_build_cyclic_code.argtypes = [C.c_int, C.c_int, C.c_int, f64p, u8p, C.c_double, i32p, i32p, f32p, f32p]
    L.agc_build_cyclic_code_opt.argtypes = [C.c_int, C.c_int, C.c_int, f64p, u8p, C.c_double, i32p, i32p, f32p, f32p,
                                            f64p, C.POINTER(C.c_int)]
    L.agc_check_unbiased.argtypes = [C.c_int, C.c_int, i32p, i32p, f32p, f32p, f64p, C.c_double, f64p]
    L.agc_second_moment_decoder.argtypes = [C.c_int, C.c_int, i32p, i32p, f32p, f64p, u8p, C.c_double, C.c_double, f32p]

    def ptr(a, t):
        return a.ctypes.data_as(t)

    rng = np.random.default_rng(5)
    calls = 0
    for n, k in [(1, 1), (2, 5), (5, 2), (7, 7), (16, 16), (64, 64), (256, 256), (256, 3)]:
        p = rng.uniform(0.05, 0.6, n)
        z_tot = int(rng.integers(2 * n, 8 * n + 1))
        pc = L.agc_phi_coef_balanced(n, ptr(p, f64p), z_tot)
        bits = np.zeros(n, np.uint8)
        assert L.agc_alloc_bits(n, ptr(p, f64p), pc, z_tot, 2, 8, ptr(bits, u8p)) == 0 and int(bits.sum()) == z_tot
        bits_dp = np.zeros(n, np.uint8)
        assert L.agc_alloc_bits_dp(n, ptr(p, f64p), pc, z_tot, 2, 8, ptr(bits_dp, u8p)) == 0
        assert L.agc_alloc_objective(n, ptr(p, f64p), pc, ptr(bits, u8p)) <= L.agc_alloc_objective(
            n, ptr(p, f64p), pc, ptr(bits_dp, u8p)) * (1 + 1e-12)
        # infeasible budgets are refused, nothing is written past the arrays
        assert L.agc_alloc_bits(n, ptr(p, f64p), pc, 2 * n - 1, 2, 8, ptr(bits_dp, u8p)) != 0
        assert L.agc_alloc_bits_dp(n, ptr(p, f64p), pc, 8 * n + 1, 2, 8, ptr(bits_dp, u8p)) != 0
        cap = n + k - 1                                    # exactly the bound of the construction
        row_ptr, col, val, w = np.zeros(n + 1, np.int32), np.zeros(cap, np.int32), np.zeros(cap, np.float32), np.zeros(n, np.float32)
        nnz = C.c_int()
        assert L.agc_build_code(n, k, ptr(p, f64p), ptr(bits, u8p), pc, ptr(row_ptr, i32p), ptr(col, i32p),
                                ptr(val, f32p), ptr(w, f32p), cap, C.byref(nnz)) == 0 and nnz.value <= cap
        res = C.c_double()
        assert L.agc_check_unbiased(n, k, ptr(row_ptr, i32p), ptr(col, i32p), ptr(val, f32p), ptr(w, f32p),
                                    ptr(p, f64p), 1e-5, C.byref(res)) == 0, res.value
        v = np.zeros(n, np.float32)
        assert L.agc_second_moment_decoder(n, k, ptr(row_ptr, i32p), ptr(col, i32p), ptr(val, f32p), ptr(p, f64p),
                                           ptr(bits, u8p), pc, 1.5, ptr(v, f32p)) == 0
        if nnz.value > 1:                                  # a capacity that is too small is an error, not an overflow
            small = nnz.value - 1
            c2, v2 = np.zeros(small, np.int32), np.zeros(small, np.float32)
            assert L.agc_build_code(n, k, ptr(p, f64p), ptr(bits, u8p), pc, ptr(row_ptr, i32p), ptr(c2, i32p),
                                    ptr(v2, f32p), ptr(w, f32p), small, C.byref(nnz)) != 0
        if n == k:
            for s in sorted({1, min(3, k), min(8, k), k if k <= 16 else 4}):
                rp, cc, vv = np.zeros(n + 1, np.int32), np.zeros(n * s, np.int32), np.zeros(n * s, np.float32)
                assert L.agc_build_cyclic_code(n, k, s, ptr(p, f64p), ptr(bits, u8p), pc, ptr(rp, i32p), ptr(cc, i32p),
                                               ptr(vv, f32p), ptr(w, f32p)) == 0
                obj, reach = C.c_double(), C.c_int()
                assert L.agc_build_cyclic_code_opt(n, k, s, ptr(p, f64p), ptr(bits, u8p), pc, ptr(rp, i32p),
                                                   ptr(cc, i32p), ptr(vv, f32p), ptr(w, f32p), C.byref(obj),
                                                   C.byref(reach)) == 0
                assert L.agc_check_unbiased(n, k, ptr(rp, i32p), ptr(cc, i32p), ptr(vv, f32p), ptr(w, f32p),
                                            ptr(p, f64p), 1e-5, C.byref(res)) == 0, res.value
        calls += 1
    print(f"host routines ok on {calls} shapes")


if __name__ == "__main__":
    main(sys.argv[1])
