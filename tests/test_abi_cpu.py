"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before touching a device.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2512_14628_amd as pkg
from paper_2512_14628_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pkg.LIB_PATH):
        pkg.build_library()
    return pkg.load_library()


def test_header_symbols_are_all_exported(lib):
    header = open(os.path.join(ROOT, "include", "hsadmm.h")).read()
    declared = set(re.findall(r"\b(hsadmm_[a-z_]+)\s*\(", header))
    declared -= {"hsadmm_plan_t", "hsadmm_layer_t"}
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    v = pkg.hsadmm_version()                     # major * 10000 + minor * 100 + patch
    assert (v // 10000, v // 100 % 100, v % 100) >= (2, 0, 0) and v // 10000 < 100
    assert pkg.hsadmm_strerror(0) == "ok"
    assert "argument" in pkg.hsadmm_strerror(-1)
    assert "workspace" in pkg.hsadmm_strerror(-2)
    assert "host memory" in pkg.hsadmm_strerror(-5)
    assert pkg.hsadmm_strerror(-99) == "unknown error code"


def _table(rows):
    rows = [tuple(r) + (0,) * (7 - len(r)) for r in rows]       # k_in defaults to 0
    cols = list(zip(*rows))
    return {"elem_off": np.array(cols[0], np.int64), "c_out": np.array(cols[1], np.int32),
            "c_in": np.array(cols[2], np.int32), "khw": np.array(cols[3], np.int32),
            "mode": np.array(cols[4], np.int32), "k": np.array(cols[5], np.int32),
            "k_in": np.array(cols[6], np.int32)}


@pytest.mark.parametrize("rows", [
    [(0, 0, 3, 1, 1, 1)],                       # c_out < 1
    [(0, 4, 3, 0, 1, 1)],                       # khw < 1
    [(0, 4, 3, 1, 5, 1)],                       # unknown mode
    [(0, 4, 3, 1, 1, 0)],                       # k < 1
    [(0, 4, 3, 1, 1, 5)],                       # k > G (filter)
    [(0, 4, 3, 1, 2, 4)],                       # k > G (channel)
    [(2, 4, 3, 1, 1, 1)],                       # elem_off not a multiple of 4
    [(0, 4, 4, 1, 1, 1), (8, 4, 4, 1, 1, 1)],   # layers overlap
    [(-4, 4, 4, 1, 1, 1)],                      # negative offset
    [(0, 4, 3, 1, 3, 2, 0)],                    # both constraints: k_in < 1
    [(0, 4, 3, 1, 3, 2, 4)],                    # both constraints: k_in > c_in
    [(0, 4, 3, 1, 3, 5, 2)],                    # both constraints: k > c_out
    [(0, 4, 3, 1, 4, 2)],                       # mode 4 is not a mode of the library (shape groups go through CHANNEL)
])
def test_plan_create_rejects_bad_tables(lib, rows):
    with pytest.raises(pkg.HsadmmError) as e:
        pkg.Plan(_table(rows))
    assert e.value.code == -1


def test_plan_create_rejects_bad_scalars(lib):
    arr = (binding._Layer * 1)()
    out = ctypes.c_void_p()
    assert lib.hsadmm_plan_create(None, 1, 1, ctypes.byref(out)) == -1
    assert lib.hsadmm_plan_create(arr, 0, 1, ctypes.byref(out)) == -1
    assert lib.hsadmm_plan_create(arr, 1, 0, ctypes.byref(out)) == -1
    assert lib.hsadmm_plan_create(arr, 1, 1, None) == -1
    assert lib.hsadmm_plan_create(arr, 5000, 1, ctypes.byref(out)) == -1
    lib.hsadmm_plan_destroy(None)               # must be a no-op


def test_plan_create_nested_rejects_bad_entries(lib):
    """Runs of channels (hsadmm_nest_t): the table is checked before any device is touched."""
    def create(mode, ci, khw, k, k_in, span, k_coarse):
        arr = (binding._Layer * 1)()
        arr[0].elem_off, arr[0].c_out, arr[0].c_in, arr[0].khw = 0, 8, ci, khw
        arr[0].mode, arr[0].k, arr[0].k_in = mode, k, k_in
        nest = (binding._Nest * 1)()
        nest[0].span, nest[0].k_coarse = span, k_coarse
        out = ctypes.c_void_p()
        return lib.hsadmm_plan_create_nested(arr, nest, 1, 1, ctypes.byref(out))
    for bad in ((1, 36, 1, 4, 0, 9, 2),       # FILTER layers have no channels to nest
                (2, 4, 9, 2, 0, 9, 2),        # not declared through the GEMM view (khw != 1)
                (2, 35, 1, 10, 0, 9, 2),      # c_in not a multiple of span
                (2, 36, 1, 10, 0, 9, 0),      # no run kept
                (2, 36, 1, 10, 0, 9, 5),      # more runs than there are
                (2, 36, 1, 19, 0, 9, 2),      # more columns than the kept runs hold
                (3, 36, 1, 4, 19, 9, 2)):     # the same for the channels of a layer under both constraints
        assert create(*bad) == -1, bad
    out = ctypes.c_void_p()
    assert lib.hsadmm_plan_create_nested(None, None, 1, 1, ctypes.byref(out)) == -1


def test_hot_calls_reject_null_plan(lib):
    assert lib.hsadmm_plan_sizes(None, None, None, None, None) == -1
    assert lib.hsadmm_project(None, None, 1, None, None, None, None, None, None, 0, None) == -1
    assert lib.hsadmm_project_compact(None, None, 1, None, None, None, None, None, None, None, None, None, 0,
                                      None) == -1
    assert lib.hsadmm_project_weighted_compact(None, None, 1, None, None, None, None, None, None, None, None, None,
                                               None, None, 0, None) == -1
    assert lib.hsadmm_project_weighted_frozen(None, None, 1, None, None, None, None, None, None, None) == -1
    assert lib.hsadmm_project_weighted_frozen_compact(None, None, 1, None, None, None, None, None, None, 0, None, None,
                                                      None, None, 0, None) == -1
    assert lib.hsadmm_retrain_project(None, None, 1, None, None, None, None, None, None, 0, None, None, None, None,
                                      None, 0, None) == -1
    assert lib.hsadmm_retrain_expand(None, None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.hsadmm_compact(None, None, None, None, None, None, None, 0, None) == -1
    assert lib.hsadmm_expand(None, None, None, None, None, 0, None) == -1
    assert lib.hsadmm_project_frozen(None, None, 1, None, None, None, None, None) == -1
    assert lib.hsadmm_project_frozen_compact(None, None, 1, None, None, None, None, 0, None, None, None, None, 0,
                                             None) == -1
    assert lib.hsadmm_mask_or(None, None, 1, None, None) == -1
    assert lib.hsadmm_average(None, None, 1, 0, None, None) == -1
    assert lib.hsadmm_dual_inter(None, None, None, None, None) == -1
    assert lib.hsadmm_compact_sum(None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.hsadmm_kernel_timing_enable(None, 1) == -1
    names = [lib.hsadmm_kernel_name(i).decode() for i in range(binding.KERNEL_COUNT)]
    assert all(names) and len(set(names)) == len(names) and lib.hsadmm_kernel_name(binding.KERNEL_COUNT) == b""
    header = open(os.path.join(ROOT, "include", "hsadmm.h")).read()
    assert int(re.search(r"#define HSADMM_KERNEL_COUNT (\d+)", header).group(1)) == binding.KERNEL_COUNT


def test_no_cpu_fallback_in_the_product_package():
    """The product path must not import the oracle (or numpy-level arithmetic) anywhere."""
    for fn in ("__init__.py", "binding.py"):
        src = open(os.path.join(ROOT, "paper_2512_14628_amd", fn)).read()
        assert "oracle" not in src.replace("no CPU fallback", "")
    csrc = os.path.join(ROOT, "paper_2512_14628_amd", "csrc")
    for fn in os.listdir(csrc):
        assert "oracle" not in open(os.path.join(csrc, fn)).read(), fn


def test_node_coefficients_host_function_against_eq_9_in_exact_arithmetic(lib):
    """hsadmm_node_coefficients runs on the host (no device needed).  Its fp32 weights are checked against Eq. (9)
    itself, a = P rho_1 / gamma and b = rho_2 / gamma with gamma = lambda / M + P rho_1 + rho_2, evaluated in exact
    rational arithmetic from the same float64 inputs -- not against the oracle's function: the product's result must
    be the correctly rounded float of the exact value, or its neighbour when the float64 evaluation lands within its
    own rounding error of a float tie."""
    from fractions import Fraction
    rng = np.random.default_rng(1)
    r1, r2 = rng.uniform(1e-4, 10, 40), rng.uniform(0, 10, 40)
    r1[:3], r2[:3] = (1.5e-3, 10.0, 2.0 ** -20), (1.5e-4, 0.0, 10.0)      # the paper's initial penalties, edge cases
    for lam, M, P in ((1e-4, 16, 4), (0.0, 1, 1), (3e-2, 64, 8), (5e-4, 3, 7)):
        a, b = pkg.hsadmm_node_coefficients(r1, r2, lam, M, P)
        for l in range(len(r1)):
            gamma = Fraction(float(lam)) / M + P * Fraction(float(r1[l])) + Fraction(float(r2[l]))
            for got, exact in ((a[l], P * Fraction(float(r1[l])) / gamma), (b[l], Fraction(float(r2[l])) / gamma)):
                got32 = np.float32(got)
                assert float(got32) == got
                lo, hi = np.nextafter(got32, np.float32(-1)), np.nextafter(got32, np.float32(2))
                half_lo = (Fraction(float(lo)) + Fraction(float(got32))) / 2
                half_hi = (Fraction(float(hi)) + Fraction(float(got32))) / 2
                slack = abs(exact) * Fraction(1, 2 ** 50)
                assert half_lo - slack <= exact <= half_hi + slack, (lam, M, P, l)
            assert abs((Fraction(a[l]) + Fraction(b[l])) - (1 - Fraction(float(lam)) / M / gamma)) < Fraction(1, 2 ** 22)
    # lambda = 0, rho_2 = 0: the plain mean (a = 1, b = 0), whatever rho_1 and P are
    a, b = pkg.hsadmm_node_coefficients([0.3, 7.0], [0.0, 0.0], 0.0, 5, 8)
    assert a == [1.0, 1.0] and b == [0.0, 0.0]
    # rejected before anything is written: gamma = 0, a negative penalty (also in a later layer), NaN
    for bad1, bad2 in (([0.0], [0.0]), ([-1.0], [3.0]), ([1.0, 1.0], [1.0, -2.0]), ([float("nan")], [1.0])):
        with pytest.raises(pkg.HsadmmError):
            pkg.hsadmm_node_coefficients(bad1, bad2, 0.0, 1, 1)
    out_a = (ctypes.c_float * 2)(7.0, 7.0)
    out_b = (ctypes.c_float * 2)(7.0, 7.0)
    r1c, r2c = (ctypes.c_double * 2)(1.0, 1.0), (ctypes.c_double * 2)(1.0, -2.0)
    assert lib.hsadmm_node_coefficients(r1c, r2c, 2, 0.0, 1, 1, out_a, out_b) == -1
    assert list(out_a) == [7.0, 7.0] and list(out_b) == [7.0, 7.0]
    assert lib.hsadmm_node_coefficients(None, r2c, 2, 0.0, 1, 1, out_a, out_b) == -1
    assert lib.hsadmm_node_coefficients(r1c, r1c, 2, 0.0, 0, 1, out_a, out_b) == -1


def test_adapt_penalties_host_function_matches_the_oracle(lib):
    """hsadmm_adapt_penalties runs on the host: the same decisions, penalties and dual factors as the oracle's rule,
    bit for bit, on random residual sums (many of them placed on or next to the rule's two boundaries)."""
    import oracle
    rng = np.random.default_rng(8)
    for trial in range(40):
        L = int(rng.integers(1, 60))
        P, n_out = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        mu = float(rng.choice([2.0, 10.0, 16.0]))
        ti, td = float(rng.choice([1.0, 1.5, 2.0])), float(rng.choice([1.0, 2.0, 3.0]))
        rho1 = 2.0 ** rng.integers(-12, 3, L).astype(np.float64)
        rho2 = 2.0 ** rng.integers(-14, 3, L).astype(np.float64)
        sq = 10.0 ** rng.uniform(-9, 2, (4, L))
        # boundary cases: ||r|| = mu ||s|| exactly representable, then nudged to either side
        for l in range(0, L, 3):
            s_raw = 4.0 ** float(rng.integers(-8, 2))
            sq[1, l] = s_raw / P
            sq[0, l] = (mu * rho1[l]) ** 2 * s_raw * (1.0 + float(rng.integers(-1, 2)) * 2.0 ** -50)
        sq[:, L - 1] = 0.0
        got = pkg.hsadmm_adapt_penalties(sq, rho1, rho2, P, n_out, mu, ti, td, 10.0, 10.0)
        want = oracle.adapt_penalties(sq, rho1, rho2, P, n_out, mu, ti, td, 10.0, 10.0)
        for g, w, dt in zip(got, want, (np.float64, np.float64, np.float32, np.float32)):
            assert np.array_equal(np.array(g, dt), w), trial
    ok = ([[1.0], [1.0], [1.0], [1.0]], [1.0], [1.0], 2, 1, 10.0, 2.0, 2.0, 10.0, 10.0)
    for pos, bad in ((1, [0.0]), (1, [11.0]), (2, [float("nan")]), (3, 0), (4, 0), (5, 0.0), (6, 0.5), (7, 0.99),
                     (0, [[1.0], [-1.0], [1.0], [1.0]])):
        args = list(ok)
        args[pos] = bad
        with pytest.raises(pkg.HsadmmError):
            pkg.hsadmm_adapt_penalties(*args)
    assert lib.hsadmm_adapt_penalties(None, 1, 1, 1, 10.0, 2.0, 2.0, 10.0, 10.0, None, None, None, None) == -1
    assert lib.hsadmm_scale_layers(None, None, None, None) == -1


def test_stopping_test_host_function_against_the_printed_thresholds_and_the_oracle(lib):
    """hsadmm_stopping_test runs on the host: checked against the thresholds written out in exact rational arithmetic
    on cases whose roots are exact (powers of two), including both boundaries, and against the oracle's decisions on
    random inputs that are not within rounding of a boundary."""
    import oracle
    from fractions import Fraction
    # one layer, n = 8, P = 1, n_out = 1: p = 16; eps_abs = 1 -> absolute part 4; eps_rel = 1/4
    # magnitudes: theta 48, z_i 16, z 9, u 4, v 1; rho_1 = 2, rho_2 = 4
    #   ||A x|| = sqrt(64) = 8, ||B z|| = sqrt(16 + 9) = 5 -> eps_pri = 4 + 2 = 6
    #   ||A^T y|| = sqrt(4 * 4 + 16 * 1) = sqrt(32): not exact; take u = 9, v = 4: sqrt(36 + 64) = 10 -> eps_dual = 6.5
    mag = [[48.0], [16.0], [9.0], [9.0], [4.0]]
    done, every = pkg.hsadmm_stopping_test([8], 1, 1, [2.0], [4.0], [[20.0], [0.0], [16.0], [0.0]], mag, 1.0, 0.25)
    assert done == [0] and not every                          # R_pri = 6 = eps_pri, and 6 < 6 is false
    done, every = pkg.hsadmm_stopping_test([8], 1, 1, [2.0], [4.0], [[20.0], [0.0], [15.0], [0.0]], mag, 1.0, 0.25)
    assert done == [1] and every                              # sqrt(35) < 6
    # dual side: R_dual^2 = 1 * 4 * sq_1 + 1 * 16 * sq_3; sq_1 = 4, sq_3 = 1.640625 -> 16 + 26.25 = 42.25 = 6.5^2
    done, _ = pkg.hsadmm_stopping_test([8], 1, 1, [2.0], [4.0], [[0.0], [4.0], [0.0], [1.640625]], mag, 1.0, 0.25)
    assert done == [0]                                        # 6.5 < 6.5 is false
    done, _ = pkg.hsadmm_stopping_test([8], 1, 1, [2.0], [4.0], [[0.0], [4.0], [0.0], [1.64]], mag, 1.0, 0.25)
    assert done == [1]
    assert Fraction(4 * 4) + Fraction(16) * Fraction(1.640625) == Fraction(13, 2) ** 2
    rng = np.random.default_rng(15)
    for trial in range(60):
        L = int(rng.integers(1, 30))
        P, n_out = int(rng.integers(1, 9)), int(rng.integers(1, 4))
        n = rng.integers(1, 10 ** 7, L)
        rho1, rho2 = 10.0 ** rng.uniform(-3, 1, L), 10.0 ** rng.uniform(-4, 1, L)
        sq, mag = 10.0 ** rng.uniform(-8, 2, (4, L)), 10.0 ** rng.uniform(-2, 4, (5, L))
        ea, er = float(10.0 ** rng.uniform(-6, -2)), float(10.0 ** rng.uniform(-5, -1))
        got, got_all = pkg.hsadmm_stopping_test(n, P, n_out, rho1, rho2, sq, mag, ea, er)
        want, want_all = oracle.stopping_test(n, P, n_out, rho1, rho2, sq, mag, ea, er)
        # (a margin of 1e-12 around either threshold: the two sides may group the products differently)
        r_pri, r_dual = np.sqrt(sq[0] + sq[2]), np.sqrt(P * rho1 ** 2 * sq[1] + n_out * rho2 ** 2 * sq[3])
        root_p = np.sqrt((P + 1.0) * n * n_out)
        e_pri = root_p * ea + er * np.maximum(np.sqrt(mag[0] + mag[1]), np.sqrt(P * mag[1] + n_out * mag[2]))
        e_dual = root_p * ea + er * np.sqrt(rho1 ** 2 * mag[3] + rho2 ** 2 * mag[4])
        clear = (np.abs(r_pri - e_pri) > 1e-12 * e_pri) & (np.abs(r_dual - e_dual) > 1e-12 * e_dual)
        assert np.array_equal(np.array(got)[clear], want[clear]), trial
        if clear.all():
            assert got_all == want_all
    ok = dict(n_elems=[4], P=1, n_out=1, rho1=[1.0], rho2=[1.0], residuals=[[0.0]] * 4, magnitudes=[[1.0]] * 5,
              eps_abs=1e-3, eps_rel=1e-3)
    assert pkg.hsadmm_stopping_test(**ok) == ([1], True)
    for key, bad in (("P", 0), ("n_out", 0), ("rho1", [0.0]), ("rho2", [-1.0]), ("eps_abs", -1.0),
                     ("eps_rel", float("nan")), ("n_elems", [0]), ("residuals", [[-1.0]] * 4),
                     ("magnitudes", [[float("nan")]] * 5)):
        args = dict(ok)
        args[key] = bad
        with pytest.raises(pkg.HsadmmError):
            pkg.hsadmm_stopping_test(**args)
    assert lib.hsadmm_stopping_test(None, 1, 1, 1, None, None, None, None, 0.0, 0.0, None, None) == -1
    assert lib.hsadmm_layer_sqnorms(None, None, None, None, 0, None) == -1


def test_step_argument_structure_has_the_layout_the_binding_fills(tmp_path):
    """hsadmm_step_args_t as a C compiler lays it out (size and the offset of every field, printed by a small program
    built from include/hsadmm.h) against the ctypes structure the binding generates from its field table."""
    import subprocess
    fields = [name for name, _, _ in binding._STEP_FIELDS]
    src = ["#include <stdio.h>", "#include <stddef.h>", '#include "hsadmm.h"', "int main(void) {",
           '  printf("%zu\\n", sizeof(hsadmm_step_args_t));']
    src += ['  printf("%%zu\\n", offsetof(hsadmm_step_args_t, %s));' % f for f in fields]
    src += ["  return 0;", "}"]
    c = tmp_path / "layout.c"
    c.write_text("\n".join(src))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(c), "-o", str(exe)])
    out = [int(x) for x in subprocess.check_output([str(exe)], text=True).split()]
    assert out[0] == ctypes.sizeof(binding._StepArgs)
    assert out[1:] == [getattr(binding._StepArgs, f).offset for f in fields]
    # every field of the header's structure is in the table (a field the binding forgot would shift nothing but stay NULL)
    header = open(os.path.join(ROOT, "include", "hsadmm.h")).read()
    body = header[header.index("typedef struct {\n    size_t struct_bytes;"):header.index("} hsadmm_step_args_t;")]
    declared = re.findall(r"([A-Za-z_0-9]+);", body)
    assert declared == fields
    # a structure of another size is refused before anything is read from it
    args = binding._StepArgs()
    args.struct_bytes = ctypes.sizeof(binding._StepArgs) - 8
    assert lib_handle().hsadmm_step(ctypes.c_void_p(1), ctypes.byref(args)) == -1
    assert lib_handle().hsadmm_step(None, ctypes.byref(args)) == -1


def lib_handle():
    return pkg.load_library()


def test_bench_refuses_more_than_one_gpu():
    """This build has no collectives: bench.py --gpus N with N > 1 exits with a message instead of running."""
    import subprocess
    import sys
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "4"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *argv], env=env, capture_output=True,
                           text=True, timeout=120)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
