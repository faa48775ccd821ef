"""CPU sanitizer leg: the oracle built with -fsanitize=address,undefined, and the host code of the HIP library built
with -fsanitize=undefined, into a temporary directory and exercised in a child process (the sanitizer runtimes have
to be loaded before Python's own allocations, hence the preload).  Any report of a sanitizer fails the child.
(The library's host code goes without the address sanitizer: a process that holds both its shadow memory and the
HIP runtime, which libhsadmm.so links, does not get through loading in any reasonable time.)"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(compiler, name):
    path = subprocess.check_output([compiler, "-print-file-name=" + name], text=True).strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("%s is not installed with %s" % (name, compiler))
    return path


def _child_env(runtimes, extra):
    env = dict(os.environ)
    preload = list(runtimes)
    if env.get("LD_PRELOAD"):
        preload.append(env["LD_PRELOAD"])           # whatever is preloaded already stays
    env["LD_PRELOAD"] = ":".join(preload)
    # Python itself is not instrumented: its interned objects look like leaks, and the runtime cannot be first in
    # the link order of an executable that was not built with it
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def test_the_oracle_pins_hold_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    so = str(tmp_path / "libhsadmm_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-o", so,
                           os.path.join(ROOT, "oracle", "hsadmm_oracle.c"), "-lm"])
    pins = ["test_oracle_pins.py", "test_oracle_frozen.py", "test_oracle_weighted.py", "test_oracle_residuals.py",
            "test_oracle_composite.py", "test_oracle_shape.py", "test_oracle_global.py", "test_oracle_penalties.py",
            "test_oracle_stopping.py"]
    files = [os.path.join(ROOT, "tests", f) for f in pins if os.path.exists(os.path.join(ROOT, "tests", f))]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                       env=_child_env([_runtime("gcc", "libasan.so"), _runtime("gcc", "libubsan.so")],
                                      {"HSADMM_ORACLE_LIB": so, "OMP_NUM_THREADS": "4"}), cwd=ROOT,
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_the_librarys_host_code_holds_under_the_undefined_behaviour_sanitizer(tmp_path):
    """The host half of libhsadmm.so (argument checks, plan tables, the host functions of Eq. (9) and of the penalty
    rule) with the sanitizer on the host pass only; the device code is compiled as always.  No kernel is launched:
    the checks are the ones of test_abi_cpu.py that need no device."""
    from paper_2512_14628_amd import binding
    so = str(tmp_path / "libhsadmm_san.so")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = "/opt/rocm/lib/llvm/bin/clang++"           # the compiler hipcc drives: its runtimes are the ones linked
    cmd = [hipcc, *binding.HIPCC_FLAGS, "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-shared-libsan",
           "-I", binding.INCLUDE_DIR, "-I", os.path.dirname(binding.SRC_PATH), "-o", so, binding.SRC_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    keep = "header_symbols or rejects or null_plan or node_coefficients or adapt_penalties or stopping"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", keep,
                        os.path.join(ROOT, "tests", "test_abi_cpu.py")],
                       env=_child_env([_runtime(clang, "libclang_rt.ubsan_standalone-x86_64.so")], {"HSADMM_LIB": so}),
                       cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
