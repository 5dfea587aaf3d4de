"""The oracle and the host side of the C-ABI boundary under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only, no GPU).

The oracle is the yardstick of every parity claim, so its own memory accesses and integer arithmetic
are checked: the source is built with -fsanitize=address,undefined and the whole pin suite, plus a
few larger shapes, runs against that build in a child process with the sanitizer runtime preloaded.
A second child plants an out-of-range row to show that the sanitizer really is watching.
The HIP library is built once more with the sanitizers on its host code only (device code unchanged) and
the argument-validation tests, which reach every error return without a launch, run against that build.
"""
import os
import subprocess
import sys

import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def gcc_file(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    asan = gcc_file("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    so = tmp_path_factory.mktemp("san") / "libmoe_oracle_san.so"
    src = os.path.join(os.path.dirname(oracle.__file__), "moe_oracle.c")
    subprocess.check_call(["gcc", "-O1", "-g", "-mfma", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-shared", "-fPIC",
                           "-o", str(so), src, "-lm"])
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=86"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return str(so), env


PRELUDE = (
    "import sys\n"
    f"sys.path.insert(0, {ROOT!r})\n"
    f"sys.path.insert(0, {HERE!r})\n"
    "import numpy as np\n"
    "import oracle, workloads as wl\n"
    "oracle._load()\n"
    "oracle._lib = oracle._serial = oracle._open({so!r})\n"
)


def test_pins_and_larger_shapes_are_clean(sanitized):
    so, env = sanitized
    child = PRELUDE.format(so=so) + (
        "import test_oracle_pins as pins\n"
        "for check in pins.PINS:\n"
        "    check()\n"
        # ragged shapes, masked / invalid ids, fixed stride, several sources, both storage types, quantised rows
        "rng = np.random.default_rng(3)\n"
        "for (T, H, k, E, R, dt) in ((257, 72, 8, 64, 8, wl.DTYPE_BF16), (31, 20, 3, 12, 4, wl.DTYPE_F32),\n"
        "                            (1, 8, 1, 1, 1, wl.DTYPE_BF16), (0, 8, 2, 4, 2, wl.DTYPE_BF16)):\n"
        "    w = wl.make(wl.Config('san', T=T, H=H, k=k, E=E, R=R, dtype=dt, seed=T))\n"
        "    K = wl.random_routing(rng, T, k, E, p_masked=0.1, p_invalid=0.1)\n"
        "    for stride in (0, max(1, T * k // R)):\n"
        "        pl = oracle.plan(K, E, R, stride)\n"
        "        rows = max(pl.window_rows, R * stride)\n"
        "        win = oracle.dispatch(w.X, pl.row_map, rows)\n"
        "        oracle.combine(oracle.expert_standin(win, K, pl.row_map, w.scale), w.W, pl.row_map)\n"
        "        oracle.combine_f64(win, w.W, pl.row_map)\n"
        "        if dt == wl.DTYPE_BF16:\n"
        "            oracle.dispatch_quant(w.X, pl.row_map, max(rows, 1))\n"
        "        M = rng.integers(0, 30, size=(R, E)).astype(np.int32)\n"
        "        pm = oracle.plan_multi(K, M, R // 2, E, R, stride)\n"
        "        oracle.dispatch(w.X, pm.row_map, max(pm.window_rows, R * stride))\n"
        "print('clean')\n"
    )
    res = subprocess.run([sys.executable, "-c", child], capture_output=True, text=True, timeout=600, env=env)
    assert res.returncode == 0 and "clean" in res.stdout, res.stderr[-3000:]


def test_the_sanitizer_is_watching(sanitized):
    """A row map that points one row past the window must stop the sanitized build (and only that build:
    the planted mistake lives in this test's input, on the CPU)."""
    so, env = sanitized
    child = PRELUDE.format(so=so) + (
        "X = np.zeros((2, 64), np.uint16)\n"
        "row_map = np.array([[0], [3]], np.int32)\n"          # the window below has 3 rows
        "oracle.dispatch(X, row_map, 3)\n"
        "print('not noticed')\n"
    )
    res = subprocess.run([sys.executable, "-c", child], capture_output=True, text=True, timeout=120, env=env)
    assert res.returncode != 0 and "AddressSanitizer" in res.stderr and "not noticed" not in res.stdout


def test_boundary_validation_is_clean(tmp_path):
    """Host code of the library (argument checks, size arithmetic, error strings) under ASan + UBSan."""
    import glob
    rt = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not rt:
        pytest.skip("the HIP compiler ships no shared AddressSanitizer runtime here")
    from paper_2605_06055_amd.build import build_library
    so = str(tmp_path / "libmoe_rbf_san.so")
    build_library(so, extra_flags=["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                   "-Xarch_host", "-fno-sanitize-recover=all", "-shared-libsan"])
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(x for x in (rt[-1], env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:exitcode=86"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["MOE_RBF_LIB"] = so
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_boundary_host.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], capture_output=True, text=True, timeout=600, env=env, cwd=ROOT)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
