"""Host-side code under the sanitizers (CPU only, no GPU involved).

1. tests/san_driver.cpp + oracle/adam_oracle.c + the library's host-only source file, built
   with -fsanitize=address,undefined -fno-sanitize-recover=all, run as a program.
2. The existing oracle pins and host-logic tests once more against UndefinedBehaviorSanitizer
   builds of the same two source files (a shared library cannot carry AddressSanitizer into an
   uninstrumented Python, hence the split)."""
import ctypes
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "_build", "san")
ORACLE_C = os.path.join(ROOT, "oracle", "adam_oracle.c")
HOST_CPP = os.path.join(ROOT, "paper_2509_21271_amd", "csrc", "so_host.cpp")
INCLUDE = os.path.join(ROOT, "include")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout + r.stderr
    return r


def test_driver_under_address_and_undefined_behaviour_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    obj = os.path.join(OUT, "adam_oracle.o")
    _run(["gcc", *san, "-std=c99", "-ffp-contract=off", "-c", ORACLE_C, "-o", obj])
    exe = os.path.join(OUT, "san_driver")
    _run(["g++", *san, "-std=c++17", "-I", INCLUDE, os.path.join(ROOT, "tests", "san_driver.cpp"), HOST_CPP, obj,
          "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer driver OK" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_pins_pass_against_an_ubsan_build_of_the_oracle():
    os.makedirs(OUT, exist_ok=True)
    lib = os.path.join(OUT, "liboracle_ubsan.so")
    _run(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
          "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", lib, ORACLE_C, "-lm"])
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=lib, UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stdout + r.stderr


def test_host_logic_passes_against_an_ubsan_build_of_the_host_only_functions(monkeypatch):
    """The layout / validation / loss-scale / repartitioning tests, with the binding's library
    handle swapped for one whose host-only entry points come from a sanitizer build."""
    os.makedirs(OUT, exist_ok=True)
    lib = os.path.join(OUT, "libso_host_ubsan.so")
    _run(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=undefined", "-fno-sanitize-recover=all",
          "-I", INCLUDE, "-o", lib, HOST_CPP])
    import paper_2509_21271_amd as pkg
    if not os.path.exists(pkg.LIB):
        pkg.build_library()
    from paper_2509_21271_amd import binding as B
    san = ctypes.CDLL(lib)
    host_only = ("so_version", "so_layout_plan", "so_arena_plan", "so_arena_candidate", "so_validate",
                 "so_loss_scale_next", "so_plan_resident")

    class Proxy:
        def __getattr__(self, name):
            if name in host_only:
                f = getattr(san, name)
                f.restype, f.argtypes = B._sig[name]
                return f
            return getattr(B._lib_real, name)

    monkeypatch.setattr(B, "_lib_real", B._lib, raising=False)
    monkeypatch.setattr(B, "_lib", Proxy())
    import test_host_logic as T
    for numel, bucket in ([10, 5, 7], 8), ([1, 1, 1], 1), ([0, 9, 0, 3], 4), ([64], 8), ([3], 100), ([], 5), \
            ([17, 31, 2, 2, 40], 16):
        T.test_layout_plan_matches_definition(B, numel, bucket)
    T.test_layout_plan_of_the_benchmark_configs(B)
    T.test_layout_plan_rejects_bad_arguments(B)
    for n in (0, 1, 524_289, 8_030_261_248):
        T.test_arena_plan_orders_p_g_m_q_v_on_2_mib_boundaries(B, n)
    for n, spare, second in ((524_289, 1 << 30, False), (8_030_261_248, 80 << 30, True), (1, 0, True)):
        T.test_arena_candidates_never_overlap_or_leave_the_workspace(B, n, spare, second)
    for norm, max_norm, scale in ((0.5, 1.0, 1.0), (11.155, 1.0, 1.0), (3.0, 0.0, 65536.0), (7.0, 2.5, 1024.0)):
        T.test_validate_matches_oracle_clip(B, norm, max_norm, scale)
    T.test_validate_overflow_halves_the_scale(B)
    T.test_plan_resident_is_the_smallest_n_of_the_inequality(B)
    T.test_loss_scale_schedule_follows_the_hand_worked_walk(B)
    assert "gfx950" in B.so_version()
