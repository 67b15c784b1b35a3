"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the oracle's C file with every pin run
against the instrumented build, and the host-side Stage-2 search of the library built as plain C++."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


def _asan_env(extra):
    """An instrumented shared object inside an uninstrumented python needs the sanitizer runtime loaded first;
    whatever is preloaded already stays preloaded after it."""
    rt = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(rt):
        pytest.skip("gcc has no libasan.so")
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"   # python itself is not leak-clean
    env["OMP_NUM_THREADS"] = "2"
    env.update(extra)
    return env


def test_oracle_pins_pass_on_a_sanitized_build(tmp_path):
    lib = str(tmp_path / "liblexi_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
                           *SAN, "-o", lib, os.path.join(ROOT, "oracle", "lexi_oracle.c"), "-lm"])
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=_asan_env({"LEXI_ORACLE_LIB": lib}), cwd=ROOT,
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "failed" not in r.stdout


def test_stage2_search_is_clean_under_sanitizers(tmp_path):
    """The library's Algorithm 2 is host code: built here with g++ and the sanitizers, driven over the shapes of the
    workloads, a single layer, budgets at both ends of the feasible range and heavy mutation."""
    lib = str(tmp_path / "libstage2_san.so")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", *SAN, "-x", "c++",
                           os.path.join(ROOT, "paper_2509_02753_amd", "csrc", "stage2.hip"), "-o", lib])
    prog = textwrap.dedent(f"""
        import ctypes, random
        lib = ctypes.CDLL({lib!r})
        lib.lexi_allocate_topk.restype = ctypes.c_int32
        lib.lexi_allocate_topk.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_uint64,
                                           ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
        rnd = random.Random(3)
        cases = [(1, 1, 4, 1), (1, 1, 4, 4), (1, 2, 2, 2), (2, 1, 2, 3), (16, 2, 8, 96), (16, 2, 8, 32), (16, 2, 8, 128),
                 (24, 1, 4, 72), (32, 1, 2, 48), (26, 2, 6, 104), (40, 1, 2, 60), (5, 1, 64, 100)]
        for L, k_min, k_max, B in cases:
            for eta, n_pop, g_max in ((0.0, 2, 5), (0.1, 24, 200), (1.0, 7, 200)):
                D = (ctypes.c_double * (L * (k_max + 1)))(*[rnd.uniform(0, 3) for _ in range(L * (k_max + 1))])
                out = (ctypes.c_int32 * L)()
                phi = ctypes.c_double()
                st = lib.lexi_allocate_topk(D, L, B, k_min, k_max, n_pop, g_max, eta, 11, out, ctypes.byref(phi))
                k = list(out)
                assert st == 0 and sum(k) == B and min(k) >= k_min and max(k) <= k_max, (L, k_min, k_max, B, st, k)
        print("stage2 sanitized ok")
    """)
    r = subprocess.run([sys.executable, "-c", prog], env=_asan_env({}), capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "stage2 sanitized ok" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
