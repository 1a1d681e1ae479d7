"""The C oracle and the host side of libdmt under AddressSanitizer and
UndefinedBehaviorSanitizer (CPU only; device code is compiled as always and never runs here).

Each is built into a scratch directory with -fsanitize=address,undefined and a child python
runs the pins / the host-validation tests on it with the sanitizer runtime preloaded: a heap
overflow, a use after free or undefined arithmetic in the checker or in the plan / layout /
Tower-Partitioner host code fails the child."""
import glob
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ASAN_OPTIONS = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
UBSAN_OPTIONS = "halt_on_error=1:print_stacktrace=1"


def _first(patterns):
    for p in patterns:
        hits = sorted(glob.glob(p))
        if hits:
            return hits[0]
    return None


def _run_child(code, preload, extra_env):
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS=ASAN_OPTIONS, UBSAN_OPTIONS=UBSAN_OPTIONS,
               PYTHONPATH=ROOT + os.pathsep + os.path.join(ROOT, "tests"), **extra_env)
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "passed" in r.stdout, r.stdout[-2000:]
    return r.stdout


def test_oracle_under_asan_and_ubsan():
    runtime = _first(["/usr/lib/x86_64-linux-gnu/libasan.so.*", "/usr/lib/gcc/x86_64-linux-gnu/*/libasan.so"])
    if runtime is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "libdmt_oracle_san.so")
        subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined",
                               "-fno-sanitize-recover=undefined", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", lib, os.path.join(ROOT, "oracle", "dmt_oracle.c"),
                               "-lm"])
        code = ("import sys, pytest; sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', "
                "'tests/test_oracle_lookup.py', 'tests/test_oracle_bwd.py', 'tests/test_oracle_tm.py']))")
        _run_child(code, runtime, {"DMT_ORACLE_LIB": lib})


def test_libdmt_host_code_under_asan_and_ubsan():
    runtime = _first(["/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"])
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if runtime is None or not os.path.exists(hipcc):
        pytest.skip("hipcc or its AddressSanitizer runtime is not installed")
    from concurrent.futures import ThreadPoolExecutor
    from paper_2403_00877_amd import build as hip_build
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-g", "-shared-libsan"]
    with tempfile.TemporaryDirectory() as tmp:
        srcs = hip_build.sources()
        objs = [os.path.join(tmp, os.path.basename(s)[:-4] + ".o") for s in srcs]

        def compile_one(pair):
            subprocess.run([hipcc] + hip_build.FLAGS + san + ["-c", "-o", pair[1], pair[0]], check=True,
                           stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)

        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
            list(pool.map(compile_one, zip(srcs, objs)))
        lib = os.path.join(tmp, "libdmt_san.so")
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                        "-fsanitize=undefined", "-shared-libsan", "-o", lib] + objs, check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        # the child loads the sanitized library in place of the in-tree one, then runs the tests
        # that need no GPU: argument validation, layout arithmetic, the partitioner's host stages
        code = (
            "import importlib.util, os, sys\n"
            "spec = importlib.util.spec_from_file_location('paper_2403_00877_amd.build', "
            "os.path.join(%r, 'paper_2403_00877_amd', 'build.py'))\n"
            "b = importlib.util.module_from_spec(spec); spec.loader.exec_module(b)\n"
            "b.LIB = %r; b.is_stale = lambda: False\n"
            "sys.modules['paper_2403_00877_amd.build'] = b\n"
            "import pytest\n"
            "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', 'tests/test_abi.py', "
            "'tests/test_tp_host.py']))\n" % (ROOT, lib))
        out = _run_child(code, runtime, {})
        assert "libdmt_san.so" not in out or "passed" in out
