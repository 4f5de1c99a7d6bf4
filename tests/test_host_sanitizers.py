"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

The whole library is built once more with the sanitizers switched on for the HOST side only (the
device code is compiled as usual and never runs here), and the tests that exercise host logic
without a GPU -- the head-node run bookkeeping against its oracle, and the argument paths of every
entry point -- run against that build in a child process that preloads the sanitizer runtime.  A
planted heap overflow in a scrap library, loaded the same way, shows that the set-up does report."""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_11798_amd", "csrc")
OUT = os.path.join(ROOT, "_build")
SOURCES = ["api.hip", "stage.hip", "misc.hip", "pack.hip", "kvmeta.hip", "sched.hip", "spec.hip"]
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
       "-fno-sanitize-recover=undefined"]


def _runtime():
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return hits[-1] if hits else None


def _env(lib=None):
    env = dict(os.environ)
    rt = _runtime()
    env["LD_PRELOAD"] = rt + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    if lib:
        env["PIPEINFER_LIB"] = lib
    return env


@pytest.fixture(scope="module")
def sanitized_library():
    if shutil.which("hipcc") is None or _runtime() is None:
        pytest.skip("hipcc or the sanitizer runtime is not in this image")
    os.makedirs(OUT, exist_ok=True)
    lib = os.path.join(OUT, "libpipeinfer_hostsan.so")
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, "pi_internal.h"), os.path.join(ROOT, "include", "pipeinfer.h")]
    if not os.path.exists(lib) or os.path.getmtime(lib) < max(os.path.getmtime(d) for d in deps):
        cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-g1", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + SAN + ["-o", lib] + srcs
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
    return lib


def test_a_planted_heap_overflow_is_reported(tmp_path, sanitized_library):
    src = tmp_path / "scrap.cpp"
    src.write_text('#include <cstdlib>\nextern "C" int scrap(int i) { int* p = (int*)malloc(16); p[i] = 1; int v = p[0]; free(p); return v; }\n')
    lib = tmp_path / "libscrap.so"
    r = subprocess.run(["hipcc", "-x", "c++", "-O0", "-g", "-fPIC", "-shared", "-fsanitize=address", "-o", str(lib), str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([sys.executable, "-c", "import ctypes; ctypes.CDLL(%r).scrap(4)" % str(lib)],
                       env=_env(), capture_output=True, text=True)
    assert r.returncode != 0 and "AddressSanitizer: heap-buffer-overflow" in r.stderr


def test_host_logic_is_clean_under_the_sanitizers(sanitized_library):
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_sched_parity.py"), os.path.join(ROOT, "tests", "test_abi.py")],
                       env=_env(sanitized_library), capture_output=True, text=True, cwd=ROOT)
    text = r.stdout + r.stderr
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert r.returncode == 0, text[-4000:]
    assert " passed" in r.stdout
