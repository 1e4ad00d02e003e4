"""The host-only code of the library under sanitizers, on the CPU (no GPU is touched).

* AddressSanitizer + UndefinedBehaviorSanitizer: the argument validation and launch planning
  (mts_api.hip), the cache manager (mts_cache_manager.hip) and the transfer pipeline's host code
  (mts_xfer.hip) are rebuilt with host-side instrumentation (device code is left alone) and linked
  with the kernels' ordinary objects into a second shared library; tests/test_abi.py (error codes
  before launch, random descriptors and metadata) and tests/test_cache_manager.py (random traces
  against the model) then run against THAT library in a child interpreter.
* ThreadSanitizer, and once more ASan/UBSan: the copy-thread pool (mts_copy_pool.hpp), which
  signals through atomics and polls, built on its own with tests/native/copy_pool_check.cpp.

Any sanitizer report fails the test.  If the toolchain cannot produce or start an instrumented
binary here, the case is skipped with the reason."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_22881_amd")
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "_build", "san")
HIPCC = "/opt/rocm/bin/hipcc"
REPORT_MARKS = ("ERROR: AddressSanitizer", "runtime error:", "WARNING: ThreadSanitizer", "ERROR: LeakSanitizer",
                "SUMMARY: UndefinedBehaviorSanitizer", "SUMMARY: AddressSanitizer", "SUMMARY: ThreadSanitizer")
HOST_SOURCES = ("mts_api", "mts_cache_manager", "mts_xfer")


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def _no_reports(text):
    hits = [m for m in REPORT_MARKS if m in text]
    assert not hits, f"sanitizer report ({hits}):\n{text[-4000:]}"


def test_validation_cache_manager_and_pipeline_host_code_under_asan_ubsan():
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc here")
    kernel_objs = [o for o in glob.glob(os.path.join(PKG, "_build", "*.o"))
                   if os.path.basename(o)[:-2] not in HOST_SOURCES]
    if not kernel_objs:
        pytest.skip("the library's objects are not built (python -m paper_2604_22881_amd.build)")
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        pytest.skip("the compiler ships no shared AddressSanitizer runtime")
    os.makedirs(OUT, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer",
             "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    objs = []
    for name in HOST_SOURCES:
        obj = os.path.join(OUT, name + ".o")
        r = _run([HIPCC, *flags, "-c", os.path.join(CSRC, name + ".hip"), "-o", obj])
        assert r.returncode == 0, r.stderr[-3000:]
        objs.append(obj)
    lib = os.path.join(OUT, "libmtserve_hip_asan.so")
    r = _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-fsanitize=address,undefined",
              "-fno-gpu-sanitize", "-shared-libsan", "-o", lib, *objs, *kernel_objs])
    assert r.returncode == 0, r.stderr[-3000:]
    runner = os.path.join(OUT, "run_under_asan.py")
    with open(runner, "w") as f:
        f.write(f"""import sys
sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})
import paper_2604_22881_amd.binding as B
B.LIB_PATH = {lib!r}
import pytest
rc = pytest.main(["-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                  {os.path.join(ROOT, 'tests', 'test_abi.py')!r}, {os.path.join(ROOT, 'tests', 'test_cache_manager.py')!r}])
assert B.lib()._name == {lib!r}
maps = open("/proc/self/maps").read()
assert "libmtserve_hip_asan.so" in maps and "libclang_rt.asan" in maps, "the instrumented library was not the one loaded"
print("INSTRUMENTED LIBRARY LOADED")
sys.exit(rc)
""")
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt[0] + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = _run([sys.executable, runner], env=env, timeout=600)
    text = r.stdout + r.stderr
    _no_reports(text)
    assert r.returncode == 0, text[-4000:]
    assert "INSTRUMENTED LIBRARY LOADED" in text and " passed" in text
    print(text.strip().splitlines()[-2])


@pytest.mark.parametrize("sanitizer,rounds", [("thread", 10), ("address,undefined", 40)])
def test_copy_thread_pool_under_sanitizers(sanitizer, rounds):
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "copy_pool_check_" + sanitizer.replace(",", "_"))
    r = _run(["g++", "-O1", "-g", "-std=c++17", "-pthread", "-fsanitize=" + sanitizer,
              os.path.join(ROOT, "tests", "native", "copy_pool_check.cpp"), "-o", exe])
    if r.returncode != 0:
        pytest.skip(f"g++ cannot build with -fsanitize={sanitizer} here: {r.stderr[-300:]}")
    r = _run([exe, str(rounds)], timeout=600)
    text = r.stdout + r.stderr
    if "FATAL: ThreadSanitizer: unexpected memory mapping" in text or "FATAL: ThreadSanitizer: unsupported" in text:
        pytest.skip("ThreadSanitizer cannot map its shadow memory in this container")
    _no_reports(text)
    assert r.returncode == 0 and "0 mismatching copies" in text, text[-2000:]
