"""Host code under sanitizers (the GPU has none): the CPU oracle and the test-only host build of the kernels'
per-environment code run rollouts of every mode and rule flag, both observations, export and import under
AddressSanitizer + UndefinedBehaviorSanitizer, and the host build also under clang's MemorySanitizer (reads of
uninitialised memory), with its functions inlined as in the kernels and again with every function out of line."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SAN = os.path.join(HERE, "sanitize")
CLANG = next((c for c in ("/opt/rocm/llvm/bin/clang++", shutil.which("clang++")) if c and os.path.exists(c)), None)


def _variants():
    cxx = CLANG or "g++"
    v = {
        "oracle_asan": ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        os.path.join(SAN, "san_oracle.c")],
        "host_asan": [cxx, "-O1", "-g", "-std=c++17", "-Wno-unknown-pragmas", "-fsanitize=address,undefined",
                      "-fno-sanitize-recover=undefined", os.path.join(SAN, "san_hostbuild.cpp")],
    }
    if CLANG:
        msan = [CLANG, "-g", "-std=c++17", "-Wno-unknown-pragmas", "-fsanitize=memory", "-fsanitize-memory-track-origins=2",
                "-fno-omit-frame-pointer", "-fsanitize-ignorelist=" + os.path.join(SAN, "msan_ignore.txt"),
                os.path.join(SAN, "san_hostbuild.cpp")]
        v["host_msan_inline"] = msan + ["-O1"]
        v["host_msan_out_of_line"] = msan + ["-O0", "-DSAN_OUT_OF_LINE"]
    return v


@pytest.fixture(scope="module")
def built(tmp_path_factory):
    """the four instrumented programs, compiled side by side (each compile takes about half a minute)"""
    from concurrent.futures import ThreadPoolExecutor
    d = str(tmp_path_factory.mktemp("san"))
    v = _variants()

    def build(name):
        out = os.path.join(d, name)
        p = subprocess.run(v[name] + ["-o", out], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return name, (out if p.returncode == 0 else None), p.stdout
    with ThreadPoolExecutor(len(v)) as ex:
        res = {n: (o, log) for n, o, log in ex.map(build, list(v))}
    return res


def _run(built, name, expect=9):
    if name not in built:
        pytest.skip("MemorySanitizer needs clang")
    exe, log = built[name]
    assert exe, log[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env.pop("LD_PRELOAD", None)                 # a sanitizer runtime has to come first in the library list
    # the slow ones (the recursive oracle, the unoptimised out-of-line build) get a smaller batch
    size = ["16", "900"] if name in ("oracle_asan", "host_msan_out_of_line") else ["64", "1200"]
    p = subprocess.run([exe] + size, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert p.returncode == 0, p.stdout[-3000:]
    assert p.stdout.count(" ok, ") == expect and "runtime error" not in p.stdout, p.stdout[-3000:]


@pytest.mark.parametrize("name", ["oracle_asan", "host_asan", "host_msan_inline", "host_msan_out_of_line"])
def test_clean_under_sanitizer(built, name):
    _run(built, name)
