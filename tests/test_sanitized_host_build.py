"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the oracle (the whole C file) and
the host side of the C ABI (argument checks, dispatch, the header check) are rebuilt with the sanitizers and the
oracle's pins and the ABI tests are run again on those builds, in a child process that preloads the sanitizer
runtime.  Any report (a read past a buffer, signed overflow, a misaligned access, ...) aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    import oracle
    from paper_2307_09782_amd import build
    d = str(tmp_path_factory.mktemp("san"))
    rt = build.sanitizer_runtime()
    if not os.path.exists(rt):
        pytest.skip("no AddressSanitizer runtime in this toolchain")
    env = dict(os.environ)
    env["ZQFP_ORACLE_LIB"] = oracle.build_oracle_sanitized(os.path.join(d, "libzqfp_oracle_san.so"))
    env["ZQFP_LIB_PATH"] = build.build_host_sanitized(os.path.join(d, "libzqfp_san.so"))
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")  # the runtime must come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    return env


def _run(env, code_or_args, timeout=600):
    return subprocess.run([sys.executable, *code_or_args], cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)


def test_the_sanitizer_is_live_in_the_child(sanitized):
    """A deliberate 50-byte header handed to the (88-byte) header check must be reported: shows that the runs
    below would see a real defect."""
    code = ("import ctypes, os\n"
            "L = ctypes.CDLL(os.environ['ZQFP_LIB_PATH'])\n"
            "libc = ctypes.CDLL(None)\n"
            "libc.malloc.restype = ctypes.c_void_p; libc.malloc.argtypes = [ctypes.c_size_t]\n"
            "L.zqfp_packed_weight_check.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]\n"
            "L.zqfp_packed_weight_check(libc.malloc(50), 512, 200, 64)\n")
    r = _run(sanitized, ["-c", code])
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stderr


def test_oracle_pins_and_abi_checks_pass_under_the_sanitizers(sanitized):
    files = ["tests/test_oracle_formats.py", "tests/test_oracle_quant.py", "tests/test_oracle_gemm.py",
             "tests/test_oracle_producers.py", "tests/test_oracle_rmsnorm.py", "tests/test_library_abi.py"]
    r = _run(sanitized, ["-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not bench_refuses and not spills",
                         *files], timeout=1500)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail
