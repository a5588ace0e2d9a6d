"""The CPU-side code under AddressSanitizer + UndefinedBehaviorSanitizer: the oracle (all its pins) and
the host side of the library (argument validation, workspace carving, the sizing call; the ABI tests).
Each is rebuilt with the sanitizers into a temporary directory and the corresponding tests are rerun in a
child process with the sanitizer runtime preloaded; any report aborts the child and fails the test.
No GPU is involved: kernels are never launched by these tests."""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_under(preload, env_extra, test_files):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = preload + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]
                       + test_files, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail


def test_oracle_pins_under_asan_ubsan(tmp_path):
    import oracle
    lib = oracle.build_sanitized(str(tmp_path / "libkvm_oracle_san.so"))
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert len(files) >= 10
    _run_under(oracle.asan_runtime(), {"KVM_ORACLE_LIB": lib}, files)


def test_library_host_side_under_asan_ubsan(tmp_path):
    from paper_2604_26968_amd import _build
    rt = _build.asan_runtime()
    assert rt, "the compiler's shared AddressSanitizer runtime was not found"
    lib = _build.build(sanitize=True, out=str(tmp_path / "libkvm_san.so"))
    _run_under(rt, {"KVM_LIB": lib}, [os.path.join(ROOT, "tests", "test_abi.py")])
