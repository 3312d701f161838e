"""Host sanitizer runs (CPU only, never the GPU): the C oracle and the C-ABI argument layer are rebuilt with
AddressSanitizer + UndefinedBehaviorSanitizer and the oracle pins / the host ABI tests run again under them in
child processes that preload the sanitizer run-time.  A report from either sanitizer fails the child."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(env_extra, args, timeout):
    env = dict(os.environ)
    env.update(env_extra)
    # the leak checker would report the interpreter's own allocations; the link order check does not apply
    # to a preloaded run-time
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=66"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=67"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=timeout)
    text = r.stdout + r.stderr
    assert "ERROR: AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert r.returncode == 0, text[-4000:]
    return text


def _preload(path):
    keep = os.environ.get("LD_PRELOAD", "")
    return path + (":" + keep if keep else "")


def test_oracle_pins_under_address_and_ub_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    ubsan = subprocess.run(["gcc", "-print-file-name=libubsan.so"], capture_output=True, text=True).stdout.strip()
    if not (os.path.isabs(asan) and os.path.exists(asan)):
        pytest.skip("gcc has no AddressSanitizer run-time here")
    pre = asan + (":" + ubsan if os.path.isabs(ubsan) and os.path.exists(ubsan) else "")
    text = _run({"EBS_ORACLE_SANITIZE": "1", "LD_PRELOAD": _preload(pre), "OMP_NUM_THREADS": "2"},
                ["tests/test_oracle_pins.py"], timeout=900)
    assert " passed" in text


def test_abi_argument_layer_under_address_and_ub_sanitizers():
    rt = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not rt:
        pytest.skip("the HIP compiler has no shared AddressSanitizer run-time here")
    import torch
    if torch.cuda.is_available():
        pytest.skip("host-only sanitizer run: not on a machine with a GPU")
    from paper_2003_07577_amd.build import build_host_sanitized
    lib = build_host_sanitized()
    text = _run({"EBS_LIBRARY_PATH": lib, "LD_PRELOAD": _preload(rt[-1])},
                ["tests/test_abi_host.py", "--deselect", "tests/test_abi_host.py::test_bench_refuses_more_than_one_gpu"],
                timeout=900)
    assert " passed" in text
