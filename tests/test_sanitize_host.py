"""AddressSanitizer + UBSan build of the host side of the library (C ABI validation, device and
scratch registry, cost model, selector) and of the C oracle, driven by tests/host_sanitize/driver.cpp.
Host only: kernels are not part of this build (their launchers are link-time stand-ins that abort if
ever reached; without a GPU every call must return MTNN_ERR_NO_DEVICE first)."""
import os
import subprocess

from paper_1702_03192_amd import build


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = build.build_host_sanitized(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
               HIP_VISIBLE_DEVICES="-1", MTNN_MODEL="")
    res = subprocess.run([exe, str(tmp_path)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "ALL OK" in res.stdout
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]


def test_host_state_is_race_free_under_tsan(tmp_path):
    """ThreadSanitizer build with tests/host_sanitize/driver_threads.cpp: readers query the selector (single,
    batched, three-way) and the cost model while other threads retrain, load, unload and save the model and
    register / withdraw scratch."""
    exe = build.build_host_sanitized(str(tmp_path), kind="thread")
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0:report_signal_unsafe=0", HIP_VISIBLE_DEVICES="-1", MTNN_MODEL="")
    res = subprocess.run([exe, str(tmp_path)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-6000:]
    assert "ALL OK" in res.stdout
    assert "ThreadSanitizer" not in res.stdout, res.stdout[-6000:]
