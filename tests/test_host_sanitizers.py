"""Host-side sanitizer leg (CPU only, nothing here touches a GPU).

1. The C oracle and a driver that walks ragged batches through every one of its entry points are compiled with
   AddressSanitizer and UndefinedBehaviorSanitizer and run; any report, leak, mismatch against the scalar
   definition in the driver, or nonzero exit fails.
2. The C-ABI library is built once more with its HOST code under the same two sanitizers (the device code is
   compiled as always and never runs here), and a C driver calls every entry point with arguments that the
   validation has to reject before the first launch."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_c_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "sanitize_check"
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-Wall", "-Wextra",
           os.path.join(ROOT, "oracle", "hydra_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c"), "-o", str(exe), "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr and "LeakSanitizer" not in res.stderr, res.stderr
    assert res.stdout.count(": ok") == 8 and "MISMATCH" not in res.stdout


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="no ROCm compiler")
def test_boundary_host_code_under_sanitizers(tmp_path):
    lib = tmp_path / "libhydra_attn_san.so"
    # (each -fsanitize goes to the host pass only; the device pass of this pool's compiler must not see one)
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-shared", "-fPIC",
                           os.path.join(ROOT, "paper_2505_12658_amd", "csrc", "hydra_api.hip"), "-o", str(lib)],
                          stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    exe = tmp_path / "boundary_sanitize_check"
    subprocess.check_call([CLANG, "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", os.path.join(ROOT, "tests", "boundary_sanitize_check.c"),
                           "-o", str(exe), f"-L{tmp_path}", "-lhydra_attn_san", f"-Wl,-rpath,{tmp_path}"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")  # (the HIP runtime keeps its own allocations)
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
    assert "all statuses as expected" in res.stdout
