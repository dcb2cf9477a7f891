"""The library's HOST code (argument validation, launch plans, workspace arithmetic) under AddressSanitizer and
UndefinedBehaviorSanitizer, on a machine without a GPU: tests/abi_sanitize_main.cpp calls every entry point with
arguments that must be rejected before any HIP call.  Only the host pass of aasd.hip is compiled (seconds); the
symbol that would hold the device code object is satisfied by a zero-filled stand-in, which is never looked at
because nothing is launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) or shutil.which("nm") is None, reason="needs hipcc and nm")
def test_host_code_runs_clean_under_sanitizers(tmp_path):
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    common = [HIPCC, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "--offload-host-only", *san,
              "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2505_13204_amd", "csrc"), "-c"]
    lib_o, main_o, stub_c, stub_o, exe = (str(tmp_path / n) for n in ("aasd_host.o", "main_host.o", "stub.c", "stub.o", "abi_san"))
    subprocess.check_call([*common, "-o", lib_o, os.path.join(ROOT, "paper_2505_13204_amd", "csrc", "aasd.hip")], stderr=subprocess.DEVNULL)
    subprocess.check_call([*common, "-x", "hip", "-o", main_o, os.path.join(ROOT, "tests", "abi_sanitize_main.cpp")], stderr=subprocess.DEVNULL)
    syms = [ln.split()[-1] for ln in subprocess.check_output(["nm", lib_o], text=True).splitlines() if " U __hip_fatbin_" in ln]
    assert len(syms) == 1, syms
    with open(stub_c, "w") as f:
        f.write(f"const char {syms[0]}[4096] __attribute__((aligned(4096))) = {{0}};\n")
    subprocess.check_call(["gcc", "-c", stub_c, "-o", stub_o])
    subprocess.check_call([HIPCC, "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe, lib_o, main_o, stub_o],
                          stderr=subprocess.DEVNULL)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"     # (the HIP runtime keeps its own allocations until exit)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    run = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "0 mismatches" in run.stdout and "gfx950" in run.stdout
