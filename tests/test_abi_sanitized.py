"""Host code of libef under AddressSanitizer and UndefinedBehaviorSanitizer
(device code is compiled as usual): tests/abi_sanitized_driver.cpp walks the
argument checks of every entry point and the creation and release of a plan.
No GPU is needed; with one present the driver also rebuilds the plan's lists."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def test_library_host_code_runs_clean_under_sanitizers(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_san")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
           "-fhip-fp32-correctly-rounded-divide-sqrt", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1905_10936_amd", "csrc"),
           "-x", "hip", os.path.join(HERE, "abi_sanitized_driver.cpp"),
           os.path.join(ROOT, "paper_1905_10936_amd", "csrc", "ef_api.hip"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr[-4000:]
    # what the GPU runtime's own libraries keep until the process ends is not this library's leak
    supp = tmp_path / "lsan.supp"
    supp.write_text("leak:libhsa-runtime64\nleak:libamdhip64\nleak:libhsakmt\nleak:libdrm\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1",
               LSAN_OPTIONS="suppressions=%s:print_suppressions=0" % supp)
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr[-4000:]
    assert "abi sanitized run ok" in run.stdout
