"""The four host files of the library (recorder, barrier, lowering, stream schedule), built for the
CPU with AddressSanitizer and UndefinedBehaviorSanitizer and driven through the C ABI on the null
device by tests/host_sanitize/driver.cpp (kernel launchers are stubs: nothing here touches a GPU)."""
import os
import subprocess

from conftest import ROOT

CSRC = os.path.join(ROOT, "paper_2102_13267_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")


def test_host_files_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "lt_host_asan")
    srcs = [os.path.join(CSRC, f) for f in ("lt_api.cpp", "lt_barrier.cpp", "lt_lower.cpp", "lt_schedule.cpp")]
    srcs += [os.path.join(HERE, "stubs.cpp"), os.path.join(HERE, "driver.cpp")]
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", "-o", exe] + srcs + \
          [f"-L{rocm}/lib", "-lamdhip64", f"-Wl,-rpath,{rocm}/lib"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    out = run.stdout + run.stderr
    assert run.returncode == 0 and "host sanitizer driver: ok" in run.stdout, out[-6000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-6000:]
