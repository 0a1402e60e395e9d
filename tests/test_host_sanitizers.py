"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

The argument checks, the launch planning (work-item lists, key ranges, tile order, the memo of
the last plans) and the page map are host code in two files without any device code
(csrc/cs_api.hip, csrc/cs_page_map.hip).  They are compiled here for the host only with both
sanitizers, linked with stand-ins for the kernel launchers, and driven through the C ABI by
tests/host_sanitize/driver.cpp: random batches of every shape planned for three chip sizes, the
largest sequence count, and a few thousand random page-map operations checked against a plain
model.  Any sanitizer report fails the test.  No GPU is needed (GPU sanitizers are not used)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_01228_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")
CLANG = "/opt/rocm/lib/llvm/bin/clang++"


@pytest.mark.skipif(shutil.which("hipcc") is None or not os.path.exists(CLANG), reason="no ROCm toolchain")
def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-O1", "-g", "-std=c++17"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    for src in (os.path.join(CSRC, "cs_api.hip"), os.path.join(CSRC, "cs_page_map.hip"), os.path.join(HERE, "stubs.hip")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run(["hipcc", "--offload-arch=gfx950", "--cuda-host-only", "-fPIC", *san, *inc, "-c", src, "-o", obj],
                       check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        # these files must stay free of device code, or they cannot be linked on their own
        undefined = subprocess.run(["nm", "-u", obj], check=True, capture_output=True, text=True).stdout
        assert "__hip_fatbin" not in undefined, os.path.basename(src) + " now holds device code"
        objs.append(obj)
    drv = str(tmp_path / "driver.o")
    subprocess.run([CLANG, *san, *inc, "-c", os.path.join(HERE, "driver.cpp"), "-o", drv], check=True)
    exe = str(tmp_path / "driver")
    subprocess.run([CLANG, "-fsanitize=address,undefined", drv, *objs, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib",
                    "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, "sanitizer driver failed:\n" + run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.strip().startswith("ok "), run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
