"""The library's host code (argument validation, launch plans, error text) built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by tests/abi_validation_driver.cpp.  No GPU: every call of the driver is settled on
the host.  The device side of each translation unit is compiled without optimisation only so that the objects link; it
never runs."""

import os
import subprocess
import sys

from paper_2502_11101_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def test_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2502_11101_amd", "csrc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", csrc]
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]
    procs, objs = [], []
    for src in B.SOURCES:
        obj = str(tmp_path / (src[:-4] + ".o"))
        objs.append(obj)
        cmd = [HIPCC, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "--offload-arch=gfx950", "-Xarch_device", "-O0",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, *inc, "-c", os.path.join(csrc, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate(timeout=600)
        assert p.returncode == 0, f"{src}:\n{out[-3000:]}"
    drv_obj = str(tmp_path / "driver.o")
    subprocess.run([CLANGXX, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
                    os.path.join(ROOT, "tests", "abi_validation_driver.cpp"), "-o", drv_obj], check=True, timeout=300)
    exe = str(tmp_path / "abi_validation")
    subprocess.run([CLANGXX, *SAN, drv_obj, *objs, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
                   check=True, timeout=300)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    print(r.stdout[-2000:], file=sys.stderr)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "0 failed" in r.stdout and "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout
