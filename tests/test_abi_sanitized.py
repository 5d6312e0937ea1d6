"""The C-ABI layer's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU).

`csrc/api.hip` is compiled with the sanitizers on its host side only, linked with a driver that calls every entry
point with arguments its validation has to refuse (so nothing is ever enqueued) and with the library's ordinary
kernel objects, and run as an executable of its own.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2407_07304_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def test_abi_layer_is_clean_under_host_sanitizers(tmp_path):
    from paper_2407_07304_amd import build
    kernels = [os.path.join(CSRC, s.replace(".hip", ".o")) for s in build.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in kernels):
        build.build()
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("api_san.o", "driver_san.o", "abi_sanitize_driver"))
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all"]

    def run(cmd):
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-3000:]

    run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC"] + host_san +
        ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-c", os.path.join(CSRC, "api.hip"), "-o", api_o])
    run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
         os.path.join(HERE, "host_models", "abi_sanitize_driver.cpp"), "-o", drv_o])
    run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address,undefined", api_o, drv_o] + kernels + ["-o", exe])
    # (leak detection off: the HIP runtime keeps its own allocations until the process ends)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "clean" in r.stdout, r.stdout[-4000:]
