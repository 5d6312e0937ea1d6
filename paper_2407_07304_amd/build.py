"""Builds ``libslimattn.so`` (the C-ABI library) and ``libslimprobe.so`` (the measurement kernels of
``include/slimprobe.h``) from ``csrc/`` with hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libslimattn.so")
SOURCES = ["api.hip", "kv_quant.hip", "decode.hip", "decode_gqa.hip", "prefill.hip", "prefill_strip.hip"]
PROBE_LIB = os.path.join(HERE, "libslimprobe.so")
PROBE_SOURCES = ["probes.hip", "decode_gqa.hip"]   # (the grouped-query decode kernel has a traffic-only form)
# prefill.hip: MFMA results stay in arch VGPRs (no AGPR copies around the softmax), and fmaxf needs no
# NaN quieting (NaN inputs are documented as undefined).  The quantiser keeps the IEEE defaults.
# -Wno-inline-asm: its buffer loads with an LDS destination set M0 themselves and say so in the clobber list.
EXTRA = {"prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans", "-mno-amdgpu-ieee", "-Wno-inline-asm"],
         "prefill_strip.hip": ["-fno-honor-nans"],
         "decode_gqa.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-fno-honor-nans"]}
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-fp32 instructions are switched off for every kernel of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _build_lib(lib, sources, verbose):
    objs = []
    for src in sources:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC] + FLAGS + EXTRA.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(ln for ln in r.stdout.splitlines() if "packed-fp32-ops" not in ln)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    tmp = lib + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stdout)
    os.replace(tmp, lib)
    return lib


def build(verbose: bool = False) -> str:
    """Compiles every source every time it is called; returns the path of the attention library."""
    _build_lib(PROBE_LIB, PROBE_SOURCES, verbose)
    return _build_lib(LIB, SOURCES, verbose)


if __name__ == "__main__":
    print(build(verbose=True))
