"""Builds libdpstep.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "dp_step.hip")
LIB = os.path.join(HERE, "libdpstep.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept off for every device function of the library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # (= PACKED_OFF below)
    # fp32 atomic add as one hardware instruction (embedding scatter)
    "-munsafe-fp-atomics",
]


PACKED_OFF = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def check_packed_fp32_flag(hipcc):
    """The flag that keeps packed fp32 VALU forms off must be understood by the DEVICE pass.  hipcc's host pass
    always reports the feature as unknown (x86 has none of that name), which is harmless and is why that line is
    dropped from the build output below; a device-only compile of an empty kernel must not print it."""
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "probe.hip")
        with open(src, "w") as f:
            f.write("#include <hip/hip_runtime.h>\n__global__ void probe(float2 *p) { p[0].x = p[0].x * p[0].y + p[0].x; }\n")
        r = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "--cuda-device-only", "-c"] + PACKED_OFF +
                           ["-o", os.path.join(d, "probe.o"), src], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0 or "packed-fp32-ops" in r.stdout:
            raise RuntimeError("hipcc's gfx950 pass does not accept -target-feature -packed-fp32-ops:\n" + r.stdout)


def build_library(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    check_packed_fp32_flag(hipcc)
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = r.stdout.splitlines()
    # the host pass's "unknown feature" lines are dropped; the device pass was checked above
    out = "\n".join(l for l in lines if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
