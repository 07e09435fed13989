"""Build the native test harnesses under tests/native (hipcc, gfx950, no GPU needed) into
paper_1703_06503_amd/lib/, beside the library they link against."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
LIBDIR = os.path.join(ROOT, "paper_1703_06503_amd", "lib")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
DISPATCH_OVERHEAD = os.path.join(LIBDIR, "dispatch_overhead")


def build():
    cmd = [os.path.join(ROCM, "bin", "hipcc"), "-O2", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(HERE, "dispatch_overhead.hip"), "-o", DISPATCH_OVERHEAD,
           f"-L{LIBDIR}", "-lsgemm_tuned", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{ROCM}/lib"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"command failed: {' '.join(cmd)}\n{out}")
    return DISPATCH_OVERHEAD


if __name__ == "__main__":
    print(build())
