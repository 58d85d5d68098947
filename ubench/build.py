"""Compile the hardware microbenchmarks in this folder (one executable per .hip file) into
_build/ at the repository root.  They are not part of the library: they measure what the
chip sustains (matrix-core stream with a kernel's instruction mix, fp32 atomic adds) and back
the figures quoted in profiles/.  Run the executables on the GPU by hand.

    python ubench/build.py
"""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(os.path.dirname(HERE), "_build")


def main():
    os.makedirs(OUT, exist_ok=True)
    hipcc = os.environ.get("HIPCC") or "/opt/rocm/bin/hipcc"
    for src in sorted(glob.glob(os.path.join(HERE, "*.hip"))):
        exe = os.path.join(OUT, os.path.splitext(os.path.basename(src))[0])
        cmd = [hipcc, "-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-Wno-unused-command-line-argument", src, "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode:
            raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        print(exe)


if __name__ == "__main__":
    main()
