"""Builds and runs the gfx950 microbenchmarks behind the kernel design notes (needs a GPU).

    python -m paper_2209_13443_amd.microbench.run [name ...]      # default: all of lds_bw dma_bw mfma_rate clock launch_cost dispatch_floor

Each one is a self-contained HIP program; the binaries go to a temporary directory."""
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ALL = ["clock", "mfma_rate", "lds_bw", "dma_bw", "launch_cost", "dispatch_floor"]


def main(names):
    with tempfile.TemporaryDirectory() as tmp:
        for name in names or ALL:
            exe = os.path.join(tmp, name)
            subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                                   "-Wno-unused-result", "-Wno-unused-value", "-Wno-unused-command-line-argument", os.path.join(HERE, name + ".hip"), "-o", exe])
            print(f"== {name}", flush=True)
            subprocess.check_call([exe], timeout=120)


if __name__ == "__main__":
    main(sys.argv[1:])
