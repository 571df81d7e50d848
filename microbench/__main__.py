"""Build and run the micro-benchmarks (``python -m microbench [name ...]`` from the repository root) on the visible GPU.

They measure the machine limits that the GEMM design is judged against: the issue rate of the dequantize fold next
to INT8 MFMAs (``fold_issue_rate``, and with real data dependences ``fold_chain_rate``), what the LDS fragment
reads, the stage barrier and the direct-to-LDS loads of the real K loop add to it (``kloop_overheads``), a model of the
whole K loop per tile shape and block size (``kloop_model``), and the L2 /
last-level-cache bandwidth a compute unit sees (``l2_bandwidth``).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
FLAGS = ["--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def main(names):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for name in names or ["fold_issue_rate", "fold_chain_rate", "kloop_overheads", "kloop_model", "l2_bandwidth"]:
        src, exe = os.path.join(HERE, name + ".hip"), os.path.join(HERE, "_build_" + name)
        res = subprocess.run([hipcc, *FLAGS, src, "-o", exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            sys.exit("hipcc failed:\n" + res.stdout)
        print(f"== {name}", flush=True)
        subprocess.run([exe], check=True, timeout=120)


if __name__ == "__main__":
    main(sys.argv[1:])
