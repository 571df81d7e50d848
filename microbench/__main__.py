"""Build and run the micro-benchmarks: ``python -m microbench [--build-only] [name ...]`` from the repository root.

They measure the machine limits that the kernels are judged against:
  fold_issue_rate        issue rate of the dequantize fold (Sec. 5.3) next to INT8 MFMAs;
  fold_chain_rate        the same with the real data dependences (the fold reads the tile the previous MFMA chain wrote);
  kloop_overheads        what LDS fragment reads, the stage barrier and direct-to-LDS loads of the real K loop add to it;
  kloop_model            the whole K loop per tile shape and block size;
  l2_bandwidth           L2 / last-level-cache bandwidth into a compute unit;
  quantizer_issue_rate   issue cost of the Eq. 1 rounding variants and of the other instructions of the memory-bound kernels;
  transposed_operands    weight gradient with bytes transposed inside the kernel against pre-transposed copies (needs the
                         built library).
The HIP probes are compiled with hipcc (``--build-only`` compiles them without running, e.g. on a box without a GPU; an
executable that is already there is reused).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
FLAGS = ["--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HIP_PROBES = ["fold_issue_rate", "fold_chain_rate", "kloop_overheads", "kloop_model", "l2_bandwidth", "quantizer_issue_rate"]
PY_PROBES = ["transposed_operands"]


def build(name):
    src, exe = os.path.join(HERE, name + ".hip"), os.path.join(HERE, "_build_" + name)
    if os.path.exists(exe) and os.path.getmtime(exe) >= os.path.getmtime(src):
        return exe
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    res = subprocess.run([hipcc, *FLAGS, src, "-o", exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.exit("hipcc failed:\n" + res.stdout)
    return exe


def main(argv):
    build_only = "--build-only" in argv
    names = [a for a in argv if not a.startswith("--")] or HIP_PROBES + PY_PROBES
    for name in names:
        if name in PY_PROBES:
            if not build_only:
                print(f"== {name}", flush=True)
                subprocess.run([sys.executable, os.path.join(HERE, name + ".py")], check=True, timeout=300)
            continue
        exe = build(name)
        if not build_only:
            print(f"== {name}", flush=True)
            subprocess.run([exe], check=True, timeout=120)


if __name__ == "__main__":
    main(sys.argv[1:])
