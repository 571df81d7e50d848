"""Turn raw rocprofv3 / micro-benchmark output into the short summaries under profiles/.

    python microbench/summarize_profiles.py <raw-dir>     (after the commands quoted in each summary; <raw-dir> is the folder,
                                                            relative to the repository root, that those commands wrote to)

Writes text summaries for people and two JSON files that bench.py reads: profiles/bench_config2_hbm_traffic.json (HBM
bytes of the GEMM launches of a step) and profiles/microbench_fold_ceilings.json (the attainable INT8 rate of the
dequantize fold per block size).  A section whose raw input is missing is skipped.
"""
import collections
import csv
import json
import os
import re
import sys

R = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RAW_NAME = sys.argv[1].rstrip("/") if len(sys.argv) > 1 else sys.exit(__doc__)
RAW = os.path.join(R, RAW_NAME)
OUT = os.path.join(R, "profiles")
PROLOGUE = "(run on the MI355X box from /tmp with TMPDIR=/tmp; paths relative to the repository root)"


def short(name, n=120):
    return re.sub(r"^void ", "", name)[:n]


def have(*paths):
    return all(os.path.exists(os.path.join(RAW, p)) for p in paths)


def write(name, lines):
    with open(os.path.join(OUT, name), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote profiles/" + name)


def stats_table(path, only=None):
    rows = list(csv.DictReader(open(os.path.join(RAW, path))))
    out = [f"{'avg us':>10} {'min us':>10} {'max us':>10} {'calls':>6} {'share %':>8}  kernel"]
    for r in rows:
        if only and not only(r["Name"]):
            continue
        out.append(f"{float(r['AverageNs'])/1e3:10.2f} {float(r['MinNs'])/1e3:10.2f} {float(r['MaxNs'])/1e3:10.2f} "
                   f"{int(r['Calls']):6d} {float(r['Percentage']):8.2f}  {short(r['Name'])}")
    return rows, out


def last_json_line(path):
    lines = [l for l in open(os.path.join(RAW, path)) if l.startswith("{")]
    return lines[-1].strip() if lines else None


# ------------------------------------------------------------------ kernel trace of the default benchmark
def bench_kernel_trace():
    if not have("prof_bench/bench_kernel_stats.csv", "prof_bench/bench_kernel_trace.csv"):
        return
    cmd = f"rocprofv3 --kernel-trace --stats --output-format csv -d {RAW_NAME}/prof_bench -o bench -- python3 bench.py --no-cpu-baseline --no-hbm-sized-ops --no-extra-configs"
    _, table = stats_table("prof_bench/bench_kernel_stats.csv")
    trace = [r for r in csv.DictReader(open(os.path.join(RAW, "prof_bench/bench_kernel_trace.csv"))) if "gemm" in r["Kernel_Name"]]
    trace.sort(key=lambda r: int(r["Start_Timestamp"]))
    per = collections.OrderedDict()
    for r in trace:
        per.setdefault(r["Kernel_Name"], []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    out = ["rocprofv3 kernel-trace summary of the default benchmark (config 2: tokens 4096, in 768, out 3072, block 32)",
           "command " + PROLOGUE + ":", "  " + cmd,
           "220 steps (20 warm-up + 200 timed; two GEMM launches each: gemm_kernel<32, 2, 2, 2, 2, true, true, ..> = forward product on",
           "128x128 tiles, gemm_pair_kernel = input gradient + weight gradient in one grid of 64x64 tiles), then the dedicated timing",
           "loops of bench.py (5 x 100 back-to-back launches of the forward product, the pair, dgrad alone, wgrad alone), then the",
           "per-op loops of the memory-bound kernels at the configured shape.", ""] + table + [""]
    ops = 2.0 * 4096 * 768 * 3072
    out.append("GEMM kernels, by position in the run (us): launches inside the steps run on caches that the step's other kernels")
    out.append("have just used; the loops re-read operands that the previous identical launch left in L2.")
    out.append(f"{'all launches':>14} {'in steps':>10} {'in loops':>10} {'calls':>6}  kernel")
    summary = {}
    for name, d in per.items():
        n_step = 220 if len(d) > 500 else 0
        a, b, c = sum(d) / len(d), (sum(d[:n_step]) / n_step if n_step else float("nan")), sum(d[-500:]) / len(d[-500:])
        out.append(f"{a:14.2f} {b:10.2f} {c:10.2f} {len(d):6d}  {short(name, 100)}")
        summary[name] = (a, b, c)
    fwd = [v for k, v in summary.items() if "gemm_kernel<32, 2, 2, 2, 2, true, true" in k]
    pair = [v for k, v in summary.items() if "gemm_pair_kernel" in k]
    if fwd and pair:
        for label, i in (("all launches", 0), ("launches inside the steps", 1), ("launches of the timing loops", 2)):
            t = fwd[0][i] + pair[0][i]
            out.append(f"forward + backward pair, {label}: {t:.2f} us per step -> {3 * ops / (t * 1e-6) * 1e-12:.1f} TOP/s "
                       f"({3 * ops / (t * 1e-6) * 1e-12 / 5000:.4f} of the 5.0 POP/s INT8 MFMA peak)")
    line = last_json_line("prof_bench.log")
    if line:
        out += ["", "JSON line printed by the profiled run (its HIP-event times carry the profiler's per-dispatch overhead):", line]
    write("bench_config2_kernel_trace.txt", out)


# ------------------------------------------------------------------ HBM traffic of the default benchmark
def bench_hbm_traffic():
    if not have("pmc_fetch/p_counter_collection.csv", "pmc_write/p_counter_collection.csv"):
        return

    def collect(path):
        d = collections.defaultdict(list)
        for r in csv.DictReader(open(os.path.join(RAW, path))):
            d[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return d
    fe, wr = collect("pmc_fetch/p_counter_collection.csv"), collect("pmc_write/p_counter_collection.csv")
    copyk = [k for k in fe if "copyBuffer" in k][0]
    cf, cw = max(fe[copyk]), max(wr[copyk])
    sf, sw = 262144.0 / cf, 262144.0 / cw

    def avg(d, pat):
        v = [x for k in d if pat(k) for x in d[k]]
        return sum(v) / len(v) if v else 0.0
    flags = "--no-cpu-baseline --no-hbm-sized-ops --no-extra-configs --steps 5 --warmup 2 --gemm-loop-launches 2 --pmc-calibration"
    out = ["HBM traffic per launch from two rocprofv3 --pmc runs of the default benchmark workload (config 2)",
           "commands " + PROLOGUE + ":",
           f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d {RAW_NAME}/pmc_fetch -o p -- python3 bench.py {flags}",
           f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d {RAW_NAME}/pmc_write -o p -- python3 bench.py {flags}",
           f"calibration: a plain 256 MiB device-to-device copy (torch copy_, kernel __amd_rocclr_copyBuffer) reads FETCH_SIZE = {cf:.0f}",
           f"and WRITE_SIZE = {cw:.0f} for 262144 KiB each way -> scale factors {sf:.3f} (fetch) and {sw:.3f} (write) KiB per count",
           "", f"{'kernel':44s} {'fetch KiB':>10} {'write KiB':>12} {'total MB':>10}  algorithmic MB"]
    ent = [("gemm forward (gemm_kernel 128x128)", lambda k: "gemm_kernel<32, 2, 2, 2, 2, true, true" in k, 18.2),
           ("gemm dgrad + wgrad (gemm_pair_kernel)", lambda k: "gemm_pair_kernel" in k, 36.3),
           ("gemm dgrad alone (64x64, deep stage)", lambda k: "gemm_kernel<32, 1, 1, 2, 2, true, false" in k, 18.2),
           ("gemm wgrad alone (64x64)", lambda k: "gemm_kernel<32, 1, 1, 2, 2, false, false" in k, 18.2)]
    per = {}
    for name, pat, alg in ent:
        f, w = avg(fe, pat) * sf, avg(wr, pat) * sw
        per[name] = (f + w) * 1024
        out.append(f"{name:44s} {f:10.0f} {w:12.0f} {(f + w) * 1024 / 1e6:10.1f} {alg:15.1f}")
    step = per[ent[0][0]] + per[ent[1][0]]
    out += ["", f"the two GEMM launches of a step: {step / 1e6:.1f} MB (algorithmic 3 x 18.1 = 54.4 MB).",
            "The excess on the read side is re-reading by the eight XCDs: each XCD's L2 pulls its own copy of the operand band it",
            "works on from the Infinity Cache / HBM (FETCH_SIZE counts L2 misses, many of which hit the Infinity Cache).", ""]
    others = [("quantize (mean over X, W, dH)", "quantize_kernel"), ("gelu fwd", "gelu_strip32_kernel<false"), ("gelu bwd", "gelu_strip32_kernel<true"),
              ("layernorm fwd: row statistics", "layernorm_row_stats_kernel"), ("layernorm fwd: normalise (strips)", "layernorm_apply_strip32_kernel"),
              ("layernorm bwd: sums", "layernorm_bwd_sums_kernel"), ("layernorm bwd: dx (strips)", "layernorm_bwd_apply_strip32_kernel"),
              ("colsum (dgamma, dbeta)", "colsum_kernel")]
    for name, key in others:
        f, w = avg(fe, lambda k: key in k) * sf, avg(wr, lambda k: key in k) * sw
        out.append(f"{name:44s} {f:10.0f} {w:12.0f} {(f + w) * 1024 / 1e6:10.1f}")
    write("bench_config2_hbm_traffic.txt", out)
    json.dump({"workload": "config 2 (tokens 4096, in 768, out 3072, block 32)", "gemm_bytes_per_step_launches": int(step),
               "per_kernel_bytes": {k: int(v) for k, v in per.items()}, "source": "profiles/bench_config2_hbm_traffic.txt"},
              open(os.path.join(OUT, "bench_config2_hbm_traffic.json"), "w"), indent=1)
    print("wrote profiles/bench_config2_hbm_traffic.json")


# ------------------------------------------------------------------ large-GEMM sweep
def sweep_trace():
    if not have("prof_sweep/sweep_kernel_stats.csv", "prof_sweep.log"):
        return
    _, table = stats_table("prof_sweep/sweep_kernel_stats.csv", only=lambda n: "jf::" in n)
    log = [l.rstrip() for l in open(os.path.join(RAW, "prof_sweep.log")) if l.startswith("# sweep")]
    out = ["rocprofv3 kernel-trace summary of the large-GEMM sweep (config 5: M=N=K in {2048,4096,8192}, tokens 16384 x LLaMA-7B linears; block 32/64/128)",
           "command " + PROLOGUE + ":",
           f"  rocprofv3 --kernel-trace --stats --output-format csv -d {RAW_NAME}/prof_sweep -o sweep -- python3 bench.py --sweep",
           "A kernel name covers all shapes of one (block, product, tile shape), so the averages below mix shapes; the per-shape",
           "figures are the '# sweep' lines the run prints (HIP events around back-to-back launches), copied underneath.", ""] + table + [""] + log
    write("sweep_config5_kernel_trace.txt", out)


# ------------------------------------------------------------------ memory-bound operators on HBM-sized tensors
def hbm_sized_trace():
    if not have("prof_hbm/hbm_kernel_trace.csv", "prof_hbm.log"):
        return
    rows = [r for r in csv.DictReader(open(os.path.join(RAW, "prof_hbm/hbm_kernel_trace.csv"))) if "jf::" in r["Kernel_Name"]]
    per = collections.defaultdict(list)
    for r in rows:
        per[(r["Kernel_Name"], int(r["Grid_Size_X"]))].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    out = ["rocprofv3 kernel trace of the memory-bound operators on tensors that no cache holds (0.8 GB per operand: 262144 x 3072 for",
           "GELU / Add / Dropout, 1048576 x 768 for LayerNorm and the FP32 quantizer of 262144 x 3072), block 32",
           "command " + PROLOGUE + ":",
           f"  rocprofv3 --kernel-trace --output-format csv -d {RAW_NAME}/prof_hbm -o hbm -- python3 bench.py --no-cpu-baseline --no-extra-configs --steps 5 --warmup 2 --gemm-loop-launches 2",
           "Only launches of at least 100 us are listed (the same kernels also run on the configured shapes).  GB/s = algorithmic bytes",
           "of the operator (as in bench.py) / the kernel's average duration; LayerNorm forward and backward are two resp. three kernels.", "",
           f"{'avg us':>10} {'min us':>10} {'calls':>6} {'grid':>10}  kernel"]
    for (name, grid), d in sorted(per.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
        if sum(d) / len(d) >= 100.0:
            out.append(f"{sum(d) / len(d):10.1f} {min(d):10.1f} {len(d):6d} {grid:10d}  {short(name, 110)}")
    line = last_json_line("prof_hbm.log")
    if line:
        j = json.loads(line)
        out += ["", "memory_bound_ops_hbm_sized of the JSON line of the same run (graph replays between HIP events):"]
        for k, v in j.get("memory_bound_ops_hbm_sized", {}).items():
            out.append(f"  {k:34s} {v['ms'] * 1e3:9.1f} us {v['GB/s']:8.1f} GB/s  {v['frac_hbm_peak']:.3f} of 8 TB/s")
    write("memory_bound_ops_hbm_sized_kernel_trace.txt", out)


# ------------------------------------------------------------------ matrix-core / vector-ALU utilisation of the GEMMs
def gemm_pmc():
    tags = [("bench", "config 2 (tokens 4096, in 768, out 3072, block 32): forward, backward pair, dgrad and wgrad alone"),
            ("sweep", "8192 x 8192 -> 8192, blocks 32 / 64 / 128: forward, dgrad, wgrad each")]
    if not all(have(f"pmcg_{t}_{p}/p_counter_collection.csv") for t, _ in tags for p in "ab"):
        return
    c1 = "SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_WAIT_INST_ANY"
    c2 = "SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_WAIT_ANY SQ_INSTS_SALU SQ_WAVES TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum"
    b = "python3 bench.py --no-cpu-baseline --no-hbm-sized-ops --no-extra-configs --steps 10 --warmup 2 --gemm-loop-launches 2"
    out = ["rocprofv3 --pmc counters of the GEMM kernels: matrix-core and vector-ALU utilisation, LDS, L2 (MI355X, one GPU)",
           "commands " + PROLOGUE + "; two runs per workload because one run holds at most 8 SQ and 4 TCC counters:",
           f"  rocprofv3 --pmc {c1} --output-format csv -d {RAW_NAME}/pmcg_bench_a -o p -- {b}",
           f"  rocprofv3 --pmc {c2} --output-format csv -d {RAW_NAME}/pmcg_bench_b -o p -- {b}",
           "  the same two counter sets with `-- python3 bench.py --sweep --sweep-only 8192,8192,8192` (directories pmcg_sweep_a / pmcg_sweep_b)",
           "units: SQ_BUSY_CU_CYCLES = cycles summed over the 256 compute units; SQ_VALU_MFMA_BUSY_CYCLES = cycles summed over the 1024 SIMDs",
           "(32 per v_mfma_i32_32x32x32_i8); SQ_ACTIVE_INST_VALU and SQ_WAVE_CYCLES count 4-cycle quads per SIMD resp. wave.",
           "  matrix-core busy = MFMA_BUSY / (4 x BUSY_CU);  vector-ALU issue busy = 4 x ACTIVE_INST_VALU / (4 x BUSY_CU);",
           "  VALU per MFMA = (INSTS_VALU - INSTS_MFMA) / INSTS_MFMA (32 / 16 / 8 is the minimum for block 32 / 64 / 128);",
           "  L2 miss = TCC_MISS / TCC_REQ (requests of up to 128 B);  wave waiting = WAIT_INST_ANY / WAVE_CYCLES.", ""]
    hdr = f"{'kernel':66s} {'MFMA busy':>9} {'VALU busy':>9} {'VALU/MFMA':>9} {'LDS act':>8} {'L2 miss':>8} {'L2 req M':>9} {'wait':>6}"
    for tag, title in tags:
        res = collections.defaultdict(lambda: collections.defaultdict(list))
        for part in "ab":
            for r in csv.DictReader(open(os.path.join(RAW, f"pmcg_{tag}_{part}/p_counter_collection.csv"))):
                if "gemm" in r["Kernel_Name"]:
                    res[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
        out += [title, hdr]
        for k, c in res.items():
            m = re.search(r"(gemm_(?:pair_)?kernel)<(.*)>", k)
            name = (("pair " if "pair" in m.group(1) else "") + m.group(2))[:64]
            a = lambda n: sum(c[n]) / len(c[n]) if c[n] else float("nan")
            busy = a("SQ_BUSY_CU_CYCLES") * 4
            out.append(f"{name:66s} {a('SQ_VALU_MFMA_BUSY_CYCLES') / busy:9.3f} {4 * a('SQ_ACTIVE_INST_VALU') / busy:9.3f} "
                       f"{(a('SQ_INSTS_VALU') - a('SQ_INSTS_MFMA')) / a('SQ_INSTS_MFMA'):9.1f} {a('SQ_LDS_IDX_ACTIVE') / a('SQ_BUSY_CU_CYCLES'):8.3f} "
                       f"{a('TCC_MISS_sum') / a('TCC_REQ_sum'):8.3f} {a('TCC_REQ_sum') / 1e6:9.2f} {a('SQ_WAIT_INST_ANY') / a('SQ_WAVE_CYCLES'):6.3f}")
        out.append("")
    out += ["Template arguments: block, sub-blocks per wave (rows, columns), waves per workgroup (rows, columns), A K-major, B K-major, ...",
            "Reading: at block 32 and 64 the vector ALU is the saturated pipe and the matrix cores are busy a fraction of the time that",
            "follows from the fold's instruction count per MFMA (Sec. 5.3): the dequantize fold bounds the kernel, not the MFMA rate."]
    write("gemm_pmc_mfma_valu_utilisation.txt", out)


# ------------------------------------------------------------------ micro-benchmarks
def microbench():
    if not have("microbench.txt"):
        return
    text = [l for l in open(os.path.join(RAW, "microbench.txt")).read().rstrip().split("\n") if "amdgpu.ids" not in l]
    head = ["Micro-benchmarks of the machine limits the kernels are judged against (MI355X, one GPU).",
            "command (run on the MI355X box from the repository root):",
            f"  python -m microbench > {RAW_NAME}/microbench.txt",
            "fold_issue_rate: time of one wave-iteration on a SIMD for the instruction mixes of the dequantize fold (Sec. 5.3), operands",
            "  that no MFMA writes; '1 mfma + 16 cvt + 16 fmac' / '+ 8 cvt + 8 fmac' / '+ 4 cvt + 4 fmac' are block size 32 / 64 / 128;",
            "  'MFMA rate' = 65536 ops x 1024 SIMDs / that time.  fold_chain_rate: the same mixes with the real data flow (the fold reads the",
            "  tile the previous MFMA chain wrote, tiles in VGPRs).  kloop_overheads: the block-32 pattern of fold_chain_rate plus, one kind at a",
            "  time, the other instructions of the real K loop (variant 1: one ds_read_b128 per unit; 2: + stage barrier; 3: + direct-to-LDS",
            "  loads with 64-bit lane addresses; 4: + scalar scale loads and their product; 5: loads with scalar base + 32-bit lane offset,",
            "  the form the GEMM kernel uses; 6: 5 with a stage's eight fragment reads issued at once).  kloop_model: the whole K loop",
            "  written the naive way for the tile shapes and block sizes in use ('KC' = K bytes per stage).  l2_bandwidth: bytes per",
            "  second into the compute units.  quantizer_issue_rate: issue cost per element of the Eq. 1 rounding variants and of the other",
            "  instructions of the memory-bound kernels.  transposed_operands: the weight gradient with its operands transposed inside the",
            "  kernel against the same product from pre-transposed copies, and what writing those copies costs the quantizer.", ""]
    write("microbench_machine_limits.txt", head + text)
    bare, loop = {}, {}
    for l in text:
        m = re.match(r"block\s+(\d+) \(chain of \d\), tiles in VGPRs, (\d) waves/SIMD:\s+[\d.]+ ns per MFMA ->\s+(\d+) TOP/s", l)
        if m:
            bare[m.group(1)] = max(bare.get(m.group(1), 0.0), float(m.group(3)))
        m = re.match(r"variant 5, (\d) waves/SIMD:\s+[\d.]+ ns per MFMA\+fold ->\s+(\d+) TOP/s", l)
        if m:
            loop["32"] = max(loop.get("32", 0.0), float(m.group(2)))
        m = re.match(r"B=(\d+)\s+\S+, \d waves\s+full loop \d waves/SIMD:\s+[\d.]+ ns per MFMA ->\s+(\d+) TOP/s", l)
        if m and m.group(1) != "32":
            loop[m.group(1)] = max(loop.get(m.group(1), 0.0), float(m.group(2)))
    json.dump({"bare_fold_TOPS": bare, "with_k_loop_overheads_TOPS": loop, "peak_TOPS": 5000.0,
               "note": "best over 2-4 waves per SIMD; bare = MFMA chain + fold with no memory traffic (fold_chain_rate), with overheads = "
                       "plus fragment reads, stage barrier, direct-to-LDS loads, scale loads (kloop_overheads variant 5 at block 32, kloop_model at 64 / 128)",
               "source": "profiles/microbench_machine_limits.txt"}, open(os.path.join(OUT, "microbench_fold_ceilings.json"), "w"), indent=1)
    print("wrote profiles/microbench_fold_ceilings.json")


if __name__ == "__main__":
    for fn in (bench_kernel_trace, bench_hbm_traffic, sweep_trace, hbm_sized_trace, gemm_pmc, microbench):
        fn()
