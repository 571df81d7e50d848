#!/usr/bin/env python3
"""Benchmark of the per-block INT8 hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch at the GPT-2-small MLP shape
(tokens 4096, in 768, out 3072, block 32), every tensor already resident in HBM:

    quantize X, W, dH  ->  LayerNorm fwd  ->  linear fwd  ->  GELU fwd  ->  GELU bwd
                       ->  linear dgrad + wgrad (one call, jf_linear_bwd)  ->  LayerNorm bwd

`value` is 6*N*C*D INT8 ops (forward + dgrad + wgrad) divided by the wall time of the WHOLE step, i.e. it
charges the quantize / GELU / LayerNorm time to the linear layer as well.  The roofline object describes the
GEMM kernels (two launches per step: the forward product, and both backward products in one grid), timed in
loops of their own -- 5 x 100 back-to-back launches each between HIP events on the launch stream -- and, as a
cross-check, by events around their launches on every n-th step of the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense INT8 matrix peak, TOP/s
HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--block", type=int, default=32)
    ap.add_argument("--tokens", type=int, default=4096)
    ap.add_argument("--in-features", type=int, default=768)
    ap.add_argument("--out-features", type=int, default=3072)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="oracle time budget of the CPU baseline leg")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch plain 256 MiB device copies, the reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--gemm-loop-launches", type=int, default=100,
                    help="back-to-back launches per repeat (5 repeats) of the dedicated GEMM timing loops")
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="skip the compact config 4 (transformer block) and config 5 (large GEMMs) records of the default line")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the GEMM launches with HIP events on every n-th timed step only")
    ap.add_argument("--no-hbm-sized-ops", action="store_true",
                    help="skip timing GELU / LayerNorm / quantize on tensors too large for the last-level cache")
    ap.add_argument("--graph", action="store_true", help="also time the step replayed from a captured HIP graph")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the default step: time fwd/dgrad/wgrad over the large-GEMM sweep (config 5: "
                         "M=N=K in {2048,4096,8192} and tokens 16384 x LLaMA-7B linears, block 32/64/128)")
    ap.add_argument("--block-layer", action="store_true",
                    help="instead of the default step: time one GPT-2-large-shaped transformer block (config 4), forward + "
                         "backward, INT8 data flow between the layers, stock FP16 attention in between")
    ap.add_argument("--sweep-blocks", type=str, default="32,64,128")
    ap.add_argument("--sweep-shape", type=int, default=0, help="force a GEMM tile shape in the sweep (test hook)")
    ap.add_argument("--sweep-only", type=str, default="", help="run one sweep shape only, as tokens,in,out")
    ap.add_argument("--sweep-max-dim", type=int, default=16384, help="skip sweep shapes with a larger dimension")
    return ap.parse_args()


def cpu_baseline(args, N, C, D, block):
    """Time the unmodified oracle on the host cores: the whole step on all cores, the same step on a token slice
    on one core, and (config 5) a sample of output blocks of the 8192^3 forward product, extrapolated."""
    import numpy as np
    import oracle
    from paper_2403_12422_amd import workloads

    g = workloads.rng(77)
    gamma = (1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    Xf, W, dHf = workloads.linear_layer(2, N, C, D)
    oracle.quantize_block(Xf[:block], block)            # load the library outside the timed part

    def oracle_step(X, dH):
        Xq, SX = oracle.quantize_block(X, block)
        Wq, SW = oracle.quantize_block(W, block)
        Gq, SG = oracle.quantize_block(dH, block)
        Xn, SXn, mean, rstd, _ = oracle.layernorm_q(Xq, SX, gamma, beta, 1e-5, block)
        Y, SY, _, _ = oracle.linear_fwd(Xn, SXn, Wq, SW, block)
        oracle.gelu_q(Y, SY, block)
        dY, SdY, _ = oracle.gelu_q_bwd(Gq, SG, Y, SY, block)
        dXn, SdXn, _, _ = oracle.linear_dgrad(dY, SdY, Wq, SW, block)
        oracle.linear_wgrad(dY, SdY, Xn, SXn, block)
        oracle.layernorm_q_bwd(dXn, SdXn, Xq, SX, gamma, mean, rstd, block)

    def timed(fn, seconds, max_reps):
        reps, t0 = 0, time.perf_counter()
        while True:
            fn()
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= seconds or reps >= max_reps:
                return dt / reps, reps

    cores = oracle.max_threads()
    n = min(args.cpu_sample_tokens, N)
    dt_all, reps_all = timed(lambda: oracle_step(Xf[:n], dHf[:n]), args.cpu_seconds, 64)
    # one core: a slice of 512 tokens (weights full size), so that the leg stays within seconds
    n1 = min(512, n)
    oracle.set_threads(1)
    dt_one, reps_one = timed(lambda: oracle_step(Xf[:n1], dHf[:n1]), 0.4 * args.cpu_seconds, 8)
    oracle.set_threads(cores)
    out = {
        "value": 6.0 * n * C * D / dt_all * 1e-12,
        "unit": "TOPS",
        "cores": cores,
        "kind": "oracle",
        "sample": f"whole step on the first {n} of {N} tokens (weights full size), {reps_all} repetitions, "
                  f"{dt_all:.2f} s of oracle time each",
        "single_thread": {"value": 6.0 * n1 * C * D / dt_one * 1e-12, "unit": "TOPS", "cores": 1,
                          "sample": f"whole step on the first {n1} tokens, {reps_one} repetitions, {dt_one:.2f} s each"},
    }
    if not args.no_extra_configs:
        # config 5: 8192^3 forward product at block 32, a seeded sample of 256 output blocks (each over the full K;
        # blocks are independent), extrapolated to the 65536 blocks of the product
        M = 8192
        gq = workloads.rng(85)
        A = gq.integers(-127, 128, size=(M, M), dtype=np.int8)
        Bm = gq.integers(-127, 128, size=(M, M), dtype=np.int8)
        SA = gq.random((M // 32, M // 32), dtype=np.float32) + np.float32(0.01)
        SB = gq.random((M // 32, M // 32), dtype=np.float32) + np.float32(0.01)
        flat = gq.choice((M // 32) ** 2, size=256, replace=False)
        t0 = time.perf_counter()
        oracle.linear_nt_blocks(A, SA, Bm, SB, flat // (M // 32), flat % (M // 32), 32)
        dt = time.perf_counter() - t0
        out["config5_8192_cubed_block32_fwd"] = {
            "value": 2.0 * 256 * 32 * 32 * M / dt * 1e-12, "unit": "TOPS", "cores": cores,
            "sample": f"256 of 65536 output blocks in {dt:.2f} s; the whole product extrapolates to {dt * 256:.0f} s"}
    return out


SWEEP_SHAPES = [  # (tokens N, in C, out D)
    (2048, 2048, 2048), (4096, 4096, 4096), (8192, 8192, 8192),
    (16384, 4096, 4096), (16384, 4096, 11008), (16384, 11008, 4096),
]


def sweep(args, shapes=None, emit=True):
    """Large-GEMM sweep (config 5): kernel time of each product from HIP events around back-to-back launches.

    Values are N(0,1) with 0.5 % outlier columns x50, drawn on the GPU (torch.randn, seeded) because the largest
    tensors have 1.8e8 elements; they are quantized by jf_quantize_block.  One JSON line with one record per
    (shape, block)."""
    import torch

    import paper_2403_12422_amd as jf

    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(240312422 + 5)

    def draw(r, c):
        x = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32)
        n_out = max(1, round(0.005 * c))
        cols = torch.randperm(c, generator=gen, device=dev)[:n_out]
        x[:, cols] *= 50.0
        return x

    def time_ms(fn, ops):
        fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        one = max(e0.elapsed_time(e1), 1e-3)
        reps = int(min(200, max(5, 60.0 / one)))          # about 60 ms of kernel time per measurement
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    jf.jf_debug_set_gemm_shape(args.sweep_shape)
    records = []
    blocks = [int(b) for b in args.sweep_blocks.split(",")]
    if shapes is None:
        shapes = [tuple(int(v) for v in args.sweep_only.split(","))] if args.sweep_only else SWEEP_SHAPES
    for (N, C, D) in shapes:
        if max(N, C, D) > args.sweep_max_dim:
            continue
        Xf, Wf, Gf = draw(N, C), draw(D, C), draw(N, D)
        for B in blocks:
            Xq, SX = jf.jf_quantize_block(Xf, B)
            Wq, SW = jf.jf_quantize_block(Wf, B)
            Gq, SG = jf.jf_quantize_block(Gf, B)
            i8 = lambda r, c: torch.empty((r, c), dtype=torch.int8, device=dev)
            sc = lambda r, c: torch.empty((r // B, c // B), dtype=torch.float32, device=dev)
            oY, odX, odW = (i8(N, D), sc(N, D), None), (i8(N, C), sc(N, C), None), (i8(D, C), sc(D, C), None)
            ops = 2.0 * N * C * D
            ms = {
                "fwd": time_ms(lambda: jf.jf_linear_fwd(Xq, SX, Wq, SW, B, out=oY), ops),
                "dgrad": time_ms(lambda: jf.jf_linear_dgrad(Gq, SG, Wq, SW, B, out=odX), ops),
                "wgrad": time_ms(lambda: jf.jf_linear_wgrad(Gq, SG, Xq, SX, B, out=odW), ops),
            }
            tops = {k: ops / (v * 1e-3) * 1e-12 for k, v in ms.items()}
            total = 3 * ops / (sum(ms.values()) * 1e-3) * 1e-12
            rec = {"tokens": N, "in": C, "out": D, "block": B,
                   "ms": {k: round(v, 4) for k, v in ms.items()},
                   "TOPS": {k: round(v, 1) for k, v in tops.items()},
                   "TOPS_fwd_dgrad_wgrad": round(total, 1), "frac_int8_mfma_peak": round(total / INT8_MFMA_PEAK_TOPS, 4)}
            records.append(rec)
            if emit:
                print(f"# sweep {N}x{C}->{D} block {B}: " + ", ".join(f"{k} {ms[k]:.3f} ms {tops[k]:.0f} TOP/s" for k in ms)
                      + f" | all three {total:.0f} TOP/s ({100 * total / INT8_MFMA_PEAK_TOPS:.1f} % of INT8 MFMA peak)",
                      file=sys.stderr, flush=True)
            del Xq, Wq, Gq, oY, odX, odW
        del Xf, Wf, Gf
        torch.cuda.empty_cache()
    jf.jf_debug_set_gemm_shape(0)
    if not emit:
        return records
    best = max(records, key=lambda r: r["TOPS_fwd_dgrad_wgrad"])
    print(json.dumps({
        "metric": "per-block INT8 linear TOPS (fwd+dgrad+wgrad), large-GEMM sweep", "unit": "TOPS",
        "value": best["TOPS_fwd_dgrad_wgrad"], "n_gpus": 1, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "config 5: large-GEMM sweep; `value` is the best (shape, block) record"},
        "peak_TOPS": INT8_MFMA_PEAK_TOPS, "sweep": records}), flush=True)


def block_layer(args, emit=True):
    """Config 4: one GPT-2-large-shaped transformer block (hidden 1280, 20 heads, FFN 5120, 8 x 1024 tokens, block 32),
    forward + backward with the INT8 data flow between the layers; no bias, no dropout.  The attention core is the
    stock torch FP16 scaled_dot_product_attention (forward and autograd backward); it is timed on its own as well and
    its time is taken out of the INT8 figure.  966.4 GOP of INT8 linear work per step."""
    import torch

    import paper_2403_12422_amd as jf

    dev = torch.device("cuda:0")
    B, batch, seq, H, heads, F = 32, 8, 1024, 1280, 20, 5120
    N = batch * seq
    gen = torch.Generator(device=dev)
    gen.manual_seed(240312422 + 4)
    rnd = lambda r, c, sd: torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * sd
    x = rnd(N, H, 1.0)
    x[:, torch.randperm(H, generator=gen, device=dev)[:13]] *= 20.0
    Q = lambda t: jf.jf_quantize_block(t, B)
    (X, SX), (Wq, SWq), (Wo, SWo), (W1, SW1), (W2, SW2), (dY, SdY) = (
        Q(t) for t in (x, rnd(3 * H, H, 0.02), rnd(H, H, 0.02), rnd(F, H, 0.02), rnd(H, F, 0.02), rnd(N, H, 1e-3)))
    vec = lambda m, sd: (m + sd * torch.randn((H,), generator=gen, device=dev, dtype=torch.float32))
    g1, b1, g2, b2 = vec(1.0, 0.1), vec(0.0, 0.1), vec(1.0, 0.1), vec(0.0, 0.1)
    ws = torch.empty((max(16, jf.jf_workspace_bytes(7, N, H, 0, B)),), dtype=torch.uint8, device=dev)

    def heads_view(t16):
        return t16.view(batch, seq, heads, H // heads).transpose(1, 2)

    def attention(qkv16, grad16=None):
        q, k, v = (heads_view(qkv16[:, i * H:(i + 1) * H]) for i in range(3))
        if grad16 is None:
            o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
            return o.transpose(1, 2).reshape(N, H).contiguous(), None
        q, k, v = (t.detach().requires_grad_(True) for t in (q, k, v))
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
        o.backward(heads_view(grad16))
        dqkv = torch.cat([t.grad.transpose(1, 2).reshape(N, H) for t in (q, k, v)], dim=1).contiguous()
        return None, dqkv

    def step():
        # forward
        A1, SA1, mean1, rstd1 = jf.jf_layernorm_q(X, SX, g1, b1, 1e-5, B)
        QKV, SQKV, _ = jf.jf_linear_fwd(A1, SA1, Wq, SWq, B)
        qkv16 = jf.jf_dequantize_block(QKV, SQKV, B, torch.float16)
        att16, _ = attention(qkv16)
        AT, SAT = jf.jf_quantize_block(att16, B)
        P, SP, _ = jf.jf_linear_fwd(AT, SAT, Wo, SWo, B)
        R1, SR1, rm, rq = jf.jf_add_q(X, SX, P, SP, B, want_partials=True)
        A2, SA2, mean2, rstd2 = jf.jf_layernorm_q_partials(R1, SR1, rm, rq, g2, b2, 1e-5, B)
        H1, SH1, _ = jf.jf_linear_fwd(A2, SA2, W1, SW1, B)
        GE, SGE = jf.jf_gelu_q(H1, SH1, B)
        H2, SH2, _ = jf.jf_linear_fwd(GE, SGE, W2, SW2, B)
        jf.jf_add_q(R1, SR1, H2, SH2, B)
        # backward
        (dGE, SdGE, _), _ = jf.jf_linear_bwd(dY, SdY, W2, SW2, GE, SGE, B)
        dH1, SdH1 = jf.jf_gelu_q_bwd(dGE, SdGE, H1, SH1, B)
        (dA2, SdA2, _), _ = jf.jf_linear_bwd(dH1, SdH1, W1, SW1, A2, SA2, B)
        dR1a, SdR1a, _, _ = jf.jf_layernorm_q_bwd(dA2, SdA2, R1, SR1, g2, mean2, rstd2, B, workspace=ws)
        dR1, SdR1 = jf.jf_add_q(dY, SdY, dR1a, SdR1a, B)
        (dAT, SdAT, _), _ = jf.jf_linear_bwd(dR1, SdR1, Wo, SWo, AT, SAT, B)
        dat16 = jf.jf_dequantize_block(dAT, SdAT, B, torch.float16)
        _, dqkv16 = attention(qkv16, dat16)
        dQKV, SdQKV = jf.jf_quantize_block(dqkv16, B)
        (dA1, SdA1, _), _ = jf.jf_linear_bwd(dQKV, SdQKV, Wq, SWq, A1, SA1, B)
        dXa, SdXa, _, _ = jf.jf_layernorm_q_bwd(dA1, SdA1, X, SX, g1, mean1, rstd1, B, workspace=ws)
        jf.jf_add_q(dR1, SdR1, dXa, SdXa, B)
        return qkv16, dat16

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    steps, warmup = min(args.steps, 50), min(args.warmup, 10)
    qkv16, dat16 = step()
    ms_block = timed(step, steps, warmup)
    ms_attn = timed(lambda: (attention(qkv16), attention(qkv16, dat16)), steps, warmup)
    gop = 2.0 * 3 * N * H * (3 * H + H + F + F) * 1e-9      # fwd + dgrad + wgrad of the four linears
    ms_int8 = ms_block - ms_attn
    rec = {
        "metric": "per-block INT8 linear TOPS (fwd+dgrad+wgrad), transformer block with the INT8 data flow",
        "value": round(gop / ms_int8, 3), "unit": "TOPS (966.4 GOP of INT8 linear work / time of the INT8 operators of one block step)",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_block, 4), "dtype": "int8", "data": "synthetic",
        "config": {"workload": "config 4: GPT-2-large-shaped block, hidden 1280, 20 heads, FFN 5120, 8x1024 tokens, block 32, "
                               "forward + backward, no bias, no dropout; outputs allocated by torch inside the step"},
        "ms_attention_fp16_fwd_bwd": round(ms_attn, 4), "ms_int8_operators": round(ms_int8, 4),
        "int8_linear_gop": round(gop, 1), "frac_int8_mfma_peak": round(gop / ms_int8 / INT8_MFMA_PEAK_TOPS, 4)}
    if emit:
        print(json.dumps(rec), flush=True)
    return rec


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2403_12422_amd as jf
    from paper_2403_12422_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    jf.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.sweep:
        sweep(args)
        return
    if args.block_layer:
        block_layer(args)
        return
    N, C, D, B = args.tokens, args.in_features, args.out_features, args.block

    # ---- synthetic batch (config 2 recipe), resident in HBM before the timed region
    Xh, Wh, dHh = workloads.linear_layer(2, N, C, D)
    g = workloads.rng(77)
    gamma = torch.from_numpy((1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)).to(dev)
    beta = torch.from_numpy((0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)).to(dev)
    X, W, dH = (torch.from_numpy(a).to(dev) for a in (Xh, Wh, dHh))

    i8 = lambda r, c: torch.empty((r, c), dtype=torch.int8, device=dev)
    sc = lambda r, c: torch.empty((r // B, c // B), dtype=torch.float32, device=dev)
    f32 = lambda n: torch.empty((n,), dtype=torch.float32, device=dev)
    Xq, SX, Wq, SW, Gq, SG = i8(N, C), sc(N, C), i8(D, C), sc(D, C), i8(N, D), sc(N, D)
    Xn, SXn, mean, rstd = i8(N, C), sc(N, C), f32(N), f32(N)
    Y, SY, H, SH, dY, SdY = i8(N, D), sc(N, D), i8(N, D), sc(N, D), i8(N, D), sc(N, D)
    dXn, SdXn, dW, SdW = i8(N, C), sc(N, C), i8(D, C), sc(D, C)
    dX, SdX, dgamma, dbeta = i8(N, C), sc(N, C), f32(C), f32(C)
    ws = torch.empty((max(16, jf.jf_workspace_bytes(7, N, C, 0, B)),), dtype=torch.uint8, device=dev)

    gemm_events = []

    def timed_gemm(fn, *a, **kw):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(*a, **kw)
        e1.record()
        gemm_events.append((e0, e1))

    def step(instrument):
        run = timed_gemm if instrument else (lambda fn, *a, **kw: fn(*a, **kw))
        jf.jf_quantize_block(X, B, out=(Xq, SX))
        jf.jf_quantize_block(W, B, out=(Wq, SW))
        jf.jf_quantize_block(dH, B, out=(Gq, SG))
        jf.jf_layernorm_q(Xq, SX, gamma, beta, 1e-5, B, out=(Xn, SXn, mean, rstd))
        run(jf.jf_linear_fwd, Xn, SXn, Wq, SW, B, out=(Y, SY, None))
        jf.jf_gelu_q(Y, SY, B, out=(H, SH))
        jf.jf_gelu_q_bwd(Gq, SG, Y, SY, B, out=(dY, SdY))
        run(jf.jf_linear_bwd, dY, SdY, Wq, SW, Xn, SXn, B, out=((dXn, SdXn, None), (dW, SdW, None)))
        jf.jf_layernorm_q_bwd(dXn, SdXn, Xq, SX, gamma, mean, rstd, B, workspace=ws, out=(dX, SdX, dgamma, dbeta))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i % args.event_every == 0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    if args.pmc_calibration:
        src = torch.ones((256 << 20,), dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                 # reads 256 MiB and writes 256 MiB per launch
        torch.cuda.synchronize()
        del src, dst

    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(False)
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                step(False)
            for _ in range(5):
                gr.replay()
            side.synchronize()
            t0g = time.perf_counter()
            for _ in range(args.steps):
                gr.replay()
            side.synchronize()
            graph_ms = (time.perf_counter() - t0g) / args.steps * 1e3
        torch.cuda.current_stream().wait_stream(side)

    # GEMM launches bracketed inside the timed region (two per instrumented step: forward, backward pair)
    in_step = [e0.elapsed_time(e1) for e0, e1 in gemm_events]
    median = lambda v: sorted(v)[len(v) // 2]
    gemm_ops = 2.0 * N * C * D

    # ---- the GEMM kernels in loops of their own: 5 x 100 back-to-back launches between two events each
    def loop_ms(fn, launches=args.gemm_loop_launches, repeats=5):
        fn()
        torch.cuda.synchronize()
        per_launch = []
        for _ in range(repeats):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                fn()
            e1.record()
            torch.cuda.synchronize()
            per_launch.append(e0.elapsed_time(e1) / launches)
        return {"mean": sum(per_launch) / repeats, "median": median(per_launch), "min": min(per_launch),
                "launches": launches * repeats}

    gemm_loops = {
        "fwd": loop_ms(lambda: jf.jf_linear_fwd(Xn, SXn, Wq, SW, B, out=(Y, SY, None))),
        "bwd_pair": loop_ms(lambda: jf.jf_linear_bwd(dY, SdY, Wq, SW, Xn, SXn, B, out=((dXn, SdXn, None), (dW, SdW, None)))),
        "dgrad_alone": loop_ms(lambda: jf.jf_linear_dgrad(dY, SdY, Wq, SW, B, out=(dXn, SdXn, None))),
        "wgrad_alone": loop_ms(lambda: jf.jf_linear_wgrad(dY, SdY, Xn, SXn, B, out=(dW, SdW, None))),
    }
    step_gemm_ms = gemm_loops["fwd"]["mean"] + gemm_loops["bwd_pair"]["mean"]      # the two launches of a step
    achieved = 3.0 * gemm_ops / (step_gemm_ms * 1e-3) * 1e-12

    # ---- per-op GB/s of the memory-bound kernels (separate, untimed-for-`value` loops with events)
    def op_ms(fn, reps=20, replays=7):
        """Duration of one launch: `reps` back-to-back launches captured in a HIP graph (so that the host-side launch
        cost does not hide the kernel time), replayed `replays` times, each replay between two events; the median
        replay (the first replays of a freshly allocated tensor run slower)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                for _ in range(reps):
                    fn()
            gr.replay()
            times = []
            for _ in range(replays):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                gr.replay()
                e1.record()
                side.synchronize()
                times.append(e0.elapsed_time(e1) / reps)
        torch.cuda.current_stream().wait_stream(side)
        return sorted(times)[len(times) // 2]

    sb = 4.0 / (B * B)
    ops = {
        "quantize_dH_f32": (lambda: jf.jf_quantize_block(dH, B, out=(Gq, SG)), N * D * (5 + sb)),
        "gelu_fwd": (lambda: jf.jf_gelu_q(Y, SY, B, out=(H, SH)), N * D * (2 + 2 * sb)),
        "gelu_bwd": (lambda: jf.jf_gelu_q_bwd(Gq, SG, Y, SY, B, out=(dY, SdY)), N * D * (3 + 3 * sb)),
        "layernorm_fwd": (lambda: jf.jf_layernorm_q(Xq, SX, gamma, beta, 1e-5, B, out=(Xn, SXn, mean, rstd)),
                          N * C * (2 + 2 * sb) + 8 * N + 8 * C),
        "layernorm_bwd": (lambda: jf.jf_layernorm_q_bwd(dXn, SdXn, Xq, SX, gamma, mean, rstd, B, workspace=ws,
                                                        out=(dX, SdX, dgamma, dbeta)),
                          N * C * (3 + 3 * sb) + 8 * N + 12 * C),
    }
    # the residual / dropout operators of the transformer block on the same 4096 x 3072 tensor
    mask_bits = torch.randint(0, 256, (N, D // 8), dtype=torch.uint8, device=dev)
    rm, rq = torch.empty((D // B, N), dtype=torch.float32, device=dev), torch.empty((D // B, N), dtype=torch.float32, device=dev)
    ops["add"] = (lambda: jf.jf_add_q(Y, SY, H, SH, B, out=(dY, SdY)), N * D * (3 + 3 * sb))
    ops["add_with_row_partials"] = (lambda: jf.jf_add_q(Y, SY, H, SH, B, want_partials=True, out=(dY, SdY, rm, rq)),
                                    N * D * (3 + 3 * sb + 8.0 / B))
    ops["dropout"] = (lambda: jf.jf_dropout_q(Y, SY, mask_bits, 0.1, B, out=(dY, SdY)), N * D * (2.125 + 2 * sb))
    # LayerNorm whose statistics come from the row partials of the preceding Add (the paper's own LayerNorm design):
    # partials of the 4096 x 768 input written by an Add of it with a zero tensor
    zq, zs = torch.zeros_like(Xq), torch.zeros_like(SX)
    xr, sxr = torch.empty_like(Xq), torch.empty_like(SX)
    pm, pq = (torch.empty((C // B, N), dtype=torch.float32, device=dev) for _ in range(2))
    jf.jf_add_q(Xq, SX, zq, zs, B, want_partials=True, out=(xr, sxr, pm, pq))
    ops["layernorm_fwd_from_row_partials"] = (
        lambda: jf.jf_layernorm_q_partials(xr, sxr, pm, pq, gamma, beta, 1e-5, B, out=(Xn, SXn, mean, rstd)),
        N * C * (2 + 2 * sb + 8.0 / B) + 8 * N + 8 * C)
    # the hand-over to a floating-point operator (the FP16 attention core): INT8 -> FP16
    h16 = torch.empty((N, D), dtype=torch.float16, device=dev)
    ops["dequantize_f16"] = (lambda: jf.jf_dequantize_block(Y, SY, B, dtype=torch.float16, out=h16), N * D * (3 + sb))
    # and back: the quantizer on an FP16 tensor (what the attention core hands over)
    a16 = dH.to(torch.float16)
    ops["quantize_f16"] = (lambda: jf.jf_quantize_block(a16, B, out=(Gq, SG)), N * D * (3 + sb))
    memops = {}
    for name, (fn, nbytes) in ops.items():
        ms = op_ms(fn)
        memops[name] = {"ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) * 1e-9, 1),
                        "frac_hbm_peak": round(nbytes / (ms * 1e-3) * 1e-9 / HBM_PEAK_GBPS, 4)}

    # The tensors above (6-38 MB) fit the 256 MB last-level cache, so those figures are cache/latency figures.
    # The HBM fraction of the same kernels is measured on tensors of 64x (GELU) / 256x (LayerNorm) the token
    # count, 0.8 GB per operand, which no cache holds; values are codes and scales drawn on the GPU.
    memops_hbm = None
    if not args.no_hbm_sized_ops:
        memops_hbm = {}
        gen = torch.Generator(device=dev)
        gen.manual_seed(240312422 + 3)
        # codes as per-block quantization of Gaussian data leaves them: N(0, 36^2) rounded (a block's max-abs of about
        # 3.5 sigma maps to 127), not uniform over the byte range
        ri8 = lambda r, c: (torch.randn((r, c), generator=gen, device=dev, dtype=torch.float16) * 36.0).round_() \
            .clamp_(-127, 127).to(torch.int8)
        rsc = lambda r, c, m: torch.rand((r // B, c // B), generator=gen, device=dev, dtype=torch.float32) * m + 1e-3 * m
        NG, NL = 64 * N, 256 * N
        xg, sxg, gg, sgg = ri8(NG, D), rsc(NG, D, 0.06), ri8(NG, D), rsc(NG, D, 3e-5)
        yg, syg = i8(NG, D), sc(NG, D)
        big = {
            "gelu_fwd": (lambda: jf.jf_gelu_q(xg, sxg, B, out=(yg, syg)), NG * D * (2 + 2 * sb)),
            "gelu_bwd": (lambda: jf.jf_gelu_q_bwd(gg, sgg, xg, sxg, B, out=(yg, syg)), NG * D * (3 + 3 * sb)),
        }
        big["add"] = (lambda: jf.jf_add_q(xg, sxg, gg, sgg, B, out=(yg, syg)), NG * D * (3 + 3 * sb))
        mbg = torch.randint(0, 256, (NG, D // 8), generator=gen, dtype=torch.uint8, device=dev)
        big["dropout"] = (lambda: jf.jf_dropout_q(xg, sxg, mbg, 0.1, B, out=(yg, syg)), NG * D * (2.125 + 2 * sb))
        # what a plain device-to-device copy of the same tensor reaches (torch's copy kernel): the practical HBM rate
        big["plain_copy_reference"] = (lambda: yg.copy_(xg), NG * D * 2)
        for name, (fn, nbytes) in big.items():
            ms = op_ms(fn, reps=4, replays=7)
            memops_hbm[name] = {"tokens": NG, "ms": round(ms, 4), "GB/s": round(nbytes / (ms * 1e-3) * 1e-9, 1),
                                "frac_hbm_peak": round(nbytes / (ms * 1e-3) * 1e-9 / HBM_PEAK_GBPS, 4)}
        del xg, sxg, gg, sgg, yg, syg, mbg
        torch.cuda.empty_cache()
        xl, sxl, gl, sgl = ri8(NL, C), rsc(NL, C, 0.05), ri8(NL, C), rsc(NL, C, 3e-5)
        yl, syl, ml, rl = i8(NL, C), sc(NL, C), f32(NL), f32(NL)
        wsl = torch.empty((max(16, jf.jf_workspace_bytes(7, NL, C, 0, B)),), dtype=torch.uint8, device=dev)
        jf.jf_layernorm_q(xl, sxl, gamma, beta, 1e-5, B, out=(yl, syl, ml, rl))
        big = {
            "layernorm_fwd": (lambda: jf.jf_layernorm_q(xl, sxl, gamma, beta, 1e-5, B, out=(yl, syl, ml, rl)),
                              NL * C * (2 + 2 * sb) + 8 * NL + 8 * C),
            "layernorm_bwd": (lambda: jf.jf_layernorm_q_bwd(gl, sgl, xl, sxl, gamma, ml, rl, B, workspace=wsl,
                                                            out=(yl, syl, dgamma, dbeta)),
                              NL * C * (3 + 3 * sb) + 8 * NL + 12 * C),
        }
        # the paper's own LayerNorm design: statistics from the row partials of the preceding Add (written here by an Add
        # of the tensor with zeros)
        pml, pql = (torch.empty((C // B, NL), dtype=torch.float32, device=dev) for _ in range(2))
        zl, szl = torch.zeros_like(xl), torch.zeros_like(sxl)
        big["add_with_row_partials"] = (lambda: jf.jf_add_q(xl, sxl, zl, szl, B, want_partials=True, out=(yl, syl, pml, pql)),
                                        NL * C * (3 + 3 * sb + 8.0 / B))
        big["layernorm_fwd_from_row_partials"] = (
            lambda: jf.jf_layernorm_q_partials(xl, sxl, pml, pql, gamma, beta, 1e-5, B, out=(yl, syl, ml, rl)),
            NL * C * (2 + 2 * sb + 8.0 / B) + 8 * NL + 8 * C)
        for name, (fn, nbytes) in big.items():
            ms = op_ms(fn, reps=4, replays=7)
            memops_hbm[name] = {"tokens": NL, "ms": round(ms, 4), "GB/s": round(nbytes / (ms * 1e-3) * 1e-9, 1),
                                "frac_hbm_peak": round(nbytes / (ms * 1e-3) * 1e-9 / HBM_PEAK_GBPS, 4)}
        del pml, pql, zl, szl
        xq = torch.randn((NL // 4, D), generator=gen, device=dev, dtype=torch.float32)
        oq, osq = i8(NL // 4, D), sc(NL // 4, D)
        ms = op_ms(lambda: jf.jf_quantize_block(xq, B, out=(oq, osq)), reps=4, replays=7)
        nbytes = (NL // 4) * D * (5 + sb)
        memops_hbm["quantize_f32"] = {"tokens": NL // 4, "ms": round(ms, 4), "GB/s": round(nbytes / (ms * 1e-3) * 1e-9, 1),
                                      "frac_hbm_peak": round(nbytes / (ms * 1e-3) * 1e-9 / HBM_PEAK_GBPS, 4)}
        del xl, sxl, gl, sgl, yl, syl, ml, rl, wsl, xq, oq, osq
        torch.cuda.empty_cache()

    # HBM traffic of the GEMM kernels and the ceilings of the fold: measured offline (rocprofv3 --pmc resp. the
    # micro-benchmarks), summarised into JSON files under profiles/ by microbench/summarize_profiles.py
    def profile_json(name):
        path = os.path.join(ROOT, "profiles", name)
        return json.load(open(path)) if os.path.exists(path) else None

    traffic = None
    tj = profile_json("bench_config2_hbm_traffic.json")
    if (N, C, D, B) == (4096, 768, 3072, 32) and tj:
        traffic = tj.get("gemm_bytes_per_step_launches")
    fold = profile_json("microbench_fold_ceilings.json")
    ceiling = None
    if fold and str(B) in fold.get("bare_fold_TOPS", {}):
        ceiling = {"bare_TOPS": fold["bare_fold_TOPS"][str(B)],
                   "with_k_loop_overheads_TOPS": fold.get("with_k_loop_overheads_TOPS", {}).get(str(B)),
                   "frac_of_bare": round(achieved / fold["bare_fold_TOPS"][str(B)], 4),
                   "source": fold.get("source")}

    extra = {}
    if not args.no_extra_configs:
        # compact records of the other configurations, so that the one timed line carries them
        recs = sweep(args, shapes=[(8192, 8192, 8192), (16384, 4096, 11008)], emit=False)
        extra["config5"] = [{"tokens": r["tokens"], "in": r["in"], "out": r["out"], "block": r["block"], "ms": r["ms"],
                             "TOPS_fwd_dgrad_wgrad": r["TOPS_fwd_dgrad_wgrad"], "frac_int8_mfma_peak": r["frac_int8_mfma_peak"]}
                            for r in recs]
        bl = block_layer(args, emit=False)
        extra["config4"] = {k: bl[k] for k in ("value", "unit", "ms_per_step", "ms_attention_fp16_fwd_bwd", "ms_int8_operators",
                                               "int8_linear_gop", "frac_int8_mfma_peak")}

    r4 = lambda d: {k: (round(v, 5) if isinstance(v, float) else v) for k, v in d.items()}
    out = {
        "metric": "per-block INT8 linear TOPS (fwd+dgrad+wgrad) + GB/s for INT8 GELU/LayerNorm",
        "value": round(6.0 * N * C * D / (ms_per_step * 1e-3) * 1e-12, 3),
        "unit": "TOPS (6*N*C*D INT8 ops per whole-path step)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "config 2: GPT-2-small MLP, per-block INT8 linear fwd+dgrad+wgrad with quantize, "
                               "GELU and LayerNorm fwd+bwd in the step",
                   "tokens": N, "in_features": C, "out_features": D, "block": B},
        "roofline": {
            "bound": "mfma",
            "kernel": "gemm_kernel (forward product) + gemm_pair_kernel (input and weight gradient in one grid): the two "
                      "GEMM launches of a step, 3 x 2*N*C*D INT8 ops",
            "achieved": round(achieved, 2),
            "peak": INT8_MFMA_PEAK_TOPS,
            "unit": "TFLOP/s",
            "unit_note": "INT8 multiply-accumulate counted as 2 ops (TOP/s)",
            "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
            "traffic": traffic,
            "traffic_note": "HBM bytes of the two GEMM launches of a step, rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a 256 MiB "
                            "copy; algorithmic bytes are 3 x 18.1e6",
            "avg_launch_ms": round(step_gemm_ms / 2, 5),
            "launch_ms": {k: r4(v) for k, v in gemm_loops.items()},
            "launch_ms_note": f"per launch, from 5 x {args.gemm_loop_launches} back-to-back launches between HIP events on the launch stream; "
                              "`achieved` = 6*N*C*D / (fwd mean + bwd_pair mean)",
            "in_step_event_ms": {"fwd_median": round(median(in_step[0::2]), 5), "bwd_pair_median": round(median(in_step[1::2]), 5),
                                 "launches_timed": len(in_step),
                                 "note": "events around the launches inside the timed region; they add about 2.5 us per launch"},
            # second ceiling of this method on this chip: the per-K-block dequantize fold issues 32 / 16 / 8 vector
            # instructions per MFMA at block 32 / 64 / 128 (micro-benchmarks, see the profile named in `source`)
            "valu_fold_ceiling": ceiling,
            "linear_only_TOPS": round(achieved, 2),
        },
        "memory_bound_ops": memops,
        "memory_bound_ops_hbm_sized": memops_hbm,
        "paper_context": "paper reports ratios only: 1.42x transformer-layer speedup, 1.49x activation memory vs FP16 on RTX 4090",
    }
    out.update(extra)
    if graph_ms is not None:
        out["graph_replay_ms_per_step"] = round(graph_ms, 5)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args, N, C, D, B)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
