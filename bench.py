"""Benchmark of the causal attention forward + backward hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: forward, delta
preprocess, delta refinement of the first rows, dK/dV pass and dQ pass, all through the
C-ABI library on torch's current stream, with inputs resident in HBM.  The default
workload is the 7B layer at 128k tokens (B=1, H=32, S=131072, D=128).

Prints ONE JSON line.  ``value`` counts 14*D FLOPs per unmasked (query, key) pair per head
(forward 4*D, backward 10*D including the score recomputation); the paper's Table 1
convention (12*D, no recomputation) is reported beside it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_FLOP_PER_CLK_PER_CU = 4096          # dense bf16 MFMA, 4 SIMDs x 1024
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch at config 4.  NOT measured by this program: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of
# earlier runs of the same kernels at the same workload, scaled by the copy-kernel calibration
# (profiles/hbm_traffic_cfg4.md: fetched x2.00 + written x1.00).  Reported under "traffic" with its source.
TRAFFIC_CFG4_BYTES = {"fwd": (9.704e6 * 2 + 1.065e6) * 1024, "dkdv": (1.860e7 * 2 + 2.097e6) * 1024,
                      "dq": (1.238e7 * 2 + 1.049e6) * 1024}
TRAFFIC_SOURCE = "profiles/hbm_traffic_cfg4.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not collected in this run)"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload id 1..5 (default 4: the metric's workload)")
    ap.add_argument("--share-heads", type=int, default=0,
                    help="instead of a numbered workload: one GPU's share of the heads under 8-way sequence/tensor "
                         "parallelism (Section 2.2; Table 3: 2 heads for 1.3B, 4 for 3B and 7B, 5 for a 13B-like layer), "
                         "through the strided entry points on sequence-major buffers")
    ap.add_argument("--seq", type=int, default=131072, help="sequence length of the --share-heads workload")
    ap.add_argument("--layout", choices=("fused_qkv", "contiguous"), default="fused_qkv",
                    help="--share-heads: q,k,v views of one [S,B,3,H,D] buffer and [S,B,H,D] activations, or [B,H,S,D]")
    ap.add_argument("--overlap", choices=("none", "copy", "cu-mask"), default="none",
                    help="robustness of the path to a concurrent transfer (Section 4.3 hides stage-to-stage transfers "
                         "behind attention; Section 5.3 argues they take few compute units): 'copy' runs device-to-device "
                         "copies on a second stream during the timed steps, 'cu-mask' runs the steps on a stream that "
                         "may use only 256 - N compute units")
    ap.add_argument("--copy-mib", type=int, default=256, help="--overlap copy: size of one copy (256 MiB = one GPU's "
                    "share of the 2*b*s*h bytes a 7B layer boundary moves at 128k tokens, 8-way sequence parallel)")
    ap.add_argument("--copy-gbs", type=float, default=0.0, help="--overlap copy: pace the copies to about this many GB/s "
                    "(0: back to back, as fast as the device copies)")
    ap.add_argument("--masked-cus", type=int, default=16, help="--overlap cu-mask: compute units withheld from the path")
    ap.add_argument("--qkv-linear", action="store_true",
                    help="time the QKV linear layer of the attention stage (Section 4.2) instead of attention: "
                         "M = --seq tokens, K = --hidden, N = 3 * --share-heads * 128 columns (default 4 heads)")
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before anything is timed, copy this many MiB device to device once: a plain copy of known "
                         "size against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=49152)
    return ap.parse_args()


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def sustained_mfma(hx, torch, n_cu):
    """The pure MFMA loop of the library, timed here and now: TFLOP/s with constant and with random operands."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    out = {}
    for name, rnd in (("constant_operands", False), ("random_operands", True)):
        hx.helix_mfma_probe(sink, 2 * n_cu, 2000, rnd)          # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = hx.helix_mfma_probe(sink, 2 * n_cu, 100000, rnd)
        e1.record()
        torch.cuda.synchronize()
        out[name] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # the same loop with the instruction mix of the kernels: 1 LDS operand read per MFMA + 2 fma + 0.5 exp2
    # (backward passes) or + 3 fma + 1 exp2 (forward); one workgroup of 8 waves per compute unit
    for name, fwd_mix in (("random_operands_backward_mix", False), ("random_operands_forward_mix", True)):
        hx.helix_mfma_mix_probe(sink, n_cu, 4000, fwd_mix)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = hx.helix_mfma_mix_probe(sink, n_cu, 150000, fwd_mix)
        e1.record()
        torch.cuda.synchronize()
        out[name] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return out


def cpu_baseline(cfg, sample_tokens):
    """The oracle as it stands, timed on the host cores on a bounded sample."""
    from oracle import attention_ref as A
    from paper_2507_00394_amd import inputs as I

    S = min(cfg.S, sample_tokens)
    x = I.head_inputs(cfg, 0, S=S)
    t0 = time.perf_counter()
    A.head_backward(x["q"], x["k"], x["v"], x["dO"], cfg.scale, cfg.causal)
    dt = time.perf_counter() - t0
    flops = 14 * cfg.D * (S * (S + 1) // 2 if cfg.causal else S * S)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle", "cpu": cpu_model(),
            "sample": f"oracle.attention_ref.head_backward (fp64 forward + gradients) on the first {S} tokens of head 0 "
                      f"of the workload, {dt:.1f} s"}


def share_bench(args):
    """One GPU's share of a layer (few heads, full sequence) on strided views; whole calls only."""
    import torch

    from paper_2507_00394_amd import binding as hx

    B, H, S, D = 1, args.share_heads, args.seq, 128
    scale = D ** -0.5
    n_cu, clock_khz = hx.helix_attn_device_info()
    peak_tflops = n_cu * PEAK_FLOP_PER_CLK_PER_CU * clock_khz / 1e9
    gen = torch.Generator(device="cuda").manual_seed(250700394)
    rnd = lambda *shape: torch.randn(*shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    if args.layout == "fused_qkv":
        qkv, dqkv = rnd(S, B, 3, H, D), torch.empty(S, B, 3, H, D, device="cuda", dtype=torch.bfloat16)
        q, k, v = (qkv[:, :, i].permute(1, 2, 0, 3) for i in range(3))
        dq, dk, dv = (dqkv[:, :, i].permute(1, 2, 0, 3) for i in range(3))
        g = rnd(S, B, H, D).permute(1, 2, 0, 3)
        o = torch.empty(S, B, H, D, device="cuda", dtype=torch.bfloat16).permute(1, 2, 0, 3)
    else:
        q, k, v, g = (rnd(B, H, S, D) for _ in range(4))
        o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    lse = torch.empty(B, H, S, device="cuda", dtype=torch.float32)
    ws = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device="cuda")

    def step(ev=None):
        if ev: ev[0].record()
        hx.helix_attn_fwd_strided(q, k, v, o, lse, scale, True)
        if ev: ev[1].record()
        hx.helix_attn_bwd_strided(q, k, v, o, lse, g, dq, dk, dv, ws, scale, True)
        if ev: ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    unit = S * (S + 1) // 2 * B * H * D
    ms_fwd = float(np.mean([e[0].elapsed_time(e[1]) for e in evs])); ms_bwd = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    value = 14 * unit / (wall / args.steps) / 1e12
    print(json.dumps({
        "metric": "causal attn fwd+bwd TFLOP/s, one GPU's share of the heads at 8-way sequence parallelism; % of bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"per-GPU share: causal MHA fwd+bwd, B={B} H={H} S={S} D={D}, layout {args.layout}, "
                               f"bf16 iid N(0,1), scale=1/sqrt({D})", "B": B, "H": H, "S": S, "D": D, "layout": args.layout},
        "pct_of_bf16_mfma_peak": 100 * value / peak_tflops, "peak_tflops_denominator": peak_tflops,
        "fwd_ms": ms_fwd, "bwd_ms": ms_bwd, "fwd_tflops": 4 * unit / ms_fwd / 1e9, "bwd_tflops": 10 * unit / ms_bwd / 1e9,
        "roofline": None, "cpu_baseline": None}))


def overlap_bench(args, step, flops_per_step):
    """Times `step` alone, then under the chosen disturbance; prints one JSON line."""
    import torch

    def timed(n, stream=None, during=None):
        ctx = torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream())
        with ctx:
            for _ in range(2):
                step()
            torch.cuda.synchronize()
            done = torch.cuda.Event()
            t0 = time.perf_counter()
            for _ in range(n):
                step()
            done.record()
            extra = during(done) if during else None
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n, extra

    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    base, _ = timed(args.steps)
    info = {"mode": args.overlap}
    if args.overlap == "copy":
        side = torch.cuda.Stream()
        n = args.copy_mib << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda"); dst = torch.empty_like(src)
        def during(done):
            copies, t0 = 0, time.perf_counter()
            with torch.cuda.stream(side):
                while not done.query():
                    if args.copy_gbs > 0:
                        ahead = copies * n / (args.copy_gbs * 1e9) - (time.perf_counter() - t0)
                        if ahead > 0:
                            time.sleep(min(ahead, 0.005)); continue
                    elif copies % 64 == 63:
                        side.synchronize()          # keep the queue short: at most 64 copies ahead
                    dst.copy_(src, non_blocking=True); copies += 1
                side.synchronize()
            return copies, time.perf_counter() - t0
        t, (copies, dt) = timed(args.steps, during=during)
        info.update({"copy_mib": args.copy_mib, "copies": copies, "copy_gbs_each_way": copies * n / dt / 1e9,
                     "paced_to_gbs": args.copy_gbs or None})
    else:
        from paper_2507_00394_amd.streams import cu_masked_stream

        t, _ = timed(args.steps, stream=cu_masked_stream(n_cu, args.masked_cus))
        info.update({"masked_cus": args.masked_cus, "cus": n_cu,
                     "slowdown_if_proportional": n_cu / (n_cu - args.masked_cus)})
    info.update({"ms_alone": base * 1e3, "ms_disturbed": t * 1e3, "slowdown": t / base})
    print(json.dumps({"metric": "causal attn fwd+bwd TFLOP/s under a concurrent disturbance", "value": flops_per_step / t / 1e12,
                      "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": 2, "ms_per_step": t * 1e3,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "as the default run, disturbed"}, "alone_tflops": flops_per_step / base / 1e12,
                      "overlap": info, "roofline": None, "cpu_baseline": None}))


def linear_bench(args):
    """The QKV linear layer: forward and backward (input and weight gradients), one GPU's columns."""
    import torch

    from paper_2507_00394_amd import binding as hx
    from paper_2507_00394_amd import inputs as I

    H = args.share_heads or 4
    M, K, N = args.seq, args.hidden, 3 * H * 128
    n_cu, clock_khz = hx.helix_attn_device_info()
    peak_tflops = n_cu * PEAK_FLOP_PER_CLK_PER_CU * clock_khz / 1e9
    gen = torch.Generator(device="cuda").manual_seed(250700394)
    rnd = lambda r, c, std=1.0: (torch.randn(r, c, generator=gen, device="cuda", dtype=torch.float32) * std).to(torch.bfloat16)
    a, w, g = rnd(M, K), rnd(K, N, 0.02), rnd(M, N)
    qkv, da = torch.empty(M, N, device="cuda", dtype=torch.bfloat16), torch.empty(M, K, device="cuda", dtype=torch.bfloat16)
    dw = torch.empty(K, N, device="cuda", dtype=torch.float32)
    ws = torch.empty(max(hx.helix_qkv_linear_bwd_workspace_bytes(M, K, N), 1), dtype=torch.uint8, device="cuda")

    def step(ev=None):
        if ev: ev[0].record()
        hx.helix_qkv_linear_fwd(a, w, qkv)
        if ev: ev[1].record()
        hx.helix_qkv_linear_bwd(a, w, g, da, dw, ws)
        if ev: ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    flops = 2 * M * K * N
    ms_fwd = float(np.mean([e[0].elapsed_time(e[1]) for e in evs])); ms_bwd = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    value = 3 * flops / (wall / args.steps) / 1e12
    out = {"metric": "QKV linear layer fwd+bwd TFLOP/s (Table 1: 6bsh^2 per product, one GPU's columns); % of bf16 MFMA peak",
           "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"qkv[M,N] = a[M,K] w[K,N] and both backward products, M={M} K={K} N={N}, a, dqkv ~ N(0,1), "
                                  f"w ~ N(0, 0.02^2), bf16", "M": M, "K": K, "N": N},
           "pct_of_bf16_mfma_peak": 100 * value / peak_tflops, "fwd_ms": ms_fwd, "bwd_ms": ms_bwd,
           "fwd_tflops": flops / ms_fwd / 1e9, "bwd_tflops": 2 * flops / ms_bwd / 1e9,
           "roofline": {"bound": "mfma", "kernel": "gemm (forward)", "achieved": flops / ms_fwd / 1e9, "peak": peak_tflops,
                        "unit": "TFLOP/s", "frac": flops / ms_fwd / 1e9 / peak_tflops,
                        # profiles/hbm_traffic_qkv_linear.md: FETCH_SIZE x2 + WRITE_SIZE x1 of the forward product
                        "traffic": (1.21e6 * 2 + 3.933e5) * 1024 if (M, K, N) == (131072, 4096, 1536) else None,
                        "flops_per_launch": flops, "avg_launch_ms": ms_fwd}}
    if not args.no_cpu_baseline:
        from oracle import linear_ref as L
        rows = min(M, 65536)
        af, wf, gf = (t.float().cpu().numpy().astype(np.float64) for t in (a[:rows], w, g[:rows]))
        t0 = time.perf_counter(); L.linear_fwd_ref(af, wf); L.linear_bwd_ref(af, wf, gf); dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 3 * 2 * rows * K * N / dt / 1e12, "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"oracle.linear_ref forward + backward (fp64) on the first {rows} rows, {dt:.1f} s"}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every (batch, head) slice is independent; "
              "sharding over heads needs no collective and is not part of this run); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2507_00394_amd import binding as hx
    from paper_2507_00394_amd import inputs as I

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibration_copy_mib > 0:
        src = torch.zeros(args.calibration_copy_mib << 20, dtype=torch.uint8, device=dev)
        torch.empty_like(src).copy_(src)
        torch.cuda.synchronize()
        del src
    if args.qkv_linear:
        return linear_bench(args)
    if args.share_heads:
        return share_bench(args)
    cfg = I.CONFIGS[args.config]
    n_cu, clock_khz = hx.helix_attn_device_info()
    clock_ghz = clock_khz / 1e6
    peak_tflops = n_cu * PEAK_FLOP_PER_CLK_PER_CU * clock_ghz / 1e3

    bits = I.all_inputs_bits(cfg, threads=16)
    q, k, v, g = (torch.from_numpy(bits[t].view(np.int16)).to(dev).view(torch.bfloat16) for t in ("q", "k", "v", "dO"))
    del bits
    B, H, S, D = q.shape
    o = torch.empty_like(q); lse = torch.empty((B, H, S), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    stats = torch.empty(hx.helix_attn_bwd_workspace_bytes(B, H, S, D), dtype=torch.uint8, device=dev)
    stages = ["fwd", "preprocess", "delta_head", "dkdv", "dq"]

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0); hx.helix_attn_fwd(q, k, v, o, lse, cfg.scale, cfg.causal)
        mark(1); hx.helix_attn_bwd_preprocess(o, g, lse, stats)
        mark(2)
        if cfg.causal:
            hx.helix_attn_bwd_delta_head(q, k, v, g, lse, stats, hx.DELTA_HEAD_ROWS, cfg.scale, True)
        mark(3); hx.helix_attn_bwd_dkdv(q, k, v, g, stats, dk, dv, cfg.scale, cfg.causal)
        mark(4); hx.helix_attn_bwd_dq(q, k, v, g, stats, dq, cfg.scale, cfg.causal)
        mark(5)

    if args.overlap != "none":
        return overlap_bench(args, step, 14 * cfg.pairs_per_head * B * H * D)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms = {n: float(np.mean([evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)])) for i, n in enumerate(stages)}
    pairs = cfg.pairs_per_head * B * H
    unit = pairs * D
    ms_step = wall * 1e3 / args.steps
    value = 14 * unit / (wall / args.steps) / 1e12
    ms_bwd = ms["preprocess"] + ms["delta_head"] + ms["dkdv"] + ms["dq"]
    # dominant kernel: the dK/dV pass (4 contractions = 8*D FLOPs per unmasked pair, all of them part of the 10*D a
    # recomputing backward needs)
    flops_per_pair = {"fwd": 4, "dkdv": 8, "dq": 6}
    executed = {n: f * unit / (ms[n] * 1e-3) / 1e12 for n, f in flops_per_pair.items()}
    dom = max(flops_per_pair, key=lambda n: ms[n])
    sustained = sustained_mfma(hx, torch, n_cu)
    pre_bytes = 2 * q.numel() * 2 + 3 * lse.numel() * 4   # reads O, dO, LSE; writes -delta and LSE*log2(e)
    out = {
        "metric": "causal attn fwd+bwd TFLOP/s @H=32,D=128,S=128k; % of bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg_id}: causal MHA fwd+bwd, B={B} H={H} S={S} D={D}, bf16 iid N(0,1)"
                               + (f", K x{cfg.k_mult:g}" if cfg.k_mult != 1 else "") + f", scale=1/sqrt({D})",
                   "B": B, "H": H, "S": S, "D": D, "flops_per_pair": "14*D (fwd 4*D + bwd 10*D)"},
        "pct_of_bf16_mfma_peak": 100 * value / peak_tflops,
        "peak_tflops_denominator": peak_tflops,
        "peak_denominator": f"{n_cu} CU x {PEAK_FLOP_PER_CLK_PER_CU} flop/clk x {clock_ghz:.2f} GHz",
        "fwd_tflops": 4 * unit / (ms["fwd"] * 1e-3) / 1e12,
        "bwd_tflops": 10 * unit / (ms_bwd * 1e-3) / 1e12,
        "fwd_bwd_tflops_table1_convention": 12 * unit / (wall / args.steps) / 1e12,
        "kernel_ms": ms,
        "executed_tflops": executed,
        "executed_frac_of_peak": {n: x / peak_tflops for n, x in executed.items()},
        "sustained_mfma_tflops_measured": sustained,
        "pct_of_sustained_mfma_random": 100 * value / sustained["random_operands"],
        # executed rate of each kernel over the rate of the MFMA loop that carries the same instruction mix
        # (one LDS operand read per MFMA + the kernel's vector work), measured in this run
        "executed_frac_of_mix_probe": {"fwd": executed["fwd"] / sustained["random_operands_forward_mix"],
                                       "dkdv": executed["dkdv"] / sustained["random_operands_backward_mix"],
                                       "dq": executed["dq"] / sustained["random_operands_backward_mix"]},
        "preprocess_gbs": pre_bytes / (ms["preprocess"] * 1e-3) / 1e9,
        "preprocess_frac_of_hbm_peak": pre_bytes / (ms["preprocess"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": executed[dom], "peak": peak_tflops, "unit": "TFLOP/s",
                     "frac": executed[dom] / peak_tflops,
                     "traffic": TRAFFIC_CFG4_BYTES.get(dom) if cfg.cfg_id == 4 else None,
                     "traffic_source": TRAFFIC_SOURCE if cfg.cfg_id == 4 else None,
                     "flops_per_launch": flops_per_pair[dom] * unit, "avg_launch_ms": ms[dom],
                     "whole_step_counted_frac": value / peak_tflops},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
