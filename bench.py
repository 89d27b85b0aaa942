#!/usr/bin/env python3
"""Throughput of the EGTP hot path on one MI355X.

One step = one pass of the whole path over one ragged batch already resident in HBM:
offsets from lengths, fused LM-head + entropy (Eq. 2), entropy-softmax pooling (Eq. 3-4) and the
prediction head.  Prints ONE JSON line with tokens scored per second, the roofline figure of
the dominant kernel (fused LM-head + entropy, priced at 2*d*V FLOP per token against the dense
bf16 matrix-core peak) and the fp64 oracle timed on this machine's host cores on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
FP32_MFMA_PEAK_TFLOPS = 157.3    # MI355X dense fp32 matrix-core peak (what fp32 inputs would be priced against)
HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E peak


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k1_entropy_bf16_serving_hbm_traffic.txt")
K1_SOURCES = [os.path.join(ROOT, "paper_2602_11812_amd", "csrc", f) for f in ("k1_entropy_bf16.hip", "k1_common.h", "k1_plan.cpp")]


def recorded_traffic():
    """HBM bytes per launch of the fused kernel on the serving workload, from the committed rocprofv3
    counter summary -- or None when there is none or the kernel or its launch plan has changed since it was
    taken."""
    import hashlib
    try:
        kv = {}
        for line in open(TRAFFIC_FILE):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                kv[k.strip()] = v.strip()
        sha = hashlib.sha256(b"".join(open(f, "rb").read() for f in K1_SOURCES)).hexdigest()
        if kv.get("kernel_source_sha256") != sha:
            return None
        return float(kv["fetch_bytes_per_launch"]) + float(kv["write_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def bench_plp(args, gpu, wl, np, torch) -> int:
    """PLP decode workload: one step = plp_step over 512 live sequences with one fresh token each
    (fused LM-head + entropy on [512 x d], state fold, remaining-length head).  Reported apart from
    the headline metric; 16 distinct seeded step inputs are cycled."""
    import math
    spec = wl.SPECS["plp_decode"]
    w = wl.make(spec)
    B, d = spec.B, spec.d
    td = gpu.to_device
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w.w1), td(w.w2)))
    hs = [td(wl.decode_hidden(spec, t + 1)) for t in range(16)]
    pooled = torch.zeros(B, d, dtype=torch.float32, device="cuda")
    lse = torch.full((B,), -math.inf, dtype=torch.float32, device="cuda")
    pred = torch.empty(B, dtype=torch.float32, device="cuda")
    ws = sc.workspace(B, B)
    steps = args.steps if args.steps != 10 else 256
    for i in range(max(args.warmup, 1)):
        gpu.plp_step(sc.ctx, hs[i % 16], None, None, None, B, B, pooled, lse, ws, None, pred)
    torch.cuda.synchronize()
    if args.graph:
        # the decode loop as a HIP graph: the 16 distinct steps are captured once and replayed; the fused
        # kernel is timed with events on 64 eager steps afterwards (no events inside the capture)
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(16):
                    gpu.plp_step(sc.ctx, hs[i], None, None, None, B, B, pooled, lse, ws, None, pred)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, steps // 16)
        steps = reps * 16
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        gpu.egtp_profile_enable(sc.ctx, True, 64)
        for i in range(64):
            gpu.plp_step(sc.ctx, hs[i % 16], None, None, None, B, B, pooled, lse, ws, None, pred)
        torch.cuda.synchronize()
        k1_ms = gpu.egtp_profile_read(sc.ctx)
        gpu.egtp_profile_enable(sc.ctx, False)
    else:
        gpu.egtp_profile_enable(sc.ctx, True, min(1024, steps))
        t0 = time.perf_counter()
        for i in range(steps):
            gpu.plp_step(sc.ctx, hs[i % 16], None, None, None, B, B, pooled, lse, ws, None, pred)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        k1_ms = gpu.egtp_profile_read(sc.ctx)
    k1_s = float(k1_ms.mean()) * 1e-3
    flops = 2.0 * spec.d * spec.V * B
    achieved = flops / k1_s / 1e12
    print(json.dumps({
        "metric": "tokens scored/sec (PLP decode step, d=4096 V=151936, 512 sequences x 1 token)",
        "value": B * steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 1),
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"plp_decode: {B} live sequences x 1 new token per step, d={spec.d}, V={spec.V}, "
                               f"remaining-length head {spec.d}->{spec.d_h}->1, seed {spec.seed}", "B": B,
                   "launch": "hip graph of 16 steps" if args.graph else "eager"},
        "roofline": {"kernel": "k1_entropy_bf16 (fused LM-head + entropy)", "bound": "mfma", "achieved": achieved,
                     "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": None, "avg_launch_ms": k1_s * 1e3, "launches": int(k1_ms.size),
                     "w_lm_stream_TBps": spec.V * spec.d * 2 / k1_s / 1e12},
        "cpu_baseline": None}), flush=True)
    return 0


def bench_rl(args, gpu, wl, np, torch) -> int:
    """One-to-many sampling workload (64 prompts x 16 samples, d = 5120, V = 151936): EGTP on the prompts, the
    state copied to each sample's slot, then one step = a ragged plp_step folding the 64 tokens every still-live
    sample has generated since the last call (decode step 64; samples addressed through `slot`)."""
    spec = wl.SPECS["rl_prompts"]
    w = wl.make(spec)
    td = gpu.to_device
    S_PER = 16
    sc = gpu.Scorer(td(w.w_lm), gpu.make_head(td(w.w1), td(w.w2)))
    off = sc.build_offsets(torch.from_numpy(w.lengths).cuda(), w.T)
    out = sc.score(td(w.hidden), off)
    pooled = out["pooled"].repeat_interleave(S_PER, dim=0).contiguous()
    lse = out["lse"].repeat_interleave(S_PER, dim=0).contiguous()
    cont = wl.rl_continuations(spec, S_PER)
    live = np.nonzero(cont >= 64)[0].astype(np.int32)
    T = int(live.size) * 64
    hid = td(wl.draw_hidden(spec, np.random.default_rng([spec.seed, 7, 64]), T))
    coff = torch.from_numpy(np.arange(live.size + 1, dtype=np.int32) * 64).cuda()
    slot = torch.from_numpy(live).cuda()
    pred = torch.empty(live.size, dtype=torch.float32, device="cuda")
    ws = sc.workspace(T, int(live.size))

    def step():
        gpu.plp_step(sc.ctx, hid, coff, None, slot, int(live.size), T, pooled, lse, ws, None, pred)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    gpu.egtp_profile_enable(sc.ctx, True, max(1, min(1024, args.steps)))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k1_s = float(gpu.egtp_profile_read(sc.ctx).mean()) * 1e-3
    achieved = 2.0 * spec.d * spec.V * T / k1_s / 1e12
    print(json.dumps({
        "metric": f"tokens folded/sec (ragged PLP step, d={spec.d} V={spec.V}, 64 tokens per live sample)",
        "value": T * args.steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": max(args.warmup, 1), "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"rl: {spec.B} prompts x {S_PER} samples, {live.size} live at decode step 64, {T} new "
                               f"tokens per call, d={spec.d}, V={spec.V}, head {spec.d}->{spec.d_h}->1, seed {spec.seed}",
                   "B": int(live.size), "T": T},
        "roofline": {"kernel": "k1_entropy_bf16 (fused LM-head + entropy)", "bound": "mfma", "achieved": achieved,
                     "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": None, "avg_launch_ms": k1_s * 1e3},
        "cpu_baseline": None}), flush=True)
    return 0


def bench_pool(args, gpu, wl, np, torch) -> int:
    """Ablation poolers (Table 3) on the serving batch: one step = average pooling of all 137720 hidden states
    over the ragged offsets (no LM head, no entropy).  The roofline is HBM: every hidden state is read once."""
    spec = wl.SPECS["serving"]
    w = wl.make(spec)
    td = gpu.to_device
    sc = gpu.Scorer(td(w.w_lm[:256]), gpu.make_head(td(w.w1), td(w.w2)))   # the poolers never touch W_lm
    hidden = td(w.hidden)
    T, B = hidden.shape[0], spec.B
    off = sc.build_offsets(torch.from_numpy(w.lengths).cuda(), T)
    ws = sc.workspace(T, B)
    pooled = torch.empty(B, spec.d, dtype=torch.float32, device="cuda")
    steps = args.steps if args.steps != 10 else 100
    times = {}
    for kind, name in ((gpu.EGTP_POOL_AVERAGE, "average"), (gpu.EGTP_POOL_MAX, "max"), (gpu.EGTP_POOL_LAST, "last")):
        for _ in range(max(args.warmup, 1)):
            gpu.egtp_pool_ablation(sc.ctx, hidden, off, None, B, T, kind, ws, pooled, None)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            gpu.egtp_pool_ablation(sc.ctx, hidden, off, None, B, T, kind, ws, pooled, None)
        torch.cuda.synchronize()
        times[name] = (time.perf_counter() - t0) / steps
    dt = times["average"]
    gbps = 2.0 * spec.d * T / dt / 1e9
    # what a plain streaming read of the same 1.13 GB reaches on this device (after the timed region)
    sink = torch.empty(gpu.egtp_hbm_read_probe_sink_bytes(), dtype=torch.uint8, device="cuda")
    reads = gpu.egtp_hbm_read_probe(sc.ctx, hidden, sink, 12)
    read_gbps = float(reads[4:].mean())
    print(json.dumps({
        "metric": f"tokens pooled/sec (average pooling over ragged offsets, d={spec.d})",
        "value": T / dt, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 1),
        "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"pool: the serving batch ({B} ragged sequences, {T} tokens, d={spec.d}), poolers only",
                   "B": B, "T": T},
        "ms_per_step_by_pooler": {k: v * 1e3 for k, v in times.items()},
        "roofline": {"kernel": "pool_partial_kernel (sum mode) + join", "bound": "hbm", "achieved": gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "traffic": None},
        "hbm_read_probe": {"what": "plain 16-byte-per-lane streaming read of the same hidden states, mean of the "
                                   "last 8 of 12 launches", "gbps": read_gbps, "achieved_over_probe": gbps / read_gbps},
        "cpu_baseline": None}), flush=True)
    return 0


def bench_train(args, gpu, wl, np, torch) -> int:
    """Head training workload: one step = egtp_head_train_step on a batch of 16 pooled vectors
    (d = 4096, d_h = 1024, K = 20; batch size, K and optimiser of the paper's experimental setup).
    At this batch the step is a stream over W1 and its two AdamW moments (each read and written
    once: 6 x 4 x d_h x d bytes), so the roofline is HBM."""
    B, d, d_h, K = args.train_batch, 4096, 1024, 20
    sets = [wl.make_train(100 + i, B, d, d_h, K) for i in range(4)]
    td = gpu.to_device
    ts = sets[0]
    tr = gpu.HeadTrainer(td(ts.w1), td(ts.b1), td(ts.w2), td(ts.b2), td(ts.centers))
    batches = [(td(t.x), td(t.bins), td(t.y)) for t in sets]
    steps = args.steps if args.steps != 10 else 200
    for i in range(max(args.warmup, 1)):
        tr.step(*batches[i % 4])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        tr.step(*batches[i % 4])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    bytes_w1 = 6.0 * 4.0 * d_h * d
    achieved = bytes_w1 * steps / dt / 1e9
    print(json.dumps({
        "metric": "head training samples/sec (Eq. 5/7 + AdamW step, batch 16, d=4096 d_h=1024 K=20)",
        "value": B * steps / dt, "unit": "samples/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 1),
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"train: batch {B}, d={d}, d_h={d_h}, K={K}, lambda 0.95, AdamW lr 2e-5", "B": B},
        "roofline": {"kernel": "whole step (dominated by train_w1_update: W1 + two moments streamed once)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None},
        "cpu_baseline": None}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="serving", choices=["serving", "mid", "plp_decode", "rl", "pool", "train"],
                    help="serving = the workload the headline metric is quoted on (default)")
    ap.add_argument("--train-batch", type=int, default=16, help="samples per step of --workload train")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"],
                    help="storage type of hidden states and W_lm for --workload serving / mid (bf16 = the headline "
                         "configuration; f32 = the same shapes with fp32 inputs, split into bf16 pieces on the way in)")
    ap.add_argument("--oracle-tokens", type=int, default=640, help="tokens of the CPU-baseline sample (0 = skip)")
    ap.add_argument("--graph", action="store_true",
                    help="--workload plp_decode: replay the decode steps from a captured HIP graph")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the library GEMM of the same shape with the logits written out (context only)")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the register-only MFMA rate measurement reported beside the roofline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed region (reference dispatch for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2602_11812_amd import binding as gpu
    from paper_2602_11812_amd import workloads as wl

    torch.cuda.set_device(0)
    if args.workload == "plp_decode":
        return bench_plp(args, gpu, wl, np, torch)
    if args.workload == "train":
        return bench_train(args, gpu, wl, np, torch)
    if args.workload == "rl":
        return bench_rl(args, gpu, wl, np, torch)
    if args.workload == "pool":
        return bench_pool(args, gpu, wl, np, torch)
    spec = wl.SPECS[args.workload]
    f32 = args.dtype == "f32"
    if f32:
        spec = wl.scaled(spec, dtype="f32")
    t0 = time.time()
    w = wl.make(spec)
    T, B = w.T, spec.B
    print(f"[bench] generated {args.workload}: B={B} T={T} d={spec.d} V={spec.V} in {time.time() - t0:.1f}s",
          file=sys.stderr, flush=True)

    td = gpu.to_device
    w_lm_dev = td(w.w_lm)
    sc = gpu.Scorer(w_lm_dev, gpu.make_head(td(w.w1), td(w.w2)))
    hidden = td(w.hidden)
    lengths = torch.from_numpy(w.lengths).cuda()
    offsets = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    out = dict(entropy=torch.empty(T, dtype=torch.float32, device="cuda"),
               pooled=torch.empty(B, spec.d, dtype=torch.float32, device="cuda"),
               lse=torch.empty(B, dtype=torch.float32, device="cuda"),
               pred=torch.empty(B, dtype=torch.float32, device="cuda"))
    ws = sc.workspace(T, B)

    def step():
        gpu.egtp_build_offsets(sc.ctx, lengths, B, offsets, None, T)
        gpu.egtp_score(sc.ctx, hidden, offsets, None, B, T, ws, out["entropy"], out["pooled"], out["lse"], out["pred"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    gpu.egtp_profile_enable(sc.ctx, True, max(1, min(1024, args.steps)))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k1_ms = gpu.egtp_profile_read(sc.ctx)
    gpu.egtp_profile_enable(sc.ctx, False)
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = T * args.steps / dt
    k1_avg_s = float(k1_ms.mean()) * 1e-3
    flops_per_launch = 2.0 * spec.d * spec.V * T          # algorithmic: 2*d*V per token
    achieved = flops_per_launch / k1_avg_s / 1e12
    # fp32 inputs: six bf16 piece products per fp32 product are what the matrix cores execute
    executed = achieved * (6.0 * ((spec.d + 31) // 32 * 32) / spec.d if f32 else 1.0)
    peak = FP32_MFMA_PEAK_TFLOPS if f32 else BF16_MFMA_PEAK_TFLOPS

    traffic = recorded_traffic()

    # What the matrix cores of this device sustain with nothing else running (after the timed region):
    # 6 launches of about 0.15 s each per operand kind, the mean of the last 4 reported.
    probe = None
    if not args.no_mfma_probe:
        sink = torch.empty(gpu.egtp_mfma_probe_sink_floats(), dtype=torch.float32, device="cuda")
        rnd = gpu.egtp_mfma_probe(sc.ctx, sink, 60000, True, 6)
        zero = gpu.egtp_mfma_probe(sc.ctx, sink, 60000, False, 6)
        probe = {"what": "register-only 16x16x32 bf16 MFMA loop, one wave per SIMD, 1024 workgroups",
                 "random_operands_tflops": float(rnd[2:].mean()), "zero_operands_tflops": float(zero[2:].mean()),
                 "achieved_over_random": executed / float(rnd[2:].mean())}

    # Context, not part of the path: what the vendor GEMM needs for hidden . W_lm^T of the same shape on the same
    # box when the [T x V] logits are written to HBM in bf16 (the tensor this path never writes).
    lib_gemm = None
    if args.library_gemm and not f32:
        w_dev = w_lm_dev
        logits = torch.empty(T, spec.V, dtype=torch.bfloat16, device="cuda")
        for _ in range(2):
            torch.mm(hidden, w_dev.t(), out=logits)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            torch.mm(hidden, w_dev.t(), out=logits)
        e1.record()
        torch.cuda.synchronize()
        gms = e0.elapsed_time(e1) / 5
        lib_gemm = {"what": "torch.mm(hidden, W_lm^T) -> bf16 logits in HBM, same box", "ms": gms,
                    "tflops": flops_per_launch / (gms * 1e-3) / 1e12, "logits_bytes": int(logits.numel()) * 2}
        del logits

    cpu = None
    if args.oracle_tokens > 0:
        import oracle
        n = min(args.oracle_tokens, T)
        off_full = np.concatenate([[0], np.cumsum(w.lengths)]).astype(np.int64)
        sub_off = np.minimum(off_full, n)
        keep = int(np.searchsorted(off_full, n, side="left"))
        sub_off = sub_off[:keep + 1].astype(np.int32)
        t0 = time.perf_counter()
        oracle.egtp(w.hidden[:n], sub_off, w.w_lm, oracle.Head(w.w1, w.w2))
        cdt = time.perf_counter() - t0
        cpu = {"value": n / cdt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {n} tokens ({keep} sequences, the last truncated) of the same batch, full d and V, "
                         f"{cdt:.1f}s"}

    line = {
        "metric": f"tokens scored/sec (EGTP prefill, d={spec.d} V={spec.V}) + % " + ("fp32" if f32 else "bf16") + " MFMA peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}{' with fp32 inputs' if f32 else ''}: EGTP prefill, {B} ragged sequences, {T} tokens, d={spec.d}, "
                               f"V={spec.V}, head {spec.d}->{spec.d_h}->1, seed {spec.seed}",
                   "B": B, "T": T, "d": spec.d, "V": spec.V, "d_h": spec.d_h},
        ("pct_fp32_mfma_peak_whole_step" if f32 else "pct_bf16_mfma_peak_whole_step"):
            100.0 * flops_per_launch / (ms_per_step * 1e-3) / 1e12 / peak,
        "roofline": {"kernel": "k1_entropy_bf16 (fused LM-head + entropy)", "bound": "mfma", "achieved": achieved,
                     "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "executed_bf16_tflops": executed, "executed_frac_of_bf16_peak": executed / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": traffic if args.workload == "serving" and not f32 else None,
                     "traffic_source": ("profiles/k1_entropy_bf16_serving_hbm_traffic.txt (rocprofv3 FETCH_SIZE + "
                                        "WRITE_SIZE passes of an earlier run of this kernel; replayed while the kernel "
                                        "and launch-plan sources hash to the recorded value, not measured in this run)")
                     if traffic is not None and args.workload == "serving" and not f32 else None,
                     "frac_of_measured_mfma_rate": (executed / probe["random_operands_tflops"]) if probe else None,
                     "avg_launch_ms": k1_avg_s * 1e3, "min_launch_ms": float(k1_ms.min()),
                     "max_launch_ms": float(k1_ms.max()), "launches": int(k1_ms.size)},
        "mfma_probe": probe,
        "library_gemm": lib_gemm,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
