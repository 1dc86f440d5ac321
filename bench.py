"""Throughput of the fast-process local step on one MI355X.

--workload mlp runs configs[0] (the small MLP the oracle finishes in seconds: pool 256, k 64, batch 64, 4 steps).

One "step" is one pass of the whole hot path on the ResNet20 fp32 workload: score the 512-image
pool, select the 128 highest-loss samples, run 20 local SGD steps of batch 128 on them, and aggregate
10 parameter replicas with step-count weights.  Prints one JSON line.

--workload resnet20_bf16 measures the mixed-precision variant instead (bf16 activations, fp32 master
weights, pool 4096, k 1024, 50 local steps) and --workload wrn16_8_bf16 the wide residual network
(pool 2048, k 512, 4 local steps, 100 classes); the default line stays the fp32 workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM traffic per launch of the dominant kernel from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE; KiB per
# dispatch averaged over all launches of a bench run), each scaled by what the same counter reads for a plain
# 256 MiB copy (profiles/bench_resnet20_fp32_hbm_traffic.txt).  Valid only for the kernel source it was taken on.
MEASURED_TRAFFIC = {
    "wgrad_kernel": {"fetch_kib": 5268.4, "fetch_scale": 2.0, "write_kib": 4608.0, "write_scale": 1.0,
                     "source": "paper_2508_08540_amd/csrc/conv.hip", "sha256_16": "ba26845e9a8a20c1"},
    # launch-weighted mean over the 18 input-gradient launches of a local step
    "conv_kernel (input-gradient launches)": {"fetch_kib": 12235.5, "fetch_scale": 2.0, "write_kib": 9948.7, "write_scale": 1.0,
                                              "source": "paper_2508_08540_amd/csrc/conv.hip", "sha256_16": "ba26845e9a8a20c1"},
}
HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
BF16_MFMA_PEAK_TFLOPS = 2500.0


def resnet_conv_flops(widths, blocks, hw, in_ch):
    """Algorithmic forward multiply-add flops (2 per MAC) of all 3x3 convolutions for one image."""
    total, c_prev, h = 2 * 9 * in_ch * widths[0] * hw * hw, widths[0], hw
    for s, c in enumerate(widths):
        for b in range(blocks):
            stride = 2 if (b == 0 and s > 0) else 1
            h = h // stride
            total += 2 * 9 * c_prev * c * h * h + 2 * 9 * c * c * h * h
            c_prev = c
    return total


def resnet_dgrad_bytes(widths, blocks, hw, batch, elt):
    """Algorithmic bytes of the input-gradient launches of one local step (layers 1 .. L-1), each tensor counted once.

    The launch of layer l reads its upstream gradient (as the launch above stored it, behind the layer's ReLU) and the
    layer's convolution output (it applies the layer's batch-norm backward itself; the top layer reads a finished dy
    instead), the packed weights, the activation and convolution output of layer l-1 (ReLU mask and batch-norm backward
    sums of that layer) and, for the first layer of a block, the shortcut gradient; it writes dy and dx."""
    layers, c_prev, h = [], widths[0], hw      # (c_in, c_out, h_in, h_out) of layers 1 .. L-1
    for s, c in enumerate(widths):
        for b in range(blocks):
            stride = 2 if (b == 0 and s > 0) else 1
            layers.append((c_prev, c, h, h // stride))
            layers.append((c, c, h // stride, h // stride))
            c_prev, h = c, h // stride
    total = 0
    for i, (c_in, c_out, h_in, h_out) in enumerate(layers):
        out, inn = batch * h_out * h_out * c_out, batch * h_in * h_in * c_in
        conv2, top = i % 2 == 1, i == len(layers) - 1
        elems = (out if top else 2 * out + out) + 2 * inn + inn + 9 * c_in * c_out
        if not conv2:
            elems += batch * h_out * h_out * c_in    # shortcut gradient: the block's output positions, this layer's input channels
        total += elems * elt
    return total


def wrn_conv_flops(widths, blocks, hw, in_ch, stem):
    """(all convolutions, all but the stem): forward multiply-add flops for one image, 1x1 shortcuts included."""
    first = 2 * 9 * in_ch * stem * hw * hw
    total, c_prev, h = first, stem, hw
    for s, c in enumerate(widths):
        for b in range(blocks):
            stride = 2 if (b == 0 and s > 0) else 1
            h_out = h // stride
            total += 2 * 9 * c_prev * c * h_out * h_out + 2 * 9 * c * c * h_out * h_out
            if c_prev != c or stride != 1:
                total += 2 * c_prev * c * h_out * h_out
            h, c_prev = h_out, c
    return total, total - first


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="resnet20_fp32", choices=["resnet20_fp32", "resnet20_b32", "resnet20_bf16", "wrn16_8_bf16", "transformer", "transformer_fp32", "mlp"])
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the run, launch a plain copy of known size (aggregation of one replica with weight 1, "
                         "256 MiB in, 256 MiB out) three times: the reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the workload step, time top-k and aggregation stand-alone over a range of sizes")
    ap.add_argument("--topk-n", type=int, default=0,
                    help="instead of the workload step, run top-k alone on one pool of this size (k = N/4, three calls and a plain "
                         "256 MiB copy for the counter scale): the program behind the top-k profiles")
    ap.add_argument("--round-mode", default=None, choices=["sequential", "2 lanes", "4 lanes", "8 lanes", "batched"],
                    help="with --round: time only this way of running the workers (for profiles)")
    ap.add_argument("--round", action="store_true",
                    help="instead of the workload step, time communication_round (8 ResNet20 workers, 20 steps of 128 each) "
                         "with 1, 2, 4 and 8 workers side by side")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path has no multi-GPU part in this build (run with --gpus 1)")
    if args.sweep:
        return sweep()
    if args.topk_n:
        return topk_alone(args.topk_n)
    if args.round:
        return round_lanes(args.round_mode)

    import numpy as np
    import torch
    import synth
    import paper_2508_08540_amd as bls

    cfg = synth.workload(args.workload)
    N, k, B, tau, P = cfg["pool"], cfg["k"], cfg["batch"], cfg["tau"], cfg["P"]
    act_dtype = cfg.get("act_dtype", "f32")
    wide = cfg["model"] == "wrn16_8"
    seq = cfg["model"] == "transformer"
    mlp = cfg["model"] == "mlp"
    if mlp:
        model = bls.Model.mlp()
        p, b = synth.mlp_init(cfg["id"]), {}
    elif seq:
        model = bls.Model.transformer(act_dtype=act_dtype)
        p, b = synth.transformer_init(cfg["id"]), {}
        x, y = synth.token_pool(cfg["id"], N, cfg["seq_len"], cfg["classes"])
    elif wide:
        model = bls.Model.wide_resnet(act_dtype=act_dtype)
        p, b = synth.wrn_init(cfg["id"])
    else:
        model = bls.Model.resnet_cifar(act_dtype=act_dtype)
        p, b = synth.resnet_init(cfg["id"])
    d = model.num_params
    if not seq:
        x, y = synth.image_pool(cfg["id"], N, cfg["classes"])
    flat = model.pack(p)
    ctx = bls.Context(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    p0 = dev(flat)
    b0 = dev(model.pack(b, buffers=True)) if model.num_buffers else torch.zeros(1, device="cuda")
    dp, db, dm = p0.clone(), b0.clone(), torch.zeros_like(p0)
    dx, dy = dev(x), dev(y)
    if seq:
        # the other workers' replicas only feed the aggregation's bandwidth: seeded perturbations drawn on the device
        gen = torch.Generator(device="cuda").manual_seed(250808540 + cfg["id"])
        others = [p0 + 0.01 * torch.randn(p0.shape, device="cuda", generator=gen) for _ in range(P - 1)]
    else:
        others = [dev(r) for r in synth.replicas(flat, P - 1, cfg["id"])]
    w = bls.weights_from_tau(cfg["tau_workers"]) if "tau_workers" in cfg else np.asarray(cfg["weights"], dtype=np.float32)
    losses = torch.empty(N, dtype=torch.float32, device="cuda")
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    sl = torch.empty(tau * B, dtype=torch.float32, device="cuda")
    agg = torch.empty_like(p0)

    def one_step():
        dp.copy_(p0); db.copy_(b0); dm.zero_()          # every step starts the round from the same global model
        bls.score_losses(ctx, model, dp, db if model.num_buffers else None, dx, dy, losses)
        bls.topk_by_loss(ctx, losses, k, idx)
        bls.local_step(ctx, model, dp, db if model.num_buffers else None, dm, dx, dy, idx, B, tau, cfg["lr"], cfg["momentum"], cfg["weight_decay"], sl)
        bls.weighted_aggregate(ctx, [dp] + others, w, agg)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = tau * B / (elapsed / args.steps)
    finite = bool(torch.isfinite(agg).all().item() and torch.isfinite(sl).all().item())

    # Same steps again with the library's per-class HIP-event timing switched on (on the stream the
    # kernels run on), for the roofline of the dominant kernel class.
    ctx.profile_begin()
    for _ in range(args.steps):
        one_step()
    prof = ctx.profile_end()
    phases = {name: round(ms / args.steps, 4) for name, (ms, cnt) in prof.items() if cnt}
    if mlp:
        # the two products with the 3072 x 128 weight matrix: forward over scored and trained samples, weight gradient
        flop = 2 * 3072 * 128 * ((N + tau * B) + tau * B) * args.steps
        ms, cnt = prof["gemm"]
        achieved = flop / (ms * 1e-3) / 1e12
        line = {"metric": "selected samples/s per local step (MLP 3072-128-10)", "value": round(value, 1), "unit": "samples/s", "n_gpus": 1,
                "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": args.workload, "pool": N, "k": k, "batch": B, "tau": tau, "P": P, "d": int(d)}, "finite": finite,
                "phase_ms_per_step": phases,
                "roofline": {"bound": "mfma", "kernel": "gemm16_kernel (fully connected layer: forward and weight gradient)",
                             "achieved": round(achieved, 3), "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(achieved / FP32_MFMA_PEAK_TFLOPS, 5), "traffic": None, "avg_launch_us": round(1e3 * ms / cnt, 2),
                             "launches_per_step": cnt // args.steps,
                             "note": "products of 64 .. 256 rows: launch latency, not the matrix pipe, bounds this workload"}}
        if not args.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline(cfg, p, b, x, y)
        print(json.dumps(line))
        return
    if seq:
        line = sequence_line(args, cfg, model, prof, phases, value, ms_per_step, finite)
        if not args.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline_sequence(cfg, p, x, y)
        print(json.dumps(line))
        return
    # forward flops of one local step / one scoring pass; the input gradient skips the stem
    if wide:
        conv_flops_img, no_stem = wrn_conv_flops((128, 256, 512), 2, 32, 3, 16)
        stem_flops = conv_flops_img - no_stem
    else:
        conv_flops_img = resnet_conv_flops((16, 32, 64), 3, 32, 3)
        stem_flops = 2 * 9 * 3 * 16 * 32 * 32
    flops = {
        "conv_fwd": conv_flops_img * (tau * B + N),
        "conv_dgrad": (conv_flops_img - stem_flops) * tau * B,
        "conv_wgrad": conv_flops_img * tau * B,
    }
    dom = max(("conv_fwd", "conv_dgrad", "conv_wgrad"), key=lambda c: prof[c][0])
    dom_ms, dom_cnt = prof[dom]
    achieved = flops[dom] * args.steps / (dom_ms * 1e-3) / 1e12
    symbol = {"conv_fwd": "conv_kernel (forward launches)", "conv_dgrad": "conv_kernel (input-gradient launches)",
              "conv_wgrad": "wgrad_kernel"}[dom]
    if wide and dom != "conv_wgrad":
        symbol = symbol.replace("conv_kernel", "wconv_block_kernel and wconv_kernel")
    # forward and input-gradient convolutions run on the matrix instruction of the storage type; the weight
    # gradient always multiplies in fp32
    peak = BF16_MFMA_PEAK_TFLOPS if (act_dtype == "bf16" and dom != "conv_wgrad") else FP32_MFMA_PEAK_TFLOPS
    traffic = None
    rec = MEASURED_TRAFFIC.get(symbol) if args.workload == "resnet20_fp32" else None   # the counters were taken on that workload
    if rec:
        import hashlib
        with open(os.path.join(ROOT, rec["source"]), "rb") as fh:
            if hashlib.sha256(fh.read()).hexdigest()[:16] == rec["sha256_16"]:
                traffic = int(1024 * (rec["fetch_kib"] * rec["fetch_scale"] + rec["write_kib"] * rec["write_scale"]))
    roofline = {"bound": "mfma", "kernel": symbol, "achieved": round(achieved, 3), "peak": peak,
                "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": traffic,
                "avg_launch_us": round(1e3 * dom_ms / dom_cnt, 2), "launches_per_step": dom_cnt // args.steps}
    if traffic is not None:
        # not measured by this run: FETCH_SIZE / WRITE_SIZE of an earlier rocprofv3 run of this same kernel source
        roofline["traffic_source"] = "stored counter run (profiles/bench_resnet20_fp32_hbm_traffic.txt), valid for the current %s" % rec["source"]
    if dom == "conv_dgrad" and not wide:
        # These launches also carry the batch-norm backward (eight tensors per layer against 2*9*C_in*C_out flop per
        # pixel): the roof that binds is the one with the larger minimum time.
        nbytes = resnet_dgrad_bytes((16, 32, 64), 3, 32, B, 2 if act_dtype == "bf16" else 4) * tau
        if nbytes / (HBM_PEAK_GBS * 1e9) > flops[dom] / (peak * 1e12):
            gbs = nbytes * args.steps / (dom_ms * 1e-3) / 1e9
            roofline.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": round(gbs / HBM_PEAK_GBS, 4), "mfma_tflops": round(achieved, 3),
                             "algorithmic_bytes_per_launch": nbytes * args.steps // dom_cnt})

    # Aggregation bandwidth on a vector large enough to leave the caches (WRN-16-8 sized, P = 10),
    # rotating three buffer sets; algorithmic bytes = (P + 1) * d * 4.
    d_big, sets = 11007540, 3
    big = [[torch.randn(d_big, device="cuda") for _ in range(P)] for _ in range(sets)]
    out_big = torch.empty(d_big, device="cuda")
    for s in range(sets):
        bls.weighted_aggregate(ctx, big[s], w, out_big)
    torch.cuda.synchronize()
    reps_n = 30
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps_n):
        bls.weighted_aggregate(ctx, big[i % sets], w, out_big)
    e1.record()
    torch.cuda.synchronize()
    agg_gbs = (P + 1) * d_big * 4 * reps_n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del big

    line = {
        "metric": "selected samples/s per local step (%s)" % ("WRN-16-8" if wide else "ResNet20"), "value": round(value, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": act_dtype, "data": "synthetic",
        "config": {"workload": args.workload, "pool": N, "k": k, "batch": B, "tau": tau, "P": P, "d": int(d)},
        "finite": finite, "phase_ms_per_step": phases, "roofline": roofline,
        "aggregation": {"d": d_big, "P": P, "GB/s": round(agg_gbs, 1), "frac_hbm_peak": round(agg_gbs / HBM_PEAK_GBS, 4)},
    }
    if args.copy_calibration:
        n_cal = 64 * 1024 * 1024
        src, dst = torch.ones(n_cal, device="cuda"), torch.empty(n_cal, device="cuda")
        for _ in range(3):
            bls.weighted_aggregate(ctx, [src], [1.0], dst)
        torch.cuda.synchronize()
        line["copy_calibration"] = {"kernel": "agg_vec4_kernel", "last_launches": 3, "bytes_read": 4 * n_cal, "bytes_written": 4 * n_cal}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, p, b, x, y)
    print(json.dumps(line))


def sequence_line(args, cfg, model, prof, phases, value, ms_per_step, finite):
    """JSON line of the transformer workload; the roofline is that of the GEMM launches (fp32 MFMA).

    Algorithmic flops per token: 2 per weight of the linear layers and the vocabulary projection in each of forward,
    input gradient and weight gradient; the attention products add 4*L*D per layer forward and 8*L*D backward.
    """
    N, k, B, tau, P = cfg["pool"], cfg["k"], cfg["batch"], cfg["tau"], cfg["P"]
    V, L, D, F, layers = cfg["classes"], cfg["seq_len"], 512, 2048, 6
    lin = layers * (4 * D * D + 2 * D * F) + V * D
    tok_train, tok_score = tau * B * L, N * L
    flops = {
        "gemm": (2 * lin + 4 * L * D * layers) * (tok_train + tok_score) + (2 * lin + 8 * L * D * layers) * tok_train,
        "conv_wgrad": 2 * lin * tok_train,
    }
    dom = max(flops, key=lambda c: prof[c][0])
    dom_ms, dom_cnt = prof[dom]
    achieved = flops[dom] * args.steps / (dom_ms * 1e-3) / 1e12
    symbol = {"gemm": "gemm_tiled_kernel (forward, input-gradient and attention launches)",
              "conv_wgrad": "gemm_tiled_kernel (weight-gradient launches) + gemm_split_reduce_kernel"}[dom]
    bf16 = cfg.get("act_dtype") == "bf16"
    peak = BF16_MFMA_PEAK_TFLOPS if bf16 else FP32_MFMA_PEAK_TFLOPS
    symbol = symbol.replace("gemm_tiled_kernel", "gemm16_kernel").replace("gemm_split_reduce_kernel", "gemm16_split_reduce_kernel") if bf16 else symbol
    if bf16 and dom == "gemm":
        symbol = "gemm16_kernel + attention16_kernel (forward, input-gradient and attention launches)"
    roofline = {"bound": "mfma", "kernel": symbol, "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": None, "avg_launch_us": round(1e3 * dom_ms / dom_cnt, 2),
                "launches_per_step": dom_cnt // args.steps}
    return {
        "metric": "selected samples/s per local step (6-layer transformer encoder, sequences of %d tokens)" % L, "value": round(value, 1),
        "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "pool": N, "k": k, "batch": B, "tau": tau, "P": P, "d": int(model.num_params),
                   "seq_len": L, "vocab": V},
        "tokens_per_s": round(value * L, 1), "finite": finite, "phase_ms_per_step": phases, "roofline": roofline,
    }


def cpu_baseline_sequence(cfg, p, x, y):
    """The oracle on the host cores: 4 sequences scored, one local step on 2 sequences, top-k in full, aggregation on a slice."""
    import numpy as np
    import oracle
    from threadpoolctl import threadpool_info
    N, k, B, tau, P = cfg["pool"], cfg["k"], cfg["batch"], cfg["tau"], cfg["P"]
    m = oracle.TransformerLM(cfg["classes"], cfg["seq_len"], operand=oracle.round_bf16 if cfg.get("act_dtype") == "bf16" else None)
    n_score, b_step, d_agg = 4, 2, 4_000_000
    t = time.perf_counter()
    ls = oracle.score_losses(m, p, {}, x[:n_score], y[:n_score])
    t_score = (time.perf_counter() - t) / n_score
    full = np.resize(np.concatenate([ls, ls[::-1]]), N).astype(np.float32)
    t = time.perf_counter()
    sel = oracle.topk_by_loss(full, k)
    t_topk = time.perf_counter() - t
    zeros = {n: np.zeros_like(v) for n, v in p.items()}
    t = time.perf_counter()
    oracle.local_step(m, p, {}, zeros, x, y, sel, b_step, 1, cfg["lr"], cfg["momentum"], cfg["weight_decay"])
    t_step = (time.perf_counter() - t) * (B / b_step)
    d = sum(int(v.size) for v in p.values())
    rng = np.random.default_rng(cfg["id"])
    reps = rng.standard_normal((P, d_agg)).astype(np.float32)
    t = time.perf_counter()
    oracle.weighted_aggregate(reps, oracle.weights_from_tau(cfg["tau_workers"]))
    t_agg = (time.perf_counter() - t) * (d / d_agg)
    total = N * t_score + t_topk + tau * t_step + t_agg
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    return {"value": round(tau * B / total, 3), "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": "scored %d of %d sequences, full top-k, 1 of %d local steps at batch %d (scaled to batch %d), aggregation of "
                      "%d of %d floats (scaled); per-part times scaled to the whole pass" % (n_score, N, tau, b_step, B, d_agg, d),
            "host_cpus": os.cpu_count()}


def _time_calls(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def sweep():
    """Stand-alone top-k (k = N/4, |N(0,1)| + ln 10 losses), epoch sampler and aggregation timings; one JSON line.

    GB/s figures use the algorithmic bytes: 4N + 8k for top-k (read every loss, write k indices and
    values), (P + 1) * 4 * d for aggregation.  Buffers rotate so that repeats are not served from cache.
    """
    import math
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    torch.manual_seed(250808540)
    out = {"metric": "stand-alone top-k and aggregation", "unit": "GB/s (algorithmic bytes)", "hbm_peak": HBM_PEAK_GBS,
           "topk": [], "aggregate": []}
    for N in (512, 4096, 50000, 100000, 1 << 20, 1 << 24, 1 << 26):
        k = N // 4
        sets = 3 if N * 4 < (1 << 28) else 2
        arrs = [torch.randn(N, device="cuda").abs_() + math.log(10.0) for _ in range(sets)]
        idx = torch.empty(k, dtype=torch.int32, device="cuda")
        val = torch.empty(k, dtype=torch.float32, device="cuda")
        reps = 50 if N <= (1 << 20) else 10
        t = _time_calls(torch, lambda i=0: bls.topk_by_loss(ctx, arrs[i % sets], k, idx, val), reps)
        gbs = (4 * N + 8 * k) / t / 1e9
        out["topk"].append({"N": N, "k": k, "us": round(t * 1e6, 2), "GB/s": round(gbs, 2), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
        del arrs
    # epoch sampler at the paper's setting (8 fast and 2 slow workers, tau_F = 32, tau_S = 1), half of the fast
    # allocation by loss; 3 selections over N per call
    out["sample_epoch"] = []
    for N in (50000, 100000, 1 << 20):
        nf, k, ns = bls.epoch_allocation(N, 32, 8, 1, 2, 0.5)
        losses = torch.randn(N, device="cuda").abs_() + math.log(10.0)
        uf, us = torch.rand(N, device="cuda"), torch.rand(N, device="cuda")
        fast = torch.empty(nf, dtype=torch.int32, device="cuda")
        slow = torch.empty(max(ns, 1), dtype=torch.int32, device="cuda")
        t = _time_calls(torch, lambda i=0: bls.sample_epoch(ctx, losses, uf, us, 32, 8, 1, 2, 0.5, fast, slow), 30)
        out["sample_epoch"].append({"N": N, "n_fast": nf, "k": k, "n_slow": ns, "us": round(t * 1e6, 2)})
    for P, d in ((4, 394634), (10, 269722 + 1376), (10, 11007540), (10, 44000000), (10, 51747840)):
        sets = 3
        reps_sets = [[torch.randn(d, device="cuda") for _ in range(P)] for _ in range(sets)]
        w = [1.0 / P] * P
        o = torch.empty(d, device="cuda")
        t = _time_calls(torch, lambda i=0: bls.weighted_aggregate(ctx, reps_sets[i % sets], w, o), 30)
        gbs = (P + 1) * 4 * d / t / 1e9
        out["aggregate"].append({"P": P, "d": d, "us": round(t * 1e6, 2), "GB/s": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)})
        del reps_sets
    print(json.dumps(out))


def topk_alone(N, calls=3):
    """Top-k on one pool of N losses (k = N/4, |N(0,1)| + ln 10), `calls` times, then one plain copy of 256 MiB (aggregation of
    one replica with weight 1) whose FETCH_SIZE / WRITE_SIZE give the scale of the counters; one JSON line."""
    import math
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    torch.manual_seed(250808540)
    k = N // 4
    a = torch.randn(N, device="cuda").abs_() + math.log(10.0)
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, dtype=torch.float32, device="cuda")
    bls.topk_by_loss(ctx, a, k, idx, val)   # sizes the workspace
    t = _time_calls(torch, lambda i=0: bls.topk_by_loss(ctx, a, k, idx, val), calls)
    src, dst = torch.ones(1 << 26, device="cuda"), torch.empty(1 << 26, device="cuda")
    bls.weighted_aggregate(ctx, [src], [1.0], dst)
    torch.cuda.synchronize()
    print(json.dumps({"metric": "top-k alone", "N": N, "k": k, "us": round(t * 1e6, 2), "algorithmic_bytes": 4 * N + 8 * k,
                      "GB/s": round((4 * N + 8 * k) / t / 1e9, 2)}))


def round_lanes(only=None):
    """One communication round of 8 fast workers (ResNet20 fp32, tau = 20, batch 128, 2560 samples each, loss table kept),
    timed with the workers one after the other and 2, 4, 8 side by side; one JSON line, samples/s over all workers."""
    import numpy as np
    import torch
    import synth
    import paper_2508_08540_amd as bls
    cfg = synth.workload("resnet20_fp32")
    P, tau, B = 8, cfg["tau"], cfg["batch"]
    per = tau * B
    N = P * per
    model = bls.Model.resnet_cifar()
    p, b = synth.resnet_init(cfg["id"])
    x, y = synth.image_pool(cfg["id"], 2048, cfg["classes"])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    dx, dy = dev(x).repeat(N // 2048, 1, 1, 1).contiguous(), dev(y).repeat(N // 2048).contiguous()
    ctx = bls.Context(0)
    gp0, gb0 = dev(model.pack(p)), dev(model.pack(b, buffers=True))
    table = torch.zeros(N, device="cuda")
    ws = [dict(tau=tau, idx=torch.arange(i * per, (i + 1) * per, dtype=torch.int32, device="cuda"), params=torch.empty_like(gp0),
               buffers=torch.empty_like(gb0), momentum=torch.zeros_like(gp0)) for i in range(P)]
    out = {"metric": "communication round, samples/s over 8 ResNet20 workers", "unit": "samples/s", "tau": tau, "batch": B, "workers": P,
           "modes": []}
    ref = None
    # the workers one after the other, side by side on 2 / 4 / 8 streams, and side by side inside the kernels (the default)
    for name, lanes, flags in (("sequential", 1, bls.ROUND_SEQUENTIAL), ("2 lanes", 2, 0), ("4 lanes", 4, 0), ("8 lanes", 8, 0), ("batched", 1, 0)):
        if only is not None and name != only:
            continue
        ctx.set_lanes(lanes)
        times = []
        for rep in range(4):
            gp, gb = gp0.clone(), gb0.clone()
            for w in ws:
                w["momentum"].zero_()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            bls.communication_round(ctx, model, gp, gb, ws, dx, dy, B, cfg["lr"], cfg["momentum"], cfg["weight_decay"], table, flags=flags)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        t = min(times[1:])
        same = True if ref is None else bool(torch.equal(ref, gp))
        ref = gp.clone() if ref is None else ref
        out["modes"].append({"mode": name, "ms": round(1e3 * t, 2), "samples/s": round(P * per / t, 1), "same_bits_as_sequential": same})
    ctx.set_lanes(1)
    print(json.dumps(out))


def cpu_baseline(cfg, p, b, x, y):
    """The oracle timed on the host cores on a bounded sample of the same workload: once with the threads the numerical
    library takes by itself, once limited to a single thread (a smaller sample, scaled per image)."""
    import numpy as np
    import oracle
    import synth
    from threadpoolctl import threadpool_info, threadpool_limits
    import paper_2508_08540_amd as bls
    N, k, B, tau, P = cfg["pool"], cfg["k"], cfg["batch"], cfg["tau"], cfg["P"]
    storage = oracle.round_bf16 if cfg.get("act_dtype") == "bf16" else None
    kind = cfg["model"]
    wide, mlp = kind == "wrn16_8", kind == "mlp"
    m = oracle.MLP() if mlp else oracle.WideResNet(storage=storage) if wide else oracle.ResNetCifar(storage=storage)
    flat = (bls.Model.mlp() if mlp else bls.Model.wide_resnet() if wide else bls.Model.resnet_cifar()).pack(p)
    reps = synth.replicas(flat, P, cfg["id"])
    weights = oracle.weights_from_tau(cfg["tau_workers"]) if "tau_workers" in cfg else np.asarray(cfg["weights"], np.float64)
    zeros = {n: np.zeros_like(v) for n, v in p.items()}

    def timed(n_score, b_step):
        t = time.perf_counter()
        ls = oracle.score_losses(m, p, b, x[:n_score], y[:n_score])
        t_score_img = (time.perf_counter() - t) / n_score
        full = np.resize(np.concatenate([ls, ls[::-1]]), N).astype(np.float32)
        t = time.perf_counter()
        sel = oracle.topk_by_loss(full, k)
        t_topk = time.perf_counter() - t
        t = time.perf_counter()
        oracle.local_step(m, p, b, zeros, x, y, sel, b_step, 1, cfg["lr"], cfg["momentum"], cfg["weight_decay"])
        t_step = (time.perf_counter() - t) * (B / b_step)
        t = time.perf_counter()
        oracle.weighted_aggregate(reps, weights)
        t_agg = time.perf_counter() - t
        return tau * B / (N * t_score_img + t_topk + tau * t_step + t_agg)

    n_score = 16 if wide else 64
    b_step = 8 if wide else B        # the wide network's step is timed on a smaller batch and scaled per sample
    value = timed(n_score, b_step)
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    n1, b1 = (4, 2) if wide else (N, B) if mlp else (16, 16)
    with threadpool_limits(limits=1):
        single = timed(n1, b1)
    note = lambda ns, bs: "scored %d of %d pool images, full top-k, 1 of %d local steps at batch %d%s, full aggregation" % (
        ns, N, tau, bs, " (scaled to batch %d)" % B if bs != B else "")
    return {"value": round(value, 2), "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": note(n_score, b_step) + "; per-part times scaled to the whole pass",
            "single_thread": {"value": round(single, 2), "unit": "samples/s", "cores": 1, "sample": note(n1, b1)},
            "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
