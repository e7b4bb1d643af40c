"""Throughput of one GPU's share of a codistillation step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic minibatch, inputs
already resident in HBM: local forward (kept for backward), peer forward
(nothing kept), codistillation loss + gradient, local backward, momentum-SGD.
Workload: two ResNet-50 (bf16 compute, fp32 master weights), batch 256 of
224x224x3 images ~ N(0,1), 1000 uniform classes, alpha = 1.

Prints ONE JSON line.  `roofline` is for the kernel that takes the most time of the step,
bn_apply_k<bf16,8,true> (the elementwise pass of every BatchNorm forward, both models):
HBM-bound, algorithmic bytes (input, residual, output and ReLU bit mask, each once) over
the HIP-event time of its launches.  `roofline_conv` is the same for the convolution kernel
that takes the most time, igemm_kernel<0,128,256,2,2,false,1,1,false,0,false> (bf16 MFMA
implicit GEMM, forward, 128x256 tiles): its arithmetic intensity decides which roof bounds
it, and its fraction of the MFMA peak is given either way.  Both are measured in a second
pass of the same steps with the library's per-launch event timer (events on the launch
stream) switched on; that pass keeps every launch on one stream, while the timed steps run
the peer forward and the weight gradients on second streams.  `cpu_baseline` is the float64
NumPy oracle of the same step timed on the host on a small batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the two roofline kernels from hardware counters (two rocprofv3 --pmc passes of
# this script, FETCH_SIZE then WRITE_SIZE, each scaled by what the same counter read for the 1 GiB copy of
# --copy-calibration).  Valid only for the kernels the counters were taken on: set to None when one changes.
TRAFFIC_SOURCE = "profiles/resnet50_bs256_step_hbm_counters.md"
ROOFLINE_TRAFFIC_BYTES = 260.2e6        # bn_apply_k<bf16,8,true>: FETCH_SIZE 76166.7 KiB x 2.000 + WRITE_SIZE 101792.6 KiB x 1.000
ROOFLINE_CONV_TRAFFIC_BYTES = 221.0e6   # igemm_kernel<0,128,256,...>: FETCH_SIZE 40974.9 KiB x 2.000 + WRITE_SIZE 133859.5 KiB x 1.000
# Matrix-pipe busy share of that convolution kernel from hardware counters (SQ_VALU_MFMA_BUSY_CYCLES over
# GRBM_GUI_ACTIVE x 1024 SIMDs, mean over its dispatches); None when the kernel changes.
MFMA_COUNTER_SOURCE = "profiles/resnet50_bs256_step_mfma_counters.md"
ROOFLINE_CONV_MFMA_BUSY = 0.231


def roofline_of(flops, nbytes, ms, launches, kernel, traffic, event_overhead_us=None):
    """Roofline entry of one kernel class from its algorithmic flops and HBM bytes (every operand once) and
    the HIP-event time of its launches.  The bound is the roof its arithmetic intensity puts it under: HBM
    below the machine's ridge (peak flops / peak bytes), MFMA above; `achieved` is in that roof's unit and the
    fraction of the MFMA peak is given either way."""
    tflops = flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    gbs = nbytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    intensity = flops / nbytes if nbytes > 0 else 0.0
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    hbm_bound = intensity < ridge
    return {"bound": "hbm" if hbm_bound else "mfma",
            "achieved": gbs if hbm_bound else tflops,
            "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
            "unit": "GB/s" if hbm_bound else "TFLOP/s",
            "frac": gbs / PEAK_HBM_GBS if hbm_bound else tflops / PEAK_BF16_TFLOPS,
            "traffic": traffic, "traffic_source": TRAFFIC_SOURCE if traffic is not None else None,
            "algorithmic_bytes_per_launch": nbytes / max(launches, 1),
            "flop_per_launch": flops / max(launches, 1),
            "intensity_flop_per_byte": intensity, "ridge_flop_per_byte": ridge,
            "mfma_tflops": tflops, "mfma_frac": tflops / PEAK_BF16_TFLOPS,
            "kernel": kernel, "avg_launch_us": ms / max(launches, 1) * 1e3,
            # what the event pair itself adds to every launch (measured around an empty kernel): `achieved` keeps it
            # in, so a profiler's kernel durations are shorter by about this much
            "event_pair_overhead_us": event_overhead_us}


def cpu_baseline(seconds_hint=24.0):
    """Oracle step (ResNet-50, 224x224, small batch) on the host cores, with the BLAS thread pool at all cores and at
    one thread: a baseline, not a target.  Each setting: one calibration step at batch 2, then repeated steps at a batch
    sized so that the setting takes about seconds_hint / 2 seconds; the median step time is reported."""
    import numpy as np
    from oracle import nets
    from oracle.step import codistill_step
    from paper_2010_02838_amd import synth
    from threadpoolctl import threadpool_info, threadpool_limits
    all_cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    arch = nets.resnet50()
    th = synth.round_bf16(synth.he_init(arch.params, 1)).astype(np.float64)
    thp = synth.round_bf16(synth.he_init(arch.params, 2)).astype(np.float64)

    def run(batch):
        x = synth.round_bf16(synth.images(batch, 224, 224, 3, 0)).astype(np.float64)
        y = synth.labels(batch, 1000, 3)
        t0 = time.time()
        codistill_step(arch, th, [thp], x, y, 1.0, 0.1, 0.9)
        return time.time() - t0

    def measure(threads, budget):
        with threadpool_limits(limits=threads):
            per_sample = run(2) / 2                        # calibration
            reps = 3
            batch = int(max(1, min(24, budget / reps / per_sample)))
            times = sorted(run(batch) for _ in range(reps))
        med = times[len(times) // 2]
        return {"value": batch / med, "cores": int(threads), "batch": batch, "steps": reps, "median_step_s": med,
                "step_s": times}

    full = measure(all_cores, seconds_hint * 0.5)
    one = measure(1, seconds_hint * 0.5)
    return {"value": full["value"], "unit": "samples/s", "cores": full["cores"], "kind": "oracle",
            "sample": "float64 NumPy oracle step, ResNet-50 224x224: median of %d steps at batch %d with %d BLAS threads "
                      "(%.1f s per step); one thread: median of %d steps at batch %d (%.1f s per step)"
                      % (full["steps"], full["batch"], full["cores"], full["median_step_s"], one["steps"], one["batch"],
                         one["median_step_s"]),
            "all_threads": full, "one_thread": one}


def loss_kernel_cfg5(B, torch, dev, iters=20):
    """The fused loss kernel alone at [8192 x 32768] fp32, alpha 0.5 (HBM-bound: 12 bytes per logit pair)."""
    rows, cols = 8192, 32768
    g = torch.Generator(device=dev)
    g.manual_seed(11)
    z = torch.randn(rows, cols, device=dev, generator=g) * 3
    zp = torch.randn(rows, cols, device=dev, generator=g) * 3
    t = torch.randint(0, cols, (rows,), device=dev, dtype=torch.int32, generator=g)
    dz, loss = torch.empty_like(z), torch.zeros(4, device=dev)
    scratch = torch.empty(B.loss_scratch_bytes(rows, cols), dtype=torch.uint8, device=dev)
    out = {}
    for mode, name in ((B.CD_DIST_MSE_LOGITS, "mse_logits"), (B.CD_DIST_KL, "kl")):
        for _ in range(3):
            B.codistill_loss_grad(z, [zp], t, loss, dz, scratch, 0.5, 0.0, mode)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B.codistill_loss_grad(z, [zp], t, loss, dz, scratch, 0.5, 0.0, mode)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        gbs = rows * cols * 12 / (ms * 1e-3) / 1e9
        out[name] = {"ms": ms, "GB/s": gbs, "frac": gbs / PEAK_HBM_GBS, "rows_per_s": rows / (ms * 1e-3)}
    del z, zp, dz
    torch.cuda.empty_cache()
    return out


def transformer_head(args, B, synth, StepRunner, pack_flat, to_device, torch, dev):
    """One codistillation step of the Transformer output block (two models: d_model 512, d_ff 2048,
    vocabulary 32768, bf16) on 8192 target tokens: hidden states ~ N(0,1), targets uniform, label
    smoothing 0.1, alpha 1.  roofline: the fp32-output vocabulary projection (one launch per forward)."""
    rows, d, vocab = 8192, 512, 32768
    arch = B.arch_preset(B.CD_ARCH_TRANSFORMER_HEAD)
    model, peer = B.Model(arch, B.CD_BF16), B.Model(arch, B.CD_BF16)
    table = model.param_table()
    r = StepRunner(model, [peer], rows, dev)
    r.load(pack_flat(model, synth.he_init(table, 1)), [pack_flat(peer, synth.he_init(table, 2))])
    x = to_device(synth.images(rows, 1, 1, d, seed=100), torch.bfloat16, dev)
    y = torch.from_numpy(synth.labels(rows, vocab, seed=3)).to(dev)

    def step():
        r.step(x, y, 1.0, 0.1, 0.9, label_smoothing=0.1)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    loss = r.loss.cpu().numpy()
    r.overlap_peers = False           # the timer pass keeps every launch on one stream
    B.profile_reset()
    B.profile_enable(True)
    psteps = max(1, min(args.steps, 5))
    for _ in range(psteps):
        step()
    torch.cuda.synchronize()
    prof = B.profile_collect()
    B.profile_enable(False)
    lin = prof["linear"]
    hbm = {}
    for k in ("norm", "loss", "sgd"):
        if prof[k]["ms"] > 0:
            hbm[k] = {"GB/s": prof[k]["bytes"] / (prof[k]["ms"] * 1e-3) / 1e9}
            hbm[k]["frac"] = hbm[k]["GB/s"] / PEAK_HBM_GBS
    return {
        "metric": "codistill-step target tokens/sec on 1 MI355X (Transformer-base output block, 8192 tokens, vocab 32768)",
        "value": rows / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "transformer_head_codistill_step", "rows": rows, "d_model": d, "d_ff": 2048, "vocab": vocab,
                   "models": "2 x output block (local fwd+bwd+SGD, peer fwd)", "alpha": 1.0, "label_smoothing": 0.1,
                   "distillation": "mse_logits"},
        "loss": [float(v) for v in loss[:3]],
        "roofline": dict(roofline_of(lin["flops"], lin["bytes"], lin["ms"], lin["launches"],
                                     "igemm_kernel<0,128,128,2,2,true,0,1,false> (vocabulary projection, fp32 logits)",
                                     None), launches_per_step=lin["launches"] / psteps),
        "kernel_class_ms_per_step": {k: round(v["ms"] / psteps, 4) for k, v in prof.items()},
        "hbm_kernels": hbm,
        "cpu_baseline": None,
    }


def transformer(args, B, synth, StepRunner, pack_flat, torch, dev):
    """One codistillation step of the base encoder-decoder Transformer (two models: 6 + 6 layers, d_model 512,
    8 heads, d_ff 2048, shared vocabulary 32768, bf16): label smoothing 0.1, alpha 1, KL distillation term, Adam.
    Default batch: sentence pairs with source and target lengths uniform in [16, 128], drawn until they hold at
    least 8192 target tokens (109 pairs with this seed), handed to the library in packed form: the tokens of all
    sentences one after the other, each stream's rows rounded up to a multiple of 128 (the rows behind the last sentence
    hold negative ids and ignored labels).  --sentences padded: the same pairs, every sentence padded to 128 + 128 positions
    with negative ids (padding is masked as a key, embeds as zero, takes no gradient; its target rows carry
    ignore_index).  tokens/s counts the valid target tokens in both.  --sentences uniform: 64 pairs of full length
    128 + 128 (8192 target tokens, no padding).
    roofline: the kernel class that takes the most time of the step."""
    Ts, Tt, vocab = 128, 128, 32768
    arch = B.arch_preset(B.CD_ARCH_TRANSFORMER)
    big = args.transformer_size == "big"
    budget = 8192
    if big:   # the model Section 4 trains: d_model 1024, 16 heads, d_ff 4096; about the 3.8 k tokens per GPU of its recipe
        budget = 3840
        arch = B.arch_preset(B.CD_ARCH_TRANSFORMER, widths=[1024, 4096, 16])
    if args.sentences == "uniform":
        S = budget // Tt
        xh, yh = synth.tokens(S, Ts + Tt, vocab, seed=100), synth.labels(S * Tt, vocab, seed=3)
        valid, src_tokens = S * Tt, S * Ts
    else:
        xh, yh, sl, tl = synth.sentence_pairs(budget, 16, 128, vocab, seed=100)
        S, valid, src_tokens = xh.shape[0], int(tl.sum()), int(sl.sum())
    elements, target_rows = S, S * Tt
    if args.sentences == "ragged":   # packed: one batch element whose streams hold all sentences
        xh, yh, _, _ = synth.pack_sentences(xh, yh, Ts, multiple=128)
        target_rows = len(yh)
        kw = dict(in_h=xh.shape[1] - target_rows, in_w=target_rows, max_sentences=S, max_sentence_len=max(Ts, Tt))
        arch = B.arch_preset(B.CD_ARCH_TRANSFORMER, widths=[1024, 4096, 16], **kw) if big else B.arch_preset(B.CD_ARCH_TRANSFORMER, **kw)
        xh, elements = xh[None], 1
    model, peer = B.Model(arch, B.CD_BF16), B.Model(arch, B.CD_BF16)
    table = model.param_table()
    r = StepRunner(model, [peer], elements, dev)
    r.load(pack_flat(model, synth.he_init(table, 1)), [pack_flat(peer, synth.he_init(table, 2))])
    x = torch.from_numpy(xh).to(dev)
    y = torch.from_numpy(yh).to(dev)

    def step():
        # Adam with the constants of the translation recipe the paper follows (Section 4)
        r.step(x, y, 1.0, 5e-4, 0.0, label_smoothing=0.1, dist_kind=B.CD_DIST_KL, ignore_index=-1, adam=(0.9, 0.98, 1e-8))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    loss = r.loss.cpu().numpy()
    r.overlap_peers = False           # the timer pass keeps every launch on one stream
    B.profile_reset()
    B.profile_enable(True)
    psteps = max(1, min(args.steps, 5))
    for _ in range(psteps):
        step()
    torch.cuda.synchronize()
    prof = B.profile_collect()
    B.profile_enable(False)
    classes_ms = {k: round(v["ms"] / psteps, 4) for k, v in prof.items()}
    top = max(("conv_fprop", "conv_dgrad", "conv_wgrad", "attention", "linear", "loss", "norm"), key=lambda k: prof[k]["ms"])
    p = prof[top]
    roof = roofline_of(p["flops"], p["bytes"], p["ms"], p["launches"], "kernel class '%s' of the library's timer" % top, None)
    roof["launches_per_step"] = p["launches"] / psteps
    name = "big" if big else "base"
    return {
        "metric": "codistill-step target tokens/sec on 1 MI355X (Transformer-%s, %d sentence pairs, %d valid target tokens, "
                  "vocab 32768)" % (name, S, valid),
        "value": valid / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "transformer_%s_codistill_step%s" % (name, {"ragged": "", "padded": "_padded_sentences",
                                                                        "uniform": "_uniform_lengths"}[args.sentences]),
                   "sentences": S, "lengths": {"ragged": "uniform in [16, 128], packed (no padding rows)",
                                               "padded": "uniform in [16, 128], padded to 128 + 128",
                                               "uniform": "128 + 128"}[args.sentences],
                   "valid_target_tokens": valid, "valid_source_tokens": src_tokens, "target_rows": target_rows,
                   "d_model": arch.widths[0], "heads": arch.widths[2],
                   "d_ff": arch.widths[1], "layers": "6+6", "vocab": vocab,
                   "models": "2 x Transformer-%s (local fwd+bwd+Adam, peer fwd)" % name, "alpha": 1.0,
                   "label_smoothing": 0.1,
                   "distillation": "kl", "optimizer": "adam(0.9, 0.98, 1e-8), lr 5e-4"},
        "loss": [float(v) for v in loss[:3]],
        "roofline": roof,
        "kernel_class_ms_per_step": classes_ms,
        "cpu_baseline": None,
    }


def library_gemm_reference(torch, dev):
    """The vendor GEMM (torch.matmul in bf16) on the matrix shapes of ResNet-50's convolutions at batch 256: 1x1
    convolutions are plain [pixels x Cin] x [Cin x Cout] products, 3x3 convolutions are timed as the product an explicit
    im2col would feed it ([pixels x 9 Cin], the gather itself not included), weight gradients as the transposed product over
    the pixels.  A reference point for what the machine's tuned library reaches on these shapes; not part of the step."""
    fwd = [("s1.c3 64>256 1x1", 802816, 256, 64), ("s2.c3 128>512 1x1", 200704, 512, 128), ("s3.c3 256>1024 1x1", 50176, 1024, 256),
           ("s3.c1 1024>256 1x1", 50176, 256, 1024), ("s4.c3 512>2048 1x1", 12544, 2048, 512), ("s4.c1 2048>512 1x1", 12544, 512, 2048),
           ("s3.c2 3x3 256 as GEMM", 50176, 256, 2304), ("s4.c2 3x3 512 as GEMM", 12544, 512, 4608), ("8192^3", 8192, 8192, 8192)]
    wg = [("s1.c2 3x3 64", 802816, 64, 576), ("s1.c3 64>256", 802816, 256, 64), ("s2.c2 3x3 128", 200704, 128, 1152),
          ("s3.c2 3x3 256", 50176, 256, 2304), ("s3.c3 256>1024", 50176, 1024, 256), ("s4.c2 3x3 512", 12544, 512, 4608),
          ("s4.c3 512>2048", 12544, 2048, 512)]

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / 10 * 1e3

    rows = []
    for name, M, N, K in fwd:
        a = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
        w = torch.randn(N, K, device=dev, dtype=torch.bfloat16)
        us = timed(lambda: a @ w.t())
        rows.append({"product": "forward", "layer": name, "M": M, "N": N, "K": K, "us": us, "TFLOP/s": 2.0 * M * N * K / us / 1e6})
    for name, M, N, K in wg:
        dy = torch.randn(M, N, device=dev, dtype=torch.bfloat16)
        x = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
        us = timed(lambda: dy.t() @ x)
        rows.append({"product": "weight gradient", "layer": name, "M": M, "N": N, "K": K, "us": us,
                     "TFLOP/s": 2.0 * M * N * K / us / 1e6})
    return {"metric": "vendor-library bf16 GEMM time on ResNet-50 (batch 256) convolution shapes", "unit": "us", "n_gpus": 1,
            "data": "synthetic", "dtype": "bf16", "config": {"workload": "library_gemm_reference"}, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="resnet50",
                    choices=["resnet50", "transformer_head", "transformer", "library_gemm_reference"],
                    help="resnet50 (default): the headline metric.  transformer_head: the output block of the base "
                         "Transformer (feed-forward sublayer, residual, LayerNorm, vocabulary projection) on 8192 target "
                         "tokens, a separate JSON line with its own metric")
    ap.add_argument("--transformer-size", default="base", choices=["base", "big"],
                    help="--workload transformer: base (64 sentences) or big (d_model 1024, 16 heads, d_ff 4096; 30 sentences)")
    ap.add_argument("--sentences", default="ragged", choices=["ragged", "padded", "uniform"],
                    help="--workload transformer: ragged (default) = lengths uniform in [16, 128] until the batch holds 8192 "
                         "target tokens, given in packed form (no padding rows); padded = the same sentences padded to "
                         "128 + 128; uniform = 64 pairs of 128 + 128 tokens")
    ap.add_argument("--peer", default="resnet50", choices=["resnet50", "resnet18", "resnext101"],
                    help="architecture of the stale peer of the ResNet-50 workload (Section 5 pairs different "
                         "architectures); the default line is the two-ResNet-50 step")
    ap.add_argument("--exchange", default="checkpoints", choices=["checkpoints", "predictions"],
                    help="checkpoints (default): the step computes the stale peers' forward passes itself; predictions: "
                         "the peers' logits arrive from outside (Section 3's second implementation), no peer forward")
    ap.add_argument("--n-way", type=int, default=2,
                    help="models that codistill (Section 5: 2, 3, 4, 8): the step runs n-1 peer forwards; default 2")
    ap.add_argument("--local", default="resnet50", choices=["resnet50", "resnext101"],
                    help="architecture of the local model of that workload (default: ResNet-50, the benchmarked step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain 1 GiB -> 1 GiB elementwise copy three times (the known-size "
                         "kernel that hardware-counter byte counts are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU's share of the step: this build has no multi-GPU path, "
                 "run it with --gpus 1")

    import numpy as np
    import torch
    from paper_2010_02838_amd import binding as B
    from paper_2010_02838_amd import synth
    from paper_2010_02838_amd.runner import StepRunner, pack_flat, to_device

    dev = "cuda:0"
    if args.workload == "library_gemm_reference":
        print(json.dumps(library_gemm_reference(torch, dev)))
        return
    if args.workload == "transformer_head":
        print(json.dumps(transformer_head(args, B, synth, StepRunner, pack_flat, to_device, torch, dev)))
        return
    if args.workload == "transformer":
        print(json.dumps(transformer(args, B, synth, StepRunner, pack_flat, torch, dev)))
        return
    if args.copy_calibration:
        a = torch.ones(1 << 28, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.mul(a, 1.0, out=b)      # one elementwise kernel: reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    loss_cfg5 = loss_kernel_cfg5(B, torch, dev)
    batch, res, classes = args.batch, 224, 1000
    kinds = {"resnet50": B.CD_ARCH_RESNET_BOTTLENECK, "resnet18": B.CD_ARCH_RESNET_BASIC_IMAGENET,
             "resnext101": B.CD_ARCH_RESNEXT}
    if not 2 <= args.n_way <= 9:
        raise SystemExit("--n-way: 2 to 9 models (the loss takes up to 8 peers)")
    default_pair = args.peer == "resnet50" and args.local == "resnet50" and args.n_way == 2 and args.exchange == "checkpoints"
    model, peer = B.Model(B.arch_preset(kinds[args.local]), B.CD_BF16), B.Model(B.arch_preset(kinds[args.peer]), B.CD_BF16)
    table = model.param_table()
    npeers = args.n_way - 1
    r = StepRunner(model, [peer] * npeers, batch, dev)
    r.load(pack_flat(model, synth.he_init(table, 1)),
           [pack_flat(peer, synth.he_init(peer.param_table(), 2 + j)) for j in range(npeers)])
    x = torch.empty(batch, res, res, 3, dtype=torch.bfloat16, device=dev)
    for b0 in range(0, batch, 32):       # images ~ N(0,1), generated on the host in slices
        n = min(32, batch - b0)
        x[b0:b0 + n] = to_device(synth.images(n, res, res, 3, seed=100 + b0), torch.bfloat16, dev)
    y = torch.from_numpy(synth.labels(batch, classes, seed=3)).to(dev)
    alpha, lr, mu = 1.0, 0.1, 0.9

    received = [torch.randn(batch, classes, device=dev) * 3.0 for _ in range(npeers)]   # predictions mode: what peers sent

    def step():
        if args.exchange == "predictions":
            r.forward_local(x)
            r.finish(x, y, received, alpha, lr, mu)
        else:
            r.step(x, y, alpha, lr, mu)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries on the caller's stream
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        step()
    marks[-1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_median = per_step[len(per_step) // 2]
    loss = r.loss.cpu().numpy()

    # second pass: per-launch HIP events on the launch stream, per kernel class; the peer forward runs
    # after the local one here (on one stream), so that a launch's duration is its own
    r.overlap_peers = False
    B.profile_reset()
    B.profile_enable(True)
    psteps = max(1, min(args.steps, 5))
    for _ in range(psteps):
        step()
    torch.cuda.synchronize()
    prof = B.profile_collect()
    B.profile_enable(False)
    bn = prof["bn_apply"]
    ev_us = B.profile_event_overhead()
    roofline = roofline_of(bn["flops"], bn["bytes"], bn["ms"], bn["launches"],
                           "bn_apply_k<bf16,8,true> (BatchNorm forward: normalise, add the residual, ReLU, bit mask)",
                           ROOFLINE_TRAFFIC_BYTES if default_pair else None, ev_us)
    roofline["launches_per_step"] = bn["launches"] / psteps
    cw = prof["conv_fprop_wide"]
    roofline_conv = roofline_of(cw["flops"], cw["bytes"], cw["ms"], cw["launches"],
                                "igemm_kernel<0,128,256,2,2,false,1,1,false,0,false> (bf16 implicit-GEMM conv fprop on "
                                "128x256 tiles, BatchNorm column sums in the epilogue)", ROOFLINE_CONV_TRAFFIC_BYTES if default_pair else None,
                                ev_us)
    roofline_conv["launches_per_step"] = cw["launches"] / psteps
    roofline_conv["mfma_busy_frac_counters"] = ROOFLINE_CONV_MFMA_BUSY if default_pair else None
    roofline_conv["mfma_counter_source"] = MFMA_COUNTER_SOURCE if default_pair else None
    classes_ms = {k: round(v["ms"] / psteps, 4) for k, v in prof.items()}
    hbm = {}
    for k in ("bn_apply", "norm", "loss", "sgd"):
        if prof[k]["ms"] > 0:
            hbm[k] = {"GB/s": prof[k]["bytes"] / (prof[k]["ms"] * 1e-3) / 1e9}
            hbm[k]["frac"] = hbm[k]["GB/s"] / PEAK_HBM_GBS

    out = {
        "metric": "codistill-step samples/sec on 1 MI355X (%s, 224^2, bs%d)" % ("ResNet-50" if args.local == "resnet50" else args.local, batch),
        "value": batch / (ms_per_step * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_median": ms_median,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "resnet50_codistill_step", "batch": batch, "resolution": res, "classes": classes,
                   "models": "2 x ResNet-50 (local fwd+bwd+SGD, peer fwd)" if default_pair else
                             ("%s (local fwd+bwd+SGD) + %d x %s (peer fwd)" % (args.local, npeers, args.peer)
                              if args.exchange == "checkpoints" else
                              "%s (local fwd+bwd+SGD), logits of %d peer(s) received" % (args.local, npeers)), "alpha": alpha,
                   "distillation": "mse_logits", "lr": lr, "momentum": mu},
        "loss": [float(v) for v in loss[:3]],
        "roofline": roofline,
        "roofline_conv": roofline_conv,
        "kernel_class_ms_per_step": classes_ms,
        "hbm_kernels": hbm,
        "loss_kernel_8192x32768": loss_cfg5,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
