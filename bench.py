#!/usr/bin/env python3
"""Benchmark: one worker's AlexNet-shaped SGD iteration (forward + backward + per-layer
gradient aggregation over K peers + model update, overlapped on three streams) on one MI355X.

Prints ONE JSON line.  `value` is images/s of whole iterations with every input resident in
HBM, timed without any instrumentation (two HIP events around every launch cost the three-stream
step 0.35-0.45 ms, 4 %).  Right after the timed region the same iterations run again with those
events: once with the three-stream schedule (`*_three_stream_pass`: up to three kernels share the
GPU, a launch's duration is its share) and a few times with the one-stream schedule, where every
kernel has the GPU to itself: `roofline` describes the matrix-core kernel that takes the most time
inside the step and `update_roofline` the fused gradient-sum + update kernel, from that pass.
`grad_update` is the stand-alone update over the eight AlexNet buckets; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
# context only (other hardware, full AlexNet on ImageNet, paper Table 1): seconds per iteration, B=256
PAPER_ALEXNET_S_PER_ITER = {"P100": 0.1, "K80": 0.9, "KNL": 0.6, "CPU": 2.0}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


_STREAMS = []


def build_net(cg, torch, B, K, seed, n_batches=32, workload="alexnet"):
    import cg_synth
    layers, in_shape = {"alexnet": cg_synth.alexnet_layers, "inception": cg_synth.inception_layers,
                        "googlenet": lambda: cg_synth.googlenet_layers()[:2]}[workload]()
    gen = torch.Generator(device="cuda").manual_seed(seed)
    net = cg.Net(layers, B, in_shape)
    # a pool of resident batches, one per step of the run where memory allows: random images with
    # random labels can only be memorised, and a net that has memorised a small pool then diverges
    # under this learning rate, which says nothing about speed but ends in NaNs
    xs = [torch.randn((B,) + tuple(in_shape), device="cuda", generator=gen) for _ in range(n_batches)]
    ls = [torch.randint(0, 1000, (B,), device="cuda", generator=gen, dtype=torch.int32) for _ in range(n_batches)]
    st = dict(net=net, layers=layers, xs=xs, ls=ls, it=0, w={}, v={}, g={}, peers={}, masks={})
    shapes = cg_synth.infer_shapes(layers, in_shape)
    for li, wshape, nb in cg_synth.param_layers(layers, in_shape):
        n = cg.cg_net_param_count(net, li)
        fan_in = 1
        for s in wshape[1:]:
            fan_in *= s
        w = torch.zeros(n, device="cuda")
        w[:n - nb].normal_(0.0, fan_in ** -0.5, generator=gen)
        st["w"][li] = w
        st["v"][li] = torch.zeros(n, device="cuda")
        st["g"][li] = torch.zeros(n, device="cuda")
        st["peers"][li] = [torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=gen) for _ in range(K)]
        cg.cg_net_bind(net, li, w, st["v"][li], st["g"][li], st["peers"][li])
    for i, ly in enumerate(layers):
        if ly["kind"] == "dropout":
            C, H, W = shapes[i]
            st["masks"][i] = (torch.rand((B, C * H * W), device="cuda", generator=gen) >= ly["p"]).to(torch.uint8)
    st["ws"] = torch.empty(cg.cg_net_workspace_bytes(net), dtype=torch.uint8, device="cuda")
    st["loss"] = torch.zeros(4, device="cuda")
    # every workload of a run uses the same two streams: a process gets few hardware queues, and
    # streams made later may share one with each other
    if not _STREAMS:
        _STREAMS.extend([torch.cuda.Stream(), torch.cuda.Stream()])
    st["s0"], st["s1"] = _STREAMS
    return st


def run_steps(cg, torch, st, sgd, n, flags=0):
    for _ in range(n):
        i = st["it"] % len(st["xs"])
        st["it"] += 1
        cg.cg_train_step(st["net"], st["xs"][i], st["ls"][i], st["masks"], sgd, st["ws"], st["s0"], st["s1"],
                         st["loss"], flags)


def sync(torch, st):
    st["s0"].synchronize()
    st["s1"].synchronize()
    torch.cuda.synchronize()


def collect_profile(cg):
    agg = {}
    for i in range(cg.cg_profile_count()):
        r = cg.cg_profile_get(i)
        a = agg.setdefault(r["kernel"], dict(ms=0.0, launches=0, flops=0.0, bytes=0.0, passes={}))
        a["ms"] += r["ms"]; a["launches"] += 1; a["flops"] += r["flops"]; a["bytes"] += r["bytes"]
        key = f'{r["pass_"]}@{r["layer"]}'
        p = a["passes"].setdefault(key, dict(ms=0.0, launches=0, flops=0.0, bytes=0.0))
        p["ms"] += r["ms"]; p["launches"] += 1; p["flops"] += r["flops"]; p["bytes"] += r["bytes"]
    return agg


def hbm_achievable(cg, torch, reps=20):
    """What the memory system reaches with the simplest streaming kernels (one float4 per thread, all
    accesses non-temporal) on arrays of the eight buckets' total size: the measured ceilings to read
    the update kernel's fraction of the published 8 TB/s against."""
    n = 60965224 // 4 * 4
    bufs = [torch.zeros(n, device="cuda") for _ in range(6)]
    out = {}
    for name, mode, nbytes in (("read", 1, 4 * n), ("fill", 2, 4 * n), ("copy", 0, 8 * n), ("triad", 3, 12 * n)):
        def one(i):
            a, b, c = bufs[(3 * i) % 6], bufs[(3 * i + 1) % 6], bufs[(3 * i + 2) % 6]
            cg.cg_debug_stream(a, b, c, 4 * n, mode)
        for i in range(3):
            one(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            one(i)
        e1.record()
        torch.cuda.synchronize()
        out[name + "_gbps"] = round(nbytes / (e0.elapsed_time(e1) / reps) / 1e6, 1)
    out["what"] = ("244 MB arrays, one float4 per thread, non-temporal loads and stores, launches back to back between "
                   "two events; bytes counted once per array read or written")
    return out


def mfma_achievable(cg, torch, blocks=512, iters=20000, reps=5):
    """What the fp32 matrix pipeline reaches with nothing else to do (cg_debug_mfma_loop: two blocks of
    four waves per compute unit, four independent accumulators a wave, no loads, no LDS): the measured
    ceiling beside the published 157.3 TFLOP/s."""
    out = torch.empty(256 * blocks, device="cuda")
    cg.cg_debug_mfma_loop(out, blocks, iters)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        cg.cg_debug_mfma_loop(out, blocks, iters)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    tf = 2.0 * 32 * 32 * 2 * 16 * iters * blocks / ms / 1e9
    return {"tflops": round(tf, 1), "frac_of_peak": round(tf / PEAK_FP32_MFMA_TFLOPS, 4), "ms_per_launch": round(ms, 4),
            "what": f"{blocks} blocks x 4 waves x {iters} x 4 independent v_mfma_f32_32x32x2_f32, no memory traffic"}


def gpu_clocks():
    """Clock levels as the box reports them right after the timed work (rocm-smi; None if it is not there)."""
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20).stdout
        card = next(iter(json.loads(out).values()))
        return {k.strip(":"): v for k, v in card.items() if "clock speed" in k and ("sclk" in k or "mclk" in k or "fclk" in k)}
    except Exception:
        return None


def conv_layers_standalone(cg, torch, B, reps=10, math=0):
    """Configuration 2: every AlexNet-shaped convolution layer alone, forward / backward-data /
    backward-weight through the C ABI (the first layer's backward-data included, which a net skips),
    TFLOP/s of useful work 2*M*N*K*groups over the mean of `reps` back-to-back calls."""
    import cg_synth
    gen = torch.Generator(device="cuda").manual_seed(2)
    out = {}
    for name, c in cg_synth.ALEXNET_CONVS.items():
        d = cg.conv_desc(B, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
        OH, OW = cg.cg_conv_out_shape(d)
        Cg = c["C"] // c["groups"]
        fan = Cg * c["k"] ** 2
        x = torch.randn((B, c["C"], c["H"], c["H"]), device="cuda", generator=gen) * fan ** -0.5
        w = torch.randn((c["M"], Cg, c["k"], c["k"]), device="cuda", generator=gen) * fan ** -0.5
        b = torch.randn(c["M"], device="cuda", generator=gen) * 0.1
        dy = torch.randn((B, c["M"], OH, OW), device="cuda", generator=gen) * fan ** -0.5
        y, dx, dw, db = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w), torch.empty_like(b)
        ws = [torch.empty(max(cg.cg_conv_workspace_bytes(d, p), 16), dtype=torch.uint8, device="cuda") for p in range(3)]
        flop = 2.0 * c["M"] * Cg * c["k"] ** 2 * B * OH * OW
        calls = {"fwd": lambda: cg.cg_conv_fwd_math(d, x, w, b, y, ws[0], math),
                 "bwd_data": lambda: cg.cg_conv_bwd_data_math(d, dy, w, dx, ws[1], math),
                 "bwd_weight": lambda: cg.cg_conv_bwd_weight_math(d, x, dy, dw, db, ws[2], math)}
        # the least a pass must move through HBM: its two operand tensors read once, its result written once
        nbytes = {"fwd": 4.0 * (x.numel() + w.numel() + dy.numel()), "bwd_data": 4.0 * (x.numel() + w.numel() + dy.numel()),
                  "bwd_weight": 4.0 * (x.numel() + w.numel() + dy.numel())}
        res = {}
        for ps, fn in calls.items():
            fn(); fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            res[ps] = {"ms": round(ms, 4), "tflops": round(flop / ms / 1e9, 1),
                       "hbm_floor_ms": round(nbytes[ps] / PEAK_HBM_GBS / 1e6, 4)}
        out[name] = res
    out["what"] = (f"B={B}, each pass alone on the GPU through cg_conv_fwd / cg_conv_bwd_data / cg_conv_bwd_weight (filter "
                   "permutation, K-slice sums and bias gradient included in the time), useful FLOP = 2*M*N*K*groups")
    return out


def reduced_precision(cg, torch, B, K, sgd, steps=30):
    """The optional bf16 matrix-core modes, chosen explicitly (CG_STEP_BF16: operands rounded to bf16,
    parity bound 2e-2; CG_STEP_BF16X3: operands split into two bf16 numbers, three products, inside the
    fp32 parity bound): the same AlexNet-shaped step and the same stand-alone layers.  Separate lines:
    the headline stays fp32.  Rooflines: the dense bf16 matrix peak (a third of it per useful product
    in the three-product mode), or the HBM floor of the pass where that is the longer time."""
    out = {}
    for tag, flag, math, peak in (("bf16", cg.CG_STEP_BF16, cg.CG_MATH_BF16, PEAK_BF16_MFMA_TFLOPS),
                                  ("bf16x3", cg.CG_STEP_BF16X3, cg.CG_MATH_BF16X3, PEAK_BF16_MFMA_TFLOPS / 3)):
        st = build_net(cg, torch, B, K, seed=4, n_batches=min(32, steps + 5))
        torch.cuda.synchronize()
        run_steps(cg, torch, st, sgd, 5, flag)
        sync(torch, st)
        t0 = time.perf_counter()
        run_steps(cg, torch, st, sgd, steps, flag)
        sync(torch, st)
        ms = (time.perf_counter() - t0) / steps * 1e3
        loss = float(st["loss"].cpu()[0])
        del st
        torch.cuda.empty_cache()
        layers = conv_layers_standalone(cg, torch, B, math=math)
        best = None
        for name, v in layers.items():
            if name == "what":
                continue
            for ps, r in v.items():
                flop = r["tflops"] * r["ms"] * 1e9
                mfma_ms = flop / peak / 1e9
                r["bound"] = "hbm" if r["hbm_floor_ms"] > mfma_ms else "mfma"
                r["frac"] = round(max(mfma_ms, r["hbm_floor_ms"]) / r["ms"], 3)
                if best is None or r["tflops"] > best[1]["tflops"]:
                    best = (f"{name}.{ps}", r)
        out[tag] = {"workload": f"alexnet_shaped_train_step_B{B}_K{K}", "dtype": tag, "ms_per_step": ms,
                    "images_per_s": B / (ms * 1e-3), "steps": steps, "loss": loss,
                    "matrix_peak_tflops": round(peak, 1), "conv_layers_standalone": layers,
                    "fastest_pass": {"pass": best[0], **best[1]}}
    return out


def grad_update_standalone(cg, torch, steps, warmup, per_bucket=True):
    """Configuration 3: the eight AlexNet parameter buckets, K in {4, 8, 16}; GB/s of
    algorithmic traffic (4K+20 bytes per parameter) over the kernels' own durations."""
    import cg_synth
    out = {}
    gen = torch.Generator(device="cuda").manual_seed(3)
    sizes = list(cg_synth.ALEXNET_BUCKETS.values())
    sgd = cg.cg_sgd(0.01, 0.9, 5e-4, 1.0)
    bufs = []
    for n in sizes:
        w = torch.empty(n, device="cuda").normal_(0, 1e-2, generator=gen)
        bufs.append(dict(n=n, w=w, v=torch.zeros(n, device="cuda"),
                         g=[torch.empty(n, device="cuda").normal_(0, 1e-3, generator=gen) for _ in range(17)]))
    for K, fn, tag in [(4, cg.cg_grad_reduce_sgd_multi, ""), (8, cg.cg_grad_reduce_sgd_multi, ""),
                       (16, cg.cg_grad_reduce_sgd_multi, ""), (4, cg.cg_grad_reduce_sgd_tree_multi, "_tree"),
                       (16, cg.cg_grad_reduce_sgd_tree_multi, "_tree")]:
        # one launch for the eight buckets (the five convolution buckets are launch-bound one by one);
        # "_tree": the sum in binomial-tree association (section 3.2), same traffic
        def one():
            fn([b["w"] for b in bufs], [b["v"] for b in bufs], [b["g"][0] for b in bufs],
               [b["g"][1:K + 1] for b in bufs], [b["n"] for b in bufs], sgd)
        for _ in range(warmup):
            one()
        torch.cuda.synchronize()
        # `steps` launches back to back between two events on the launch stream: the per-launch time
        # includes the gaps between launches but not the event markers' own latency, which at a few
        # hundred microseconds per launch would otherwise cost several percent.  Five such rounds, the
        # median reported and all five listed: early in a process a round now and then runs at half speed
        # (seen on any K, never in a sustained run of seconds), which says nothing about the kernel.
        rounds = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                one()
            e1.record()
            torch.cuda.synchronize()
            rounds.append(e0.elapsed_time(e1) / steps)
        ms = sorted(rounds)[len(rounds) // 2]
        by = (4.0 * K + 20.0) * sum(sizes)
        if K == 4 and not tag and per_bucket:
            # bucket by bucket, one launch each: the five convolution buckets are bound by the launch
            per = {}
            for name, b in zip(cg_synth.ALEXNET_BUCKETS, bufs):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                cg.cg_grad_reduce_sgd(b["w"], b["v"], b["g"][0], b["g"][1:K + 1], b["n"], sgd)
                e0.record()
                for _ in range(steps):
                    cg.cg_grad_reduce_sgd(b["w"], b["v"], b["g"][0], b["g"][1:K + 1], b["n"], sgd)
                e1.record()
                torch.cuda.synchronize()
                per[name] = round((4.0 * K + 20.0) * b["n"] / (e0.elapsed_time(e1) / steps) / 1e6, 1)
            out["per_bucket_gbps_K4"] = per
        out[f"K{K}{tag}"] = dict(gbps=by / ms / 1e6, ms_per_launch=ms, bytes=by, frac_of_peak=by / ms / 1e6 / PEAK_HBM_GBS,
                            launches_per_update=1, buckets=len(sizes), launches_per_round=steps,
                            rounds_ms=[round(r, 4) for r in rounds])
    return out


def googlenet_workload(cg, torch, sgd, steps, flags, table=False):
    """The paper's second benchmark net by shape (Table 1: GoogLeNet, batch 32 per worker): stem, nine
    inception modules, 7.0 M parameters in 58 layer buckets, K = 8 peers.  Context beside the headline
    workload: 142 layers, most of them small, so the step is bound by launches as much as by arithmetic."""
    gst = build_net(cg, torch, 32, 8, seed=6, n_batches=8, workload="googlenet")
    torch.cuda.synchronize()
    run_steps(cg, torch, gst, sgd, 5, flags)
    sync(torch, gst)
    l0 = cg.cg_debug_launch_count()
    t0 = time.perf_counter()
    run_steps(cg, torch, gst, sgd, steps, flags)
    sync(torch, gst)
    gms = (time.perf_counter() - t0) / steps * 1e3
    launches = (cg.cg_debug_launch_count() - l0) / steps
    gflop = 3 * 2 * 1.5827 * 32 - 2 * 0.118 * 32       # forward x 3, minus the first layer's backward-data
    out = {"workload": "googlenet_shaped_train_step_224_B32_K8", "ms_per_step": gms,
           "images_per_s": 32 / (gms * 1e-3), "steps": steps, "matrix_core_tflops": gflop / gms,
           "kernel_launches_per_step": launches,
           "schedule": "serial" if flags == cg.CG_STEP_SERIAL else "overlap", "loss": float(gst["loss"][0].item())}
    if table:
        cg.cg_profile_enable(True)
        run_steps(cg, torch, gst, sgd, 3, cg.CG_STEP_SERIAL)
        sync(torch, gst)
        cg.cg_profile_enable(False)
        kernel_table(collect_profile(cg), 3)
    del gst
    torch.cuda.empty_cache()
    return out


def cpu_baseline(sample_B, K):
    """The oracle's whole iteration on `sample_B` images of the same net (one step incl. update)."""
    import cg_synth
    from oracle import net as onet
    from oracle.cgo import Oracle
    orc = Oracle("float")
    layers, in_shape = cg_synth.alexnet_layers()
    t = cg_synth.net_tensors(layers, in_shape, sample_B, K, seed=4, num_classes=1000)
    hist = {k: v * 0 for k, v in t["buckets"].items()}
    t0 = time.perf_counter()
    onet.train_step(orc, layers, t["x"], t["labels"], t["buckets"], hist, t["peers"], t["masks"], 0.01, 0.9, 5e-4)
    dt = time.perf_counter() - t0
    return dict(value=sample_B / dt, unit="images/s", cores=orc.num_threads(), kind="oracle",
                sample=f"same AlexNet-shaped net and K={K}, one whole iteration at B={sample_B} ({dt:.1f} s of CPU time)")


def load_traffic():
    """Per-launch HBM traffic by kernel label, from the committed counter summary (profiles/)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)["kernels"]
    except (OSError, ValueError, KeyError):
        return {}


def kernel_rooflines(agg, steps, traffic):
    """(dominant matrix-core kernel's roofline, update kernel's roofline, totals) from per-launch records."""
    mm = {k: a for k, a in agg.items() if k.startswith("igemm")}
    dom_name, dom = max(mm.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["flops"] / dom["ms"] / 1e9       # TFLOP/s over that kernel's own launches
    t = traffic.get(dom_name)
    roofline = dict(bound="mfma", achieved=achieved, peak=PEAK_FP32_MFMA_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_FP32_MFMA_TFLOPS,
                    traffic=(t["fetch_bytes"] + t["write_bytes"]) if t else None, kernel=dom_name,
                    avg_launch_ms=dom["ms"] / dom["launches"], launches_per_step=dom["launches"] / steps,
                    flops_per_launch=dom["flops"] / dom["launches"])
    all_flops = sum(a["flops"] for a in mm.values())
    all_ms = sum(a["ms"] for a in mm.values())
    upd = {k: a for k, a in agg.items() if k.startswith("reduce_sgd")}
    upd_bytes = sum(a["bytes"] for a in upd.values())
    upd_ms = sum(a["ms"] for a in upd.values())
    upd_name = max(upd.items(), key=lambda kv: kv[1]["ms"])[0]
    t = traffic.get(upd_name)
    n_upd = sum(a["launches"] for a in upd.values())
    update = dict(bound="hbm", achieved=upd_bytes / upd_ms / 1e6, peak=PEAK_HBM_GBS, unit="GB/s",
                  frac=upd_bytes / upd_ms / 1e6 / PEAK_HBM_GBS,
                  traffic=(t["fetch_bytes"] + t["write_bytes"]) if t else None, kernel=upd_name,
                  bytes_per_launch=upd_bytes / n_upd, avg_launch_ms=upd_ms / n_upd, launches_per_step=n_upd / steps)
    totals = dict(tflops=all_flops / all_ms / 1e9, ms_per_step=all_ms / steps,
                  frac=all_flops / all_ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, flops_per_step=all_flops / steps)
    return roofline, update, totals


def per_layer_tflops(agg, layers):
    """TFLOP/s of every convolution / FC layer's three passes (algorithmic FLOP of the pass's matrix-core
    launches over their summed durations), keyed by layer name."""
    names, nconv, nfc = {}, 0, 0
    for i, ly in enumerate(layers):
        if ly["kind"] == "conv":
            nconv += 1; names[i] = f"conv{nconv}"
        elif ly["kind"] == "fc":
            nfc += 1; names[i] = f"fc{nfc + 5}"
    acc = {}
    for a in agg.values():
        for key, p in a["passes"].items():
            ps, li = key.split("@")
            if int(li) not in names or not p["flops"]:
                continue
            e = acc.setdefault(names[int(li)], {}).setdefault(ps.split("_", 1)[1], [0.0, 0.0])
            e[0] += p["flops"]; e[1] += p["ms"]
    return {n: {ps: round(f / ms / 1e9, 1) for ps, (f, ms) in v.items()} for n, v in sorted(acc.items())}


def kernel_table(agg, steps):
    log(f"{'kernel':34s} {'pass@layer':24s} {'launch/step':>11s} {'avg ms':>9s} {'TFLOP/s':>9s} {'GB/s':>9s}")
    for k, a in sorted(agg.items(), key=lambda kv: -kv[1]["ms"]):
        for pk, p in sorted(a["passes"].items(), key=lambda kv: -kv[1]["ms"]):
            log(f"{k:34s} {pk:24s} {p['launches'] / steps:11.1f} {p['ms'] / p['launches']:9.4f} "
                f"{p['flops'] / p['ms'] / 1e9:9.1f} {p['bytes'] / p['ms'] / 1e6:9.1f}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--peers", type=int, default=4)
    ap.add_argument("--cpu-sample", type=int, default=256, help="images in the CPU-oracle sample (0 = skip)")
    ap.add_argument("--skip-layer-bench", action="store_true", help="leave out the stand-alone per-layer and B=64 figures")
    ap.add_argument("--serial", action="store_true", help="one-stream schedule (no overlap) in the timed region")
    ap.add_argument("--kernel-table", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--skip-update-bench", action="store_true", help="leave out the stand-alone update benchmark")
    ap.add_argument("--update-only", action="store_true", help="only the stand-alone update benchmark (for counter runs)")
    ap.add_argument("--googlenet-only", action="store_true", help="only the GoogLeNet-shaped workload (for profiles)")
    ap.add_argument("--googlenet-steps", type=int, default=20,
                    help="steps of the GoogLeNet-shaped workload timed after the main one (0 = skip)")
    ap.add_argument("--inception-steps", type=int, default=30,
                    help="steps of the inception-shaped workload timed after the main one (0 = skip)")
    ap.add_argument("--exclusive-steps", type=int, default=5,
                    help="steps of the extra one-stream pass that times every kernel alone on the GPU (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures ONE worker on ONE GPU; the peers' gradients are resident buffers. "
            "--gpus must be 1.")
        sys.exit(2)

    import torch
    import paper_1706_00095_amd as cg
    cg.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B, K = args.batch, args.peers
    sgd = cg.cg_sgd(0.01, 0.9, 5e-4, 1.0)
    traffic = load_traffic()
    # one plain copy of 256 MiB before anything is timed: under a counter-collecting profiler its
    # dispatch is the known traffic the other kernels' FETCH_SIZE / WRITE_SIZE readings are scaled by
    cal = torch.zeros(2, 64 << 20, device="cuda")
    cg.cg_debug_copy(cal[0], cal[1], cal[0].numel() * 4)
    torch.cuda.synchronize()
    del cal
    if args.update_only:
        # the eight-bucket launches only, so that a profiler's per-kernel means are means over one launch shape
        print(json.dumps({"grad_update": grad_update_standalone(cg, torch, max(args.steps, 1), args.warmup, per_bucket=False),
                          "hbm_achievable": hbm_achievable(cg, torch), "mfma_achievable": mfma_achievable(cg, torch)}), flush=True)
        return

    flags = cg.CG_STEP_SERIAL if args.serial else cg.CG_STEP_OVERLAP
    if args.googlenet_only:
        print(json.dumps({"googlenet_step": googlenet_workload(cg, torch, sgd, max(args.googlenet_steps, 1), flags,
                                                               args.kernel_table)}), flush=True)
        return
    extra = args.exclusive_steps if not args.serial else 0
    inst_steps = max(1, min(args.steps, 20))          # iterations of the instrumented pass of the timed schedule
    st = build_net(cg, torch, B, K, seed=4, n_batches=max(1, min(64, args.warmup + args.steps + inst_steps + extra)))
    torch.cuda.synchronize()
    run_steps(cg, torch, st, sgd, args.warmup, flags)
    sync(torch, st)

    # ---- the timed region: K whole iterations, nothing but the library's own launches on the streams
    launches0 = cg.cg_debug_launch_count()
    t0 = time.perf_counter()
    run_steps(cg, torch, st, sgd, args.steps, flags)
    sync(torch, st)
    wall = time.perf_counter() - t0
    launches_per_step = (cg.cg_debug_launch_count() - launches0) / args.steps
    clocks = gpu_clocks()
    loss = float(st["loss"].cpu()[0])
    ms_per_step = wall / args.steps * 1e3
    # ---- the same schedule again, every matrix-core and update launch bracketed by two events
    cg.cg_profile_enable(True)
    t0 = time.perf_counter()
    run_steps(cg, torch, st, sgd, inst_steps, flags)
    sync(torch, st)
    inst_ms = (time.perf_counter() - t0) / inst_steps * 1e3
    cg.cg_profile_enable(False)
    agg = collect_profile(cg)
    roofline, update_roofline, totals = kernel_rooflines(agg, inst_steps, traffic)
    roofline["measured"] = update_roofline["measured"] = (
        f"HIP events around every launch of {inst_steps} iterations run right after the timed region with its schedule" +
        ("" if args.serial else ", in which backward-data, backward-weight and the update run on three streams: "
         "a launch's duration is its share of a GPU it does not have to itself"))
    if args.kernel_table:
        kernel_table(agg, inst_steps)
        log(f"matrix-core kernels: {totals['ms_per_step']:.3f} ms/step of launch time, {totals['tflops']:.1f} TFLOP/s over it; "
            f"wall {ms_per_step:.3f} ms/step ({inst_ms:.3f} with launch events); loss {loss:.4f}")

    # ---- the same kernels alone on the GPU: a few iterations of the one-stream schedule
    roofline_excl = update_excl = totals_excl = None
    serial_ms = None
    if extra > 0:
        run_steps(cg, torch, st, sgd, 2, cg.CG_STEP_SERIAL)
        sync(torch, st)
        t0 = time.perf_counter()
        run_steps(cg, torch, st, sgd, extra, cg.CG_STEP_SERIAL)
        sync(torch, st)
        serial_ms = (time.perf_counter() - t0) / extra * 1e3          # plain, like the timed region
        cg.cg_profile_enable(True)
        run_steps(cg, torch, st, sgd, extra, cg.CG_STEP_SERIAL)
        sync(torch, st)
        cg.cg_profile_enable(False)
        agg1 = collect_profile(cg)
        roofline_excl, update_excl, totals_excl = kernel_rooflines(agg1, extra, traffic)
        totals_excl["per_layer_tflops"] = per_layer_tflops(agg1, st["layers"])
        roofline_excl["measured"] = update_excl["measured"] = (
            f"HIP events around every launch of {extra} further iterations run right after the timed region with "
            "the one-stream schedule (CG_STEP_SERIAL: same kernels, same order, one at a time)")
        # the timed region's figures for that same kernel
        if roofline_excl["kernel"] in agg:
            a = agg[roofline_excl["kernel"]]
            roofline = dict(roofline, kernel=roofline_excl["kernel"], achieved=a["flops"] / a["ms"] / 1e9,
                            frac=a["flops"] / a["ms"] / 1e9 / PEAK_FP32_MFMA_TFLOPS,
                            avg_launch_ms=a["ms"] / a["launches"], launches_per_step=a["launches"] / inst_steps,
                            flops_per_launch=a["flops"] / a["launches"], traffic=roofline_excl["traffic"])
        if args.kernel_table:
            log("-- one-stream pass --")
            kernel_table(agg1, extra)
            log(f"matrix-core kernels alone: {totals_excl['ms_per_step']:.3f} ms/step, {totals_excl['tflops']:.1f} TFLOP/s; "
                f"wall without events {serial_ms:.3f} ms/step")

    # free the net before the stand-alone update benchmark
    del st
    torch.cuda.empty_cache()
    grad_update = None if args.skip_update_bench else grad_update_standalone(cg, torch, min(max(args.steps, 5), 50), args.warmup)
    achievable = None if args.skip_update_bench else hbm_achievable(cg, torch)
    mfma_peak = None if args.skip_update_bench else mfma_achievable(cg, torch)
    if grad_update:
        for k, v in grad_update.items():
            if "bytes" not in v:
                continue        # the per-bucket table
            t = traffic.get(f"standalone_update_{k}")
            v["traffic"] = (t["fetch_bytes"] + t["write_bytes"]) if t else None

    # ---- the second workload shape of the paper (GoogLeNet-like modules), outside the timed region:
    # two inception modules on 192 x 28 x 28, B = 32, K = 8 peers; many small layers, launch-bound
    inception = None
    if args.inception_steps > 0 and not args.serial:
        ist = build_net(cg, torch, 32, 8, seed=5, n_batches=8, workload="inception")
        torch.cuda.synchronize()
        run_steps(cg, torch, ist, sgd, 5, cg.CG_STEP_OVERLAP)
        sync(torch, ist)
        t0 = time.perf_counter()
        run_steps(cg, torch, ist, sgd, args.inception_steps, cg.CG_STEP_OVERLAP)
        sync(torch, ist)
        ims = (time.perf_counter() - t0) / args.inception_steps * 1e3
        inception = {"workload": "inception_stack_192x28x28_B32_K8", "ms_per_step": ims, "images_per_s": 32 / (ims * 1e-3),
                     "steps": args.inception_steps}
        del ist
        torch.cuda.empty_cache()

    googlenet = None
    if args.googlenet_steps > 0 and not args.serial:
        googlenet = googlenet_workload(cg, torch, sgd, args.googlenet_steps, cg.CG_STEP_OVERLAP)

    # ---- configuration 2 stand-alone (every layer's three passes, the first layer's backward-data included)
    # and the other per-worker batch configuration 4 names (B = 64), as context beside the headline
    layer_bench = b64 = reduced = None
    if not args.skip_layer_bench and not args.serial:
        layer_bench = conv_layers_standalone(cg, torch, B)
        reduced = reduced_precision(cg, torch, B, K, sgd)
        if B != 64:
            st64 = build_net(cg, torch, 64, K, seed=4, n_batches=16)
            torch.cuda.synchronize()
            run_steps(cg, torch, st64, sgd, 5, cg.CG_STEP_OVERLAP)
            sync(torch, st64)
            t0 = time.perf_counter()
            run_steps(cg, torch, st64, sgd, 50, cg.CG_STEP_OVERLAP)
            sync(torch, st64)
            ms64 = (time.perf_counter() - t0) / 50 * 1e3
            b64 = {"workload": f"alexnet_shaped_train_step_B64_K{K}", "ms_per_step": ms64, "images_per_s": 64 / (ms64 * 1e-3),
                   "steps": 50}
            del st64
            torch.cuda.empty_cache()

    # the oracle last: its OpenMP workers keep spinning for a while after their last loop and would
    # take host cores from the launch-bound workloads above
    cpu = cpu_baseline(args.cpu_sample, K) if args.cpu_sample > 0 else None

    out = {
        "metric": "images/sec per fwd+bwd+update step (AlexNet-shaped B=256); grad-update HBM GB/s",
        "value": B / (ms_per_step * 1e-3), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"alexnet_shaped_train_step_B{B}_K{K}", "global_batch": B, "peers": K,
                   "schedule": "serial" if args.serial else "overlap", "lr": 0.01, "mu": 0.9, "wd": 5e-4},
        # the kernel's own speed: timed alone on the GPU (one-stream pass of the same iteration, same
        # process, HIP events around every launch); the shared-GPU durations of the timed region follow
        "roofline": roofline_excl if roofline_excl else roofline,
        "roofline_three_stream_pass" if not args.serial else "roofline_instrumented_pass": roofline,
        "update_roofline": update_excl if update_excl else update_roofline,
        "update_roofline_three_stream_pass" if not args.serial else "update_roofline_instrumented_pass": update_roofline,
        "whole_step_matrix_core": {"tflops": totals["flops_per_step"] / (ms_per_step * 1e-3) / 1e12,
                                   "frac": totals["flops_per_step"] / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                                   "what": "algorithmic FLOP of all matrix-core launches of a step / wall time of the step "
                                           "(glue layers and updates included in the time)"},
        "matrix_core_kernels_exclusive": totals_excl,
        "ms_per_step_with_launch_events": inst_ms,
        "serial_schedule_ms_per_step": serial_ms,
        "kernel_launches_per_step": launches_per_step,
        "gpu_clocks_after_timed_region": clocks,
        "grad_update": grad_update,
        "hbm_achievable": achievable,
        "mfma_achievable": mfma_peak,
        "conv_layers_standalone": layer_bench,
        "alexnet_b64_step": b64,
        "reduced_precision": reduced,
        "inception_step": inception,
        "googlenet_step": googlenet,
        "cpu_baseline": cpu,
        "loss": loss,
        "paper_context_s_per_iter_other_hw": PAPER_ALEXNET_S_PER_ITER,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
