#!/usr/bin/env python3
"""Benchmark of the out-of-core training step on one MI355X.

Workload (configs[1] of the baseline): 24-layer GPT-style pre-LN transformer, hidden 1024,
16 heads, FFN 4096, sequence 1024, batch 32, vocabulary 32000, bf16 compute with fp32 host
master weights and host Adam, HBM budget 16 GiB, seeded synthetic token ids.

One "step" = one whole training step (forward, loss, backward with swap-out / prefetch /
recompute as planned, gradient D2H, host Adam, weight H2D).  The in-core rate (same
library, same kernels, budget lifted) is measured alongside.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

GIB = 1 << 30
# configs[1] of the baseline is the benchmark workload; configs[3] (8.3B parameters, weights
# streamed per layer from the host) runs with --config 3
WORKLOADS = {
    1: dict(cfg=dict(n_layers=24, hidden=1024, heads=16, ffn=4096, vocab=32000, seq=1024, batch=32),
            budget=16 * GIB, arena=32 * GIB, seed=2008114202, stream=0,
            name="configs[1]: 24-layer pre-LN GPT, hidden 1024, 16 heads, FFN 4096, seq 1024, batch 32, "
                 "vocab 32000, bf16 + fp32 host master/Adam, HBM budget 16 GiB"),
    2: dict(cfg=dict(width=64, stage_blocks=(3, 24, 36, 3), image=224, batch=64, classes=1000),
            budget=32 * GIB, arena=40 * GIB, seed=2008114203, stream=0, kind="cnn", low_budget=4 * GIB,
            name="configs[2]: ResNet-200-shaped bottleneck CNN (stages 3/24/36/3, widths 256..2048), 224x224x3 images, "
                 "batch 64, 1000 classes, BatchNorm + ReLU, bf16, host SGD with momentum, HBM budget 32 GiB"),
    3: dict(cfg=dict(n_layers=72, hidden=3072, heads=24, ffn=12288, vocab=51200, seq=1024, batch=8),
            budget=32 * GIB, arena=96 * GIB, seed=2008114204, stream=2,
            name="configs[3]: 72-layer pre-LN GPT (8.3B parameters), hidden 3072, 24 heads, FFN 12288, seq 1024, "
                 "batch 8, vocab 51200, bf16 weights streamed per layer from pinned host memory (gradients land in the same pinned buffers), fp32 host "
                 "master/Adam, HBM budget 32 GiB"),
    4: dict(cfg=dict(n_layers=78, hidden=4256, heads=28, ffn=17024, vocab=51200, seq=1024, batch=4),
            budget=32 * GIB, arena=96 * GIB, seed=2008114205, stream=2, whole_blocks=True,
            name="configs[4]: 78-layer pre-LN GPT (17B parameters), hidden 4256, 28 heads of 152, FFN 17024, seq 1024, "
                 "batch 4, vocab 51200, bf16 weights streamed per layer from pinned host memory (gradients land in "
                 "the same pinned buffers) and activations swapped, fp32 host master/Adam (about 225 GiB of host "
                 "memory), HBM budget 32 GiB"),
    5: dict(cfg=dict(width=160, group_blocks=(4, 4, 4), image=32, batch=1024, classes=10),
            budget=16 * GIB, arena=20 * GIB, seed=2008114206, stream=0, kind="wrn", low_budget=5 * GIB,
            name="supplementary (Table III, second CNN family): WRN-28-10 (pre-activated basic blocks, widths 160/320/640), "
                 "32x32x3 images, batch 1024, 10 classes stored as 16, BatchNorm + ReLU, bf16, host SGD with momentum, "
                 "HBM budget 16 GiB"),
    6: dict(cfg=dict(width=64, stage_blocks=(3, 4, 6, 3), image=224, batch=512, classes=1000),
            budget=48 * GIB, arena=56 * GIB, seed=2008114207, stream=0, kind="cnn", low_budget=16 * GIB,
            name="supplementary (Table III; the setting of the paper's blocking study, Fig. 7): ResNet-50-shaped bottleneck CNN "
                 "(stages 3/4/6/3), 224x224x3 images, batch 512, 1000 classes, bf16, host SGD with momentum; in-core under 48 GiB, "
                 "then under a 16 GiB budget"),
    7: dict(cfg=dict(width=64, depth=4, image=512, batch=16, classes=2),
            budget=24 * GIB, arena=28 * GIB, seed=2008114208, stream=0, kind="unet", low_budget=6 * GIB,
            name="supplementary (Table III, fully convolutional; Sec. III-F.3: connections from the contracting to the expansive "
                 "path): U-Net (depth 4, 64..1024 channels, 31 M parameters), 512x512 one-channel images, batch 16, 2 classes "
                 "stored as 8, BatchNorm + ReLU, bf16, host SGD with momentum; in-core under 24 GiB, then under a 6 GiB budget"),
}
CFG = WORKLOADS[1]["cfg"]
BUDGET = WORKLOADS[1]["budget"]
ARENA = WORKLOADS[1]["arena"]
SEED = WORKLOADS[1]["seed"]
PEAK_BF16_TFLOPS = 2500.0
# HBM-side bytes per GEMM launch come from rocprofv3 counter runs of this command (FETCH_SIZE and
# WRITE_SIZE of all GEMM launches, each scaled by the same counter's reading for the 1 GiB copy
# below); the summary of those runs records the plan it was taken on.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gpt24_step_kernel_stats_and_hbm_traffic.txt")
CPU_SAMPLE_BATCH = 8   # sequences in the oracle's timed sample (about 20 s of host work)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


COSTS_DIR = os.path.join(ROOT, "paper_2008_11421_amd", "costs")


def costs_file(config):
    return os.path.join(COSTS_DIR, "configs%d_mi355x.json" % config)


def save_costs(path, layers, loss_c, link):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        json.dump({"what": "cost records measured once by karma_measure on an MI355X (Sec. III-D: the model is profiled "
                           "once); bench.py plans on these so that the benchmarked plan is the same from run to run",
                   "layers": [list(l) for l in layers], "loss": list(loss_c), "link": list(link)}, f, indent=0)
        f.write("\n")


def load_costs(path, n_layers):
    try:
        d = json.load(open(path))
    except (OSError, ValueError):
        return None
    if len(d.get("layers", ())) != n_layers:
        return None
    return [tuple(l) for l in d["layers"]], tuple(d["loss"]), tuple(d["link"])


def profiled_traffic(plan):
    """Bytes per GEMM launch from the committed counter summary, if it was taken on this very plan
    (lines `plan: <string>` and `gemm_traffic_bytes_per_launch: <number>`); None otherwise."""
    try:
        fields = dict(l.split(":", 1) for l in open(TRAFFIC_PROFILE) if l.startswith(("plan:", "gemm_traffic_bytes_per_launch:")))
        if fields["plan"].strip() == plan:
            return float(fields["gemm_traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def bandwidth_kernels(K, torch):
    """The HBM-bound kernels of the step at the workload's shapes, timed standalone with events on the stream
    they are launched on; each call works on its own buffers out of a ring larger than the 256 MB last-level
    cache, so that what is measured is memory, not cache.  Algorithmic bytes: what the kernel has to read and
    write once (LayerNorm forward x, y; its backward dy, x, the residual gradient it adds, dx; softmax
    cross-entropy reads the logits and writes their gradient)."""
    import ctypes as C
    lib = K.lib()
    rows, h, vocab, chunk = CFG["batch"] * CFG["seq"], CFG["hidden"], CFG["vocab"], 4096
    s = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: C.c_void_p(t.data_ptr())
    ring = 6
    bf = lambda *shape: [torch.randn(*shape, device="cuda").to(torch.bfloat16) for _ in range(ring)]
    x, y, dy, add = bf(rows, h), bf(rows, h), bf(rows, h), bf(rows, h)
    g = torch.ones(h, device="cuda").to(torch.bfloat16)
    b = torch.zeros(h, device="cuda").to(torch.bfloat16)
    stats = torch.empty(rows, 2, dtype=torch.float32, device="cuda")
    ws = torch.empty((rows + 63) // 64 * 3 * h, dtype=torch.float32, device="cuda")
    dg, db, cs = (torch.empty(h, dtype=torch.float32, device="cuda") for _ in range(3))
    logits = bf(chunk, vocab)
    labels = torch.randint(0, vocab, (chunk,), dtype=torch.int32, device="cuda")
    rowloss = torch.empty(chunk, dtype=torch.float32, device="cuda")
    lib.karma_k_layernorm_fwd_bf16(p(x[0]), p(g), p(b), p(y[0]), p(stats), rows, h, s)   # statistics for the backward
    calls = {
        "layernorm_fwd": (4 * rows * h, lambda k: lib.karma_k_layernorm_fwd_bf16(p(x[k]), p(g), p(b), p(y[k]), p(stats), rows, h, s)),
        "layernorm_bwd_with_residual_gradient_and_its_column_sums":
            (8 * rows * h, lambda k: lib.karma_k_layernorm_bwd_addsum_bf16(p(dy[k]), p(x[k]), p(stats), p(g), p(add[k]), p(y[k]), p(dg),
                                                                        p(db), p(cs), p(ws), C.c_uint64(ws.numel() * 4), rows, h, s)),
        "softmax_cross_entropy_4096_rows": (4 * chunk * vocab, lambda k: lib.karma_k_softmax_ce_bf16(p(logits[k]), p(labels), p(rowloss), chunk, vocab,
                                                                                                C.c_float(1.0 / chunk), s)),
    }
    out = {}
    for name, (nbytes, f) in calls.items():
        for k in range(ring):
            assert f(k) == 0, name
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 4 * ring
        e0.record()
        for k in range(reps):
            f(k % ring)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        out[name] = {"algorithmic_bytes": nbytes, "avg_us": us, "achieved_gbps": nbytes / us / 1e3, "frac_of_8000_gbps": nbytes / us / 1e3 / 8000.0}
    return out


def batch_sweep(args, K, si, torch, np, threads):
    """The benchmark model across batch sizes under one fixed HBM budget (the x-axis of the paper's Fig. 5: the
    first points fit the budget, the rest do not), each beside the same batch with all of HBM (in-core) and beside
    what the analytic cost model (operation counts on two device rates, no measurement of the model) projects.
    One JSON line; not the benchmark line."""
    rows = []
    rates = (490 * 10**12, 3 * 10**12)      # multiply-adds per second on the matrix cores, other operations per second
    for batch in (8, 16, 32, 64, 128):
        desc = dict(kind=K.MODEL_GPT, n_layers=CFG["n_layers"], width=CFG["hidden"], batch=batch, seq=CFG["seq"],
                    n_heads=CFG["heads"], ffn=CFG["ffn"], vocab=CFG["vocab"], stream_weights=0, split_blocks=1)
        a_layers, a_loss, fixed = K.karma_model_costs(desc, *rates)
        in_core_need = fixed + sum(l[3] + l[4] for l in a_layers) + 2 * max(max(l[5] for l in a_layers), a_loss[1])
        arena = max(min(in_core_need + 2 * GIB, 200 * GIB), BUDGET) // 256 * 256
        cfg = dict(optimizer=K.OPT_ADAM, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, host_threads=threads, device_update_first=1)
        ctx = K.Context(desc, cfg, arena)
        params, ids, labels = si.gpt_problem(seed=SEED, n_layers=1, hidden=CFG["hidden"], ffn=CFG["ffn"], vocab=CFG["vocab"],
                                             seq=CFG["seq"], batch=batch)
        ctx.karma_set_param(0, 0, params["wte"])
        ctx.karma_set_param(0, 1, params["wpe"])
        for i in range(CFG["n_layers"]):
            for t, name in enumerate(si.GPT_BLOCK_TENSORS):
                v = np.roll(np.asarray(params["blocks"][0][name], dtype=np.float32).reshape(-1), 97 * i)
                ctx.karma_set_param(2 * i + 1 if t < 6 else 2 * i + 2, t if t < 6 else t - 6, v)
        ctx.karma_set_param(2 * CFG["n_layers"] + 1, 0, params["lnf_g"])
        ctx.karma_set_param(2 * CFG["n_layers"] + 1, 1, params["lnf_b"])
        ids, labels = ids.astype(np.int32), labels.astype(np.int32)
        link = ctx.karma_measure(2)

        def timed(budget):
            acts, summ = ctx.karma_plan(budget)
            for _ in range(2):
                ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
            ctx.karma_finish_updates()
            torch.cuda.synchronize()
            per_step = []
            for _ in range(max(3, args.steps // 4)):
                t1 = time.perf_counter()
                ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
                per_step.append(time.perf_counter() - t1)
            ctx.karma_finish_updates()
            torch.cuda.synchronize()
            return acts, summ, median(per_step)

        acts_in, _, dt_in = timed(arena)
        ctx.karma_refine_host_costs()
        acts, summ, dt = timed(BUDGET)
        # the analytic projection of the same question: planned step over in-core step
        link3 = (int(link[0]), int(link[1]), int(link[2]))
        try:
            _, s_an = K.karma_plan_pure(a_layers, link3, a_loss, BUDGET, fixed)
            _, s_an_in = K.karma_plan_pure(a_layers, link3, a_loss, 1 << 50, fixed)
            analytic_pct = 100.0 * s_an_in["makespan_ns"] / s_an["makespan_ns"]
        except K.KarmaError:
            analytic_pct = None
        row = {"batch": batch, "in_core_fits_budget": acts == [K.KEEP] * len(acts), "in_core_ms_per_step": dt_in * 1e3,
               "in_core_samples_per_s": batch / dt_in, "budget_ms_per_step": dt * 1e3, "budget_samples_per_s": batch / dt,
               "pct_of_in_core": 100.0 * dt_in / dt, "predicted_ms": summ["makespan_ns"] / 1e6,
               "analytic_model_pct_of_in_core": analytic_pct, "plan": "".join("KSRrc"[a] for a in acts),
               "in_core_arena_gib": arena / GIB, "link_gib_each_way": [summ["bytes_d2h"] / GIB, summ["bytes_h2d"] / GIB]}
        log("batch %d: in-core %.1f ms (%.0f samples/s, arena %.0f GiB), %d GiB budget %.1f ms (%.0f samples/s, %.1f %%), plan %s"
            % (batch, dt_in * 1e3, batch / dt_in, arena / GIB, BUDGET // GIB, dt * 1e3, batch / dt, 100 * dt_in / dt, row["plan"]))
        row["in_core_run_kept_everything"] = acts_in == [K.KEEP] * len(acts_in)
        rows.append(row)
        ctx.close()
        del ctx
        torch.cuda.empty_cache()
    print(json.dumps({"what": "batch sweep of the configs[1] model under a %d GiB HBM budget, beside the same batch in-core"
                              % (BUDGET // GIB), "unit": "samples/s", "data": "synthetic", "dtype": "bf16", "rows": rows}), flush=True)


def cpu_baseline(n_seq):
    """The oracle as it stands, timed on the host: a few sequences at true widths with the
    depth truncated to 1 and to 2 blocks; block and head costs extrapolated to 24 blocks."""
    import numpy as np
    from oracle import nn
    import synth_inputs as si
    ts = []
    for depth in (1, 2):
        params, ids, labels = si.gpt_problem(seed=SEED, n_layers=depth, hidden=CFG["hidden"], ffn=CFG["ffn"],
                                             vocab=CFG["vocab"], seq=CFG["seq"], batch=n_seq)
        t0 = time.perf_counter()
        nn.gpt_step(params, ids, labels, CFG["heads"])
        ts.append(time.perf_counter() - t0)
    t_block = max(ts[1] - ts[0], 1e-9)
    t_rest = max(ts[0] - t_block, 0.0)
    per_sample = (CFG["n_layers"] * t_block + t_rest) / n_seq
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return dict(value=1.0 / per_sample, unit="samples/s", cores=cores, kind="oracle",
                sample="fp64 numpy oracle, full step on %d sequences of 1024 tokens at true widths, depth 1 and 2 "
                       "(%.1f s + %.1f s); per-block %.2f s and embedding+head %.2f s extrapolated to %d blocks"
                       % (n_seq, ts[0], ts[1], t_block, t_rest, CFG["n_layers"]))


def backward_stalls(ctx, step_fn, n_records):
    """The stall profile of the backward phase (Sec. V, Fig. 6): one step with events around every op; for each
    compute op from the loss on, the time the compute stream stood idle before it began (waiting for a swap-in,
    a weight copy or a free buffer), summed per layer; the plan's simulated schedule read the same way."""
    step_fn()
    ops = ctx.karma_get_op_times()
    starts = ctx.karma_get_op_starts()

    def per_layer(times):
        stall = [0.0] * (n_records + 1)
        prev_end, backward = None, False
        for (kind, layer, _, _, _), (t0, t1) in zip(ops, times):
            if kind not in "FRBL":
                continue
            backward = backward or kind == "L"
            if backward and prev_end is not None:
                stall[min(layer, n_records)] += max(0.0, t0 - prev_end)
            prev_end = t1
        return stall

    measured = per_layer([(st, st + op[4]) for op, st in zip(ops, starts)])
    predicted = per_layer([(op[2] / 1e6, op[3] / 1e6) for op in ops])
    return {"by_layer_ms": [round(x, 4) for x in measured], "total_ms": sum(measured),
            "simulated_total_ms": sum(predicted)}


STALL_NOTE = ("compute-stream idle time before the backward-phase ops (loss, recompute, backward) of each layer, from one "
              "step with events around every op; index = layer record, last = loss")


def host_memory_note():
    """Resident and pinned memory of this process as the kernel reports them (a log line only)."""
    out = []
    try:
        for line in open("/proc/self/status"):
            if line.split(":")[0] in ("VmRSS", "VmHWM", "VmLck", "VmPin"):
                out.append(" ".join(line.split()))
        for line in open("/proc/meminfo"):
            if line.split(":")[0] in ("MemAvailable",):
                out.append(" ".join(line.split()))
    except OSError:
        pass
    return ", ".join(out)


# KARMA_STEP_KERNEL_TIMES puts HIP events around one GEMM launch in eight and rotates which ones
# from step to step: events around every launch would lengthen the timed steps by several percent
TIMER_STRIDE = 8
SAMPLING_NOTE = ("HIP events on the compute stream around one launch in eight of the timed steps, rotating so that eight "
                 "steps cover every launch of a step")


def bench_cnn(args, wl, K, si, torch, np, threads):
    """configs[2]: the bottleneck CNN, and the wide residual network (the second CNN family of Table III).
    Both fit their budget in-core (the planner returns all-KEEP); a supplementary run under `low_budget`
    shows the out-of-core schedule."""
    cfg_m = wl["cfg"]
    cfg = dict(optimizer=K.OPT_SGD_MOMENTUM, lr=1e-3, beta1=0.9, beta2=0.0, eps=0.0, host_threads=threads)
    t0 = time.perf_counter()
    if wl["kind"] == "unet":
        classes = (cfg_m["classes"] + 7) // 8 * 8
        depth = cfg_m["depth"]
        desc = dict(kind=K.MODEL_UNET, n_layers=depth, width=cfg_m["width"], batch=cfg_m["batch"], seq=cfg_m["image"], n_heads=0,
                    ffn=0, vocab=classes, stream_weights=0, stage_blocks=(0, 0, 0, 0))
        ctx = K.Context(desc, cfg, wl["arena"])
        params, images, labels = si.unet_problem(seed=wl["seed"], **cfg_m)
        images = images[..., 0]
        for l, p in enumerate(params["down"]):
            for t, name in enumerate(si.LEVEL_TENSORS):
                v = p[name]
                if l == 0 and name == "w1":      # the one image channel is stored as eight
                    v = np.concatenate([v, np.zeros(v.shape[:3] + (7,))], axis=3)
                ctx.karma_set_param(l, t, v)
        for j, p in enumerate(params["up"]):
            c = p["w1"].shape[3] // 2            # the first weight as two tensors: contracting half, up-convolution half
            for t, v in enumerate((p["wu"], p["w1"][..., :c], p["w1"][..., c:], p["g1"], p["b1"], p["w2"], p["g2"], p["b2"])):
                ctx.karma_set_param(depth + 1 + j, t, v)
        hd = params["head"]
        fc = np.zeros((classes, hd["w"].shape[1]), dtype=np.float32)
        fc[:cfg_m["classes"]] = hd["w"]
        bias = np.full(classes, -30000.0, dtype=np.float32)
        bias[:cfg_m["classes"]] = hd["bias"]
        ctx.karma_set_param(2 * depth + 1, 0, fc)
        ctx.karma_set_param(2 * depth + 1, 1, bias)
        params = dict(blocks=[])
    elif wl["kind"] == "wrn":
        classes = (cfg_m["classes"] + 7) // 8 * 8      # stored classes: the extra ones can never be predicted
        desc = dict(kind=K.MODEL_WRN, n_layers=0, width=cfg_m["width"], batch=cfg_m["batch"], seq=cfg_m["image"], n_heads=0,
                    ffn=0, vocab=classes, stream_weights=0, stage_blocks=tuple(cfg_m["group_blocks"]) + (0,))
        ctx = K.Context(desc, cfg, wl["arena"])
        params, images, labels = si.wrn_problem(seed=wl["seed"], **cfg_m)
        tensors = si.BASIC_TENSORS
        w = params["stem"]["w"]
        wp = np.zeros(w.shape[:3] + (8,), dtype=np.float32)
        wp[..., :3] = w
        ctx.karma_set_param(0, 0, wp)
        L = len(params["blocks"]) + 1
        hd = params["head"]
        fc = np.zeros((classes, hd["w"].shape[1]), dtype=np.float32)
        fc[:cfg_m["classes"]] = hd["w"]
        bias = np.full(classes, -30000.0, dtype=np.float32)
        bias[:cfg_m["classes"]] = hd["bias"]
        for t, v in enumerate((hd["g"], hd["b"], fc, bias)):
            ctx.karma_set_param(L, t, v)
    else:
        desc = dict(kind=K.MODEL_CNN, n_layers=0, width=cfg_m["width"], batch=cfg_m["batch"], seq=cfg_m["image"], n_heads=0,
                    ffn=0, vocab=cfg_m["classes"], stream_weights=0, stage_blocks=cfg_m["stage_blocks"])
        ctx = K.Context(desc, cfg, wl["arena"])
        params, images, labels = si.cnn_problem(seed=wl["seed"], **cfg_m)
        tensors = si.BOTTLENECK_TENSORS
        w = params["stem"]["w"]
        wp = np.zeros(w.shape[:3] + (8,), dtype=np.float32)
        wp[..., :3] = w
        ctx.karma_set_param(0, 0, wp)
        ctx.karma_set_param(0, 1, params["stem"]["g"])
        ctx.karma_set_param(0, 2, params["stem"]["b"])
        L = len(params["blocks"]) + 1
        ctx.karma_set_param(L, 0, params["head"]["w"])
        ctx.karma_set_param(L, 1, params["head"]["b"])
    for i, (p, _) in enumerate(params["blocks"]):
        for t, name in enumerate(tensors):   # (the fully convolutional network has loaded its levels above)
            if name in p:
                ctx.karma_set_param(i + 1, t, p[name])
    del params
    images = images.astype(np.float32)
    labels = labels.astype(np.int32)
    log("setup %.1f s" % (time.perf_counter() - t0))
    link = ctx.karma_measure(3)
    layers, loss_c, fixed = ctx.karma_get_costs()
    log("link h2d %.1f GB/s d2h %.1f GB/s; fixed %.2f GiB; saved sets %.2f GiB; forward %.1f ms backward %.1f ms"
        % (link[0] / 1e9, link[1] / 1e9, fixed / GIB, sum(l[3] + l[4] for l in layers) / GIB,
           sum(l[0] for l in layers) / 1e6, sum(l[1] for l in layers) / 1e6))

    def timed(budget, flags, resident=True):
        """resident: the timed steps run on the batch already in HBM (the warm-up steps put it there); otherwise every
        step converts the fp32 images on the host and copies them over the link first."""
        acts, summ = ctx.karma_plan(budget)
        for _ in range(max(args.warmup, 1)):
            ctx.karma_step(images, labels, flags)
        ctx.karma_finish_updates()   # host updates a step put off belong to the steps that produced them
        torch.cuda.synchronize()
        n_l, ms_l, fl_l = 0, 0.0, 0.0
        per_step = []
        for _ in range(args.steps):
            t1 = time.perf_counter()
            loss = ctx.karma_step(None if resident else images, None if resident else labels, flags)
            per_step.append(time.perf_counter() - t1)
            if flags & K.STEP_KERNEL_TIMES:
                n, ms, fl = ctx.karma_get_gemm_stats()
                n_l += n; ms_l += ms; fl_l += fl
        ctx.karma_finish_updates()
        torch.cuda.synchronize()
        return acts, summ, median(per_step), loss, (n_l, ms_l, fl_l), ctx.karma_get_stats()

    _, _, dt_host, _, _, _ = timed(wl["budget"], K.STEP_APPLY_OPTIMIZER, resident=False)
    acts, summ, dt, loss, gem, st = timed(wl["budget"], K.STEP_APPLY_OPTIMIZER | K.STEP_KERNEL_TIMES)
    log("%d GiB: %.1f ms/step (%.1f when every step takes its images from host memory), all-keep=%s, peak %.2f GiB"
        % (wl["budget"] // GIB, dt * 1e3, dt_host * 1e3, acts == [0] * len(acts), summ["peak_bytes"] / GIB))
    profiled_step = lambda: ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER | K.STEP_PROFILE)
    stalls_in = backward_stalls(ctx, profiled_step, len(acts))
    acts_lo, summ_lo, dt_lo, loss_lo, _, _ = timed(wl["low_budget"], K.STEP_APPLY_OPTIMIZER)
    stalls_lo = backward_stalls(ctx, profiled_step, len(acts_lo))
    log("backward-phase stalls of the compute stream: %d GiB %.2f ms, %d GiB %.2f ms (simulated %.2f ms)"
        % (wl["budget"] // GIB, stalls_in["total_ms"], wl["low_budget"] // GIB, stalls_lo["total_ms"], stalls_lo["simulated_total_ms"]))
    log("%d GiB: %.1f ms/step, plan %s" % (wl["low_budget"] // GIB, dt_lo * 1e3, "".join("KSRrc"[a] for a in acts_lo)))
    # the same budget with the block granularity chosen by the planner as well (Sec. III-E/F, first tier)
    acts_g, summ_g, group = ctx.karma_plan_grouped(wl["low_budget"])
    for _ in range(2):
        ctx.karma_step(images, labels, K.STEP_APPLY_OPTIMIZER)
    ctx.karma_finish_updates()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        ctx.karma_step(None, None, K.STEP_APPLY_OPTIMIZER)
    ctx.karma_finish_updates()
    torch.cuda.synchronize()
    dt_g = (time.perf_counter() - t2) / args.steps
    log("%d GiB, grouped planner: blocks of %d records, %.1f ms/step (predicted %.1f vs %.1f ms), plan %s"
        % (wl["low_budget"] // GIB, group, dt_g * 1e3, summ_g["makespan_ns"] / 1e6, summ_lo["makespan_ns"] / 1e6,
           "".join("KSRrc"[a] for a in acts_g)))
    n_l, ms_l, fl_l = gem
    achieved = fl_l / (ms_l * 1e-3) / 1e12 if ms_l > 0 else 0.0
    batch = cfg_m["batch"]
    out = {
        "metric": "samples/s at fixed HBM budget", "value": batch / dt, "unit": "samples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl["name"], "hbm_budget_gib": wl["budget"] // GIB, "global_batch": batch,
                   "plan": "".join("KSRrc"[a] for a in acts)},
        "inputs": "the batch is resident in HBM during the timed steps (put there by the warm-up steps)",
        "with_inputs_from_host_memory": {"ms_per_step": dt_host * 1e3, "samples_per_s": batch / dt_host,
                                         "what": "every step converts its fp32 images to bf16 on the host and copies them over the link first"},
        "in_core_samples_per_s": batch / dt, "pct_of_in_core": 100.0, "loss": loss,
        "predicted_makespan_ms": summ["makespan_ns"] / 1e6, "arena_peak_gib": summ["peak_bytes"] / GIB,
        "supplementary_low_budget": {"hbm_budget_gib": wl["low_budget"] // GIB, "ms_per_step": dt_lo * 1e3,
                                     "samples_per_s": batch / dt_lo, "pct_of_in_core": 100.0 * dt / dt_lo,
                                     "plan": "".join("KSRrc"[a] for a in acts_lo), "arena_peak_gib": summ_lo["peak_bytes"] / GIB,
                                     "link_gib_d2h_total": summ_lo["bytes_d2h"] / GIB,
                                     "backward_stall_profile": {"what": STALL_NOTE, "in_core": stalls_in, "out_of_core": stalls_lo},
                                     "grouped_planner": {"group_size": group, "ms_per_step": dt_g * 1e3,
                                                         "predicted_makespan_ms": summ_g["makespan_ns"] / 1e6,
                                                         "plan": "".join("KSRrc"[a] for a in acts_g)}},
        "host_link_gbps": {"h2d": link[0] / 1e9, "d2h": link[1] / 1e9}, "host_opt_ms": st["host_opt_ms"],
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_kernel and gemm_bf16_dl_kernel (convolutions as implicit GEMMs, the FC layer / classifier; " + SAMPLING_NOTE + ")",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "launches_per_step": n_l * TIMER_STRIDE / max(args.steps, 1), "avg_launch_ms": ms_l / max(n_l, 1),
                     "flops_per_launch": fl_l / max(n_l, 1), "traffic": None},
    }
    ctx.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-policies", action="store_true", help="skip the comparison policies (profiling runs)")
    ap.add_argument("--config", type=int, default=1, choices=sorted(WORKLOADS))
    ap.add_argument("--whole-blocks", action="store_true",
                    help="GPT workloads: one plannable record per transformer block instead of two (attention half, "
                         "feed-forward half)")
    ap.add_argument("--costs", default="frozen", choices=("frozen", "measured"),
                    help="plan on the committed cost records of this workload (default; falls back to this run's own "
                         "measurements when there are none) or on this run's measurements")
    ap.add_argument("--save-costs", action="store_true", help="write this run's measured cost records to the committed file")
    ap.add_argument("--device-update-first", type=int, default=None,
                    help="GPT workloads: how many leading records are updated on the device instead of the host (default: the "
                         "embedding record, and for the default workload the first block's two halves as well)")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="configs[1] only: batches 8..128 under the budget and in-core (a supplementary line, not the benchmark)")
    ap.add_argument("--layers", type=int, default=0,
                    help="GPT workloads: truncate the depth to this many blocks (named in config.workload)")
    args = ap.parse_args()
    global CFG, BUDGET, ARENA, SEED
    wl = dict(WORKLOADS[args.config])
    if args.layers and wl.get("kind") not in ("cnn", "wrn", "unet") and 0 < args.layers < wl["cfg"]["n_layers"]:
        wl["cfg"] = dict(wl["cfg"], n_layers=args.layers)
        wl["name"] += " -- DEPTH TRUNCATED to %d blocks for this run" % args.layers
    CFG, BUDGET, ARENA, SEED = wl["cfg"], wl["budget"], wl["arena"], wl["seed"]
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2008_11421_amd as K
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    K.lib()   # fails loudly when the HIP library is missing

    # A plain copy of known size (1 GiB read, 1 GiB written) so that a profiler run of this
    # command holds a kernel against which its HBM byte counters can be scaled.
    cal_src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    torch.mul(cal_src, 1.0, out=cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    torch.cuda.empty_cache()

    threads = int(os.environ.get("OMP_NUM_THREADS", "16"))
    if wl.get("kind") in ("cnn", "wrn", "unet"):
        return bench_cnn(args, wl, K, si, torch, np, threads)
    if args.batch_sweep:
        if args.config != 1:
            print("bench.py: --batch-sweep is for the default workload", file=sys.stderr)
            sys.exit(2)
        return batch_sweep(args, K, si, torch, np, threads)
    desc = dict(kind=K.MODEL_GPT, n_layers=CFG["n_layers"], width=CFG["hidden"], batch=CFG["batch"], seq=CFG["seq"],
                n_heads=CFG["heads"], ffn=CFG["ffn"], vocab=CFG["vocab"], stream_weights=wl["stream"],
                split_blocks=0 if (args.whole_blocks or wl.get("whole_blocks")) else 1)
    split = bool(desc["split_blocks"])

    def slot(block, t):   # (record, tensor) of tensor t of transformer block `block`
        if not split:
            return block + 1, t
        return (2 * block + 1, t) if t < 6 else (2 * block + 2, t - 6)
    n_records = (2 if split else 1) * CFG["n_layers"] + 1
    # the embedding record and, where weights are resident, the first transformer block (last to finish in backward,
    # first to be read in forward) keep their optimiser state in HBM and are updated there; every other block and
    # the final LayerNorm are updated on the host
    cfg = dict(optimizer=K.OPT_ADAM, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, host_threads=threads,
               device_update_first=(3 if args.config == 1 else 1) if args.device_update_first is None else args.device_update_first)
    t0 = time.perf_counter()
    ctx = K.Context(desc, cfg, ARENA)
    # the 8.3B model draws one block's tensors and gives every layer a rolled copy of them
    # (drawing 8.3e9 normals on the host would take longer than the benchmark itself)
    n_drawn = CFG["n_layers"] if args.config == 1 else 1
    params, ids, labels = si.gpt_problem(seed=SEED, n_layers=n_drawn, hidden=CFG["hidden"], ffn=CFG["ffn"],
                                         vocab=CFG["vocab"], seq=CFG["seq"], batch=CFG["batch"])
    ctx.karma_set_param(0, 0, params["wte"])
    ctx.karma_set_param(0, 1, params["wpe"])
    for i in range(CFG["n_layers"]):
        b = params["blocks"][i % n_drawn]
        for t, name in enumerate(si.GPT_BLOCK_TENSORS):
            v = np.asarray(b[name], dtype=np.float32)
            ctx.karma_set_param(*slot(i, t), v if n_drawn > 1 else np.roll(v.reshape(-1), 97 * i))
        if n_drawn == 1 and i % 8 == 7:
            log("  parameters of %d layers set, %.0f s" % (i + 1, time.perf_counter() - t0))
    ctx.karma_set_param(n_records, 0, params["lnf_g"])
    ctx.karma_set_param(n_records, 1, params["lnf_b"])
    del params
    ids = ids.astype(np.int32)
    labels = labels.astype(np.int32)
    log("setup %.1f s; host memory of this process: %s" % (time.perf_counter() - t0, host_memory_note()))

    link = ctx.karma_measure(3)
    layers, loss_c, fixed = ctx.karma_get_costs()
    blk = (layers[1][0] + (layers[2][0] if split else 0), layers[1][1] + (layers[2][1] if split else 0))
    log("link h2d %.1f GB/s d2h %.1f GB/s lat %d ns (while the other direction and the host optimiser run: %.1f / %.1f); "
        "block fwd %.2f ms bwd %.2f ms; loss %.2f ms; host optimiser %.1f ms; fixed %.2f GiB"
        % (link[0] / 1e9, link[1] / 1e9, link[2], link[3] / 1e9, link[4] / 1e9, blk[0] / 1e6, blk[1] / 1e6, loss_c[0] / 1e6,
           (sum(l[8] for l in layers) + loss_c[2]) / 1e6, fixed / GIB))
    def timed(budget, flags):
        acts, summ = ctx.karma_plan(budget)
        for _ in range(args.warmup):
            ctx.karma_step(ids, labels, flags)
        ctx.karma_finish_updates()
        torch.cuda.synchronize()
        n_l, ms_l, fl_l = 0, 0.0, 0.0
        host_ms, per_step = [], []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            t1 = time.perf_counter()
            loss = ctx.karma_step(ids, labels, flags)      # returns with the streams drained
            per_step.append(time.perf_counter() - t1)
            host_ms.append(ctx.karma_get_stats()["host_opt_ms"])
            if flags & K.STEP_KERNEL_TIMES:
                n, ms, fl = ctx.karma_get_gemm_stats()
                n_l += n; ms_l += ms; fl_l += fl
        ctx.karma_finish_updates()
        torch.cuda.synchronize()
        mean_dt = (time.perf_counter() - t0) / args.steps
        # the median step (a step finishes the host updates its predecessor left pending, so steps of
        # a steady run are alike); the mean over the bracketed region is reported beside it
        dt = median(per_step)
        timed.mean_ms = mean_dt * 1e3
        st = ctx.karma_get_stats()
        # updates a step leaves pending are counted where they run (the next step, or the call above): the
        # average over the timed steps is the host optimiser's time per step
        host_ms[-1] = st["host_opt_ms"]
        st["host_opt_ms"] = sum(host_ms) / len(host_ms)
        return acts, summ, dt, loss, (n_l, ms_l, fl_l), st

    acts_in, summ_in, dt_in, loss_in, _, st_in = timed(ARENA, K.STEP_APPLY_OPTIMIZER)
    log("in-core: %.1f ms/step (host optimiser %.1f ms), plan all-keep=%s" % (dt_in * 1e3, st_in["host_opt_ms"], acts_in == [0] * len(acts_in)))
    profiled_step = lambda: ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER | K.STEP_PROFILE)
    stalls_in = backward_stalls(ctx, profiled_step, len(acts_in))
    # host-update times as the in-core steps above measured them on the real master weights and moments
    ctx.karma_refine_host_costs()
    layers, loss_c, fixed = ctx.karma_get_costs()
    log("host optimiser per step, from the steps themselves: %.1f ms" % ((sum(l[8] for l in layers) + loss_c[2]) / 1e6))
    # The plan this run's own measurements give, and the plan on the committed cost records (the model is profiled
    # once, Sec. III-D): the second is what is timed, so that the benchmarked plan is the same from run to run.
    cfile = costs_file(args.config) if not (args.layers or args.whole_blocks) else None
    if args.save_costs and cfile:
        save_costs(cfile, layers, loss_c, link)
        log("cost records written to", cfile)
    acts_own, summ_own = ctx.karma_plan(BUDGET)
    costs_used = "measured in this run"
    frozen = load_costs(cfile, len(layers)) if (cfile and args.costs == "frozen") else None
    if frozen:
        ctx.karma_set_costs(*frozen)
        costs_used = "committed records " + os.path.relpath(cfile, ROOT)
    log("costs: %s; plan on this run's own measurements: %s (predicted %.1f ms)"
        % (costs_used, "".join("KSRrc"[a] for a in acts_own), summ_own["makespan_ns"] / 1e6))

    acts, summ, dt, loss, gem, st = timed(BUDGET, K.STEP_APPLY_OPTIMIZER | K.STEP_KERNEL_TIMES)
    log("%d GiB: %.1f ms/step, plan %s, weights kept %s" % (BUDGET // GIB, dt * 1e3, acts, summ.get("wres")))
    # activations that cross the link each way (the summary's totals also count streamed weights and gradients)
    swap_bytes = sum((layers[i - 1][4] if i else 0) + (layers[i][3] if a == K.SWAP else 0)
                     for i, a in enumerate(acts) if a in (K.SWAP, K.RC_SWAP))
    log("predicted makespan %.1f ms (host optimiser done at %.1f ms), peak %.2f GiB, swap %.2f GiB each way" %
        (summ["makespan_ns"] / 1e6, summ["host_end_ns"] / 1e6, summ["peak_bytes"] / GIB, swap_bytes / GIB))

    # one more step with events around every op: achieved host-link rate during the swaps and
    # the measured occupancy of the compute stream (Eq. 1)
    stalls_out = backward_stalls(ctx, profiled_step, len(acts))
    log("backward-phase stalls of the compute stream: in-core %.2f ms, %d GiB %.2f ms (simulated %.2f ms)"
        % (stalls_in["total_ms"], BUDGET // GIB, stalls_out["total_ms"], stalls_out["simulated_total_ms"]))
    st_prof = ctx.karma_get_stats()
    swap = {"O": [0.0, 0.0], "I": [0.0, 0.0]}
    for kind, layer, t0_, t1_, ms in ctx.karma_get_op_times():
        if kind in swap:
            nbytes = (layers[layer - 1][4] if layer else 0) + (layers[layer][3] if acts[layer] == K.SWAP else 0)
            swap[kind][0] += nbytes
            swap[kind][1] += ms
    link_achieved = {("d2h" if k == "O" else "h2d"): (v[0] / (v[1] * 1e-3) / 1e9 if v[1] > 0 else None) for k, v in swap.items()}
    occupancy = st_prof["compute_busy_ms"] / st_prof["step_ms"] if st_prof["step_ms"] > 0 else None
    log("swap link achieved: %s GB/s; compute busy %.1f of %.1f ms" % (link_achieved, st_prof["compute_busy_ms"], st_prof["step_ms"]))

    # The comparison policies of Fig. 2 through the same executor, kernels and budget:
    # (a) eager swapping of every block, the last one included; (b) capacity-based swapping
    # without recompute (longest resident tail, the prefix swapped); plain checkpointing
    # every 5 blocks.  A few steps each: context for the planner's choice, not the metric.
    L = len(acts)
    swapped_prefix = 0
    candidates = {"eager_swap_all": [K.SWAP] * L,
                  "checkpoint_every_5": [K.RC_KEEP if i % 5 == 0 else K.RC_CHAIN for i in range(L)]}
    for k in range(1, L + 1):
        cand = [K.SWAP] * k + [K.KEEP] * (L - k)
        try:
            ctx.karma_set_plan(BUDGET, cand)
        except K.KarmaError:
            continue
        candidates["capacity_swap_no_recompute"] = cand
        swapped_prefix = k
        break
    policies = {}
    n_pol = max(2, min(5, args.steps))
    for name, cand in ({} if args.no_policies else candidates).items():
        try:
            sp = ctx.karma_set_plan(BUDGET, cand)
        except K.KarmaError as e:
            policies[name] = {"feasible": False, "reason": str(e)}
            continue
        ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
        ctx.karma_finish_updates()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(n_pol):
            ctx.karma_step(ids, labels, K.STEP_APPLY_OPTIMIZER)
        ctx.karma_finish_updates()
        torch.cuda.synchronize()
        dtp = (time.perf_counter() - t1) / n_pol
        stalls_p = backward_stalls(ctx, profiled_step, L)
        extra = {"swapped_prefix_records": swapped_prefix, "of_records": L} if name == "capacity_swap_no_recompute" else {}
        policies[name] = {"feasible": True, "ms_per_step": dtp * 1e3, "samples_per_s": CFG["batch"] / dtp,
                          "predicted_makespan_ms": sp["makespan_ns"] / 1e6, "planned_over_this": dtp / dt,
                          "backward_stall_ms": stalls_p["total_ms"], "backward_stall_simulated_ms": stalls_p["simulated_total_ms"],
                          **extra}
        log("policy %s: %.1f ms/step (planned schedule is %.2fx faster), backward-phase stalls %.1f ms (simulated %.1f)"
            % (name, dtp * 1e3, dtp / dt, stalls_p["total_ms"], stalls_p["simulated_total_ms"]))

    n_l, ms_l, fl_l = gem
    achieved = fl_l / (ms_l * 1e-3) / 1e12 if ms_l > 0 else 0.0
    out = {
        "metric": "samples/s at fixed HBM budget",
        "value": CFG["batch"] / dt,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "ms_per_step_is": "median of the timed steps",
        "ms_per_step_mean": timed.mean_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl["name"],
                   "hbm_budget_gib": BUDGET // GIB, "global_batch": CFG["batch"], "seq_len": CFG["seq"],
                   "weights_kept_between_forward_and_backward": summ.get("wres"),
                   "records": "embedding, then per transformer block its attention half and its feed-forward half"
                              if split else "embedding, then one per transformer block",
                   "plan": "".join("KSRrc"[a] for a in acts), "plan_legend": "K keep, S swap, R recompute from kept input, "
                   "r recompute from swapped input, c recompute in chain"},
        "in_core_samples_per_s": CFG["batch"] / dt_in,
        "in_core_ms_per_step": dt_in * 1e3,
        "pct_of_in_core": 100.0 * dt_in / dt,
        "loss": loss,
        "predicted_makespan_ms": summ["makespan_ns"] / 1e6,
        "predicted_host_optimiser_end_ms": summ["host_end_ns"] / 1e6,
        "predicted_over_measured": summ["makespan_ns"] / 1e6 / (dt * 1e3),
        "costs": costs_used,
        "plan_on_this_runs_measurements": {"plan": "".join("KSRrc"[a] for a in acts_own),
                                           "predicted_makespan_ms": summ_own["makespan_ns"] / 1e6},
        "arena_peak_gib": summ["peak_bytes"] / GIB,
        "swap_gib_each_way": swap_bytes / GIB,
        "plan_moves_gib": {"d2h": summ["bytes_d2h"] / GIB, "h2d": summ["bytes_h2d"] / GIB},
        "host_link_gbps": {"h2d": link[0] / 1e9, "d2h": link[1] / 1e9, "h2d_loaded": link[3] / 1e9, "d2h_loaded": link[4] / 1e9},
        "swap_link_achieved_gbps": link_achieved,
        "compute_occupancy_measured": occupancy,
        "compute_occupancy_predicted": summ["busy_ns"] / max(summ["busy_ns"] + summ["stall_ns"], 1),
        "host_opt_ms": st["host_opt_ms"],
        "backward_stall_profile": {"what": STALL_NOTE, "in_core": stalls_in, "out_of_core": stalls_out},
        "comparison_policies": policies,
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_kernel and gemm_bf16_dl_kernel (" + SAMPLING_NOTE + ")",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "launches_per_step": n_l * TIMER_STRIDE / max(args.steps, 1), "avg_launch_ms": ms_l / max(n_l, 1),
                     "flops_per_launch": fl_l / max(n_l, 1),
                     "traffic": profiled_traffic("".join("KSRrc"[a] for a in acts)) if args.config == 1 else None,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a plain copy; null when the "
                                     "committed counter summary was taken on another plan)"},
    }
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if args.config == 1 and not args.no_policies:
        out["bandwidth_bound_kernels"] = bandwidth_kernels(K, torch)
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(CPU_SAMPLE_BATCH if args.config == 1 else 1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
