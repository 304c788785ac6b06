#!/usr/bin/env python3
"""Throughput of the Virtual-Expert MoE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c5|c4]

Prefill workloads (c2, c3, c5): one "step" is one pass of the whole hot path
(route, importance, permute, expert FFN, combine) through every stacked MoE
layer of the workload, on synthetic inputs already resident in HBM.  The
default, c3, is the Switch-base-64 prefill shape (E=64, K=16 resident,
d_model=768, d_ff=3072, T=4096 tokens, 6 stacked layers with independent
weights, bf16), the shape the headline metric is quoted on.  Layer l+1 reads
layer l's output plus the residual stream, so the six layers' 906 MB of
resident weights are walked in turn and no layer's weights stay cache-resident
between uses.  `value` = T * layers / step time: tokens through a MoE layer per
second.

Decode workload (c4): one step is one decode step (T=32 tokens, one token per
stream) through `--decode-layers` layers; the resident set follows the
importance scores inside the timed region.  `--updates sync` (default): every
`period` (16) steps the scores are read back, the policy picks the new resident
set and the changed slots are reloaded from the expert bank before the next
step.  `--updates async`: the scores travel to the host behind the compute
stream, smoe_update_begin plans the changes and smoe_update_tick, called
between steps, loads one expert per spare slot on a second stream and switches
the maps when a load has arrived (amortized, asynchronous loading).  `--bank
pinned` keeps the bank in host memory, so loads cross PCIe.
`value` = T * layers * steps / time.

Prints ONE JSON line.  `roofline` is for the expert FFN's two grouped-GEMM
launches: their duration is measured live with HIP events attached to the two
product dispatches of one layer call per sampled step, in a second pass over
the same K steps right after the throughput pass (a dispatch that carries
events stalls the queue behind it, so the two cannot share a pass).
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload on
this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0      # MI355X dense bf16
PEAK_HBM_GBS = 8000.0

# HBM-side traffic of the dominant kernels is not measured live (it needs two rocprofv3 --pmc runs);
# `roofline.traffic` is read from the committed counter summary of the same command, and only if
# that summary names the kernel instances this run has just timed (smoe_describe_ffn).
PROFILE_FILES = {
    "c3": "profiles/grouped_gemm_bf16_c3_prefill_hbm_counters.txt",
    "c4": "profiles/decode_step_c4_hbm_counters.txt",
    "c5": "profiles/grouped_gemm_bf16_c5_prefill_hbm_counters.txt",
}


def stored_traffic(workload, kernels_now):
    """(bytes per launch or None, note).  The summary carries two machine-readable lines:
    `bench.roofline.kernels = <first> | <second>` and `bench.roofline.traffic_bytes_per_launch = <n>`."""
    path = os.path.join(ROOT, PROFILE_FILES.get(workload, ""))
    if not os.path.isfile(path):
        return None, "no counter summary for this workload under profiles/"
    keys = {}
    for line in open(path):
        if line.startswith("bench.roofline.") and "=" in line:
            k, v = line.split("=", 1)
            keys[k.strip()] = v.strip()
    kernels = keys.get("bench.roofline.kernels")
    if kernels != kernels_now:
        return None, f"{PROFILE_FILES[workload]} was collected with other kernels ({kernels}); re-collect it"
    try:
        return float(keys["bench.roofline.traffic_bytes_per_launch"]), PROFILE_FILES[workload]
    except (KeyError, ValueError):
        return None, f"{PROFILE_FILES[workload]} holds no traffic figure"


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def dev_t(a, dev):
    import numpy as np
    import torch
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)


def make_layer(b, wl, cfg, l, experts, dev, spare_slots=0, pinned_bank=False):
    """One bound layer with `experts` (bank order) uploaded; slots 0..K-1 hold the
    first K of them.  Returns (layer, device bank, host copies of layer data)."""
    import torch
    Wr = wl.router_weights(cfg, l)
    W1, W2 = wl.expert_bank(cfg, l, experts)
    lay = b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, cfg.T, cfg.dtype, router_w=torch.from_numpy(Wr),
                  device=dev, spare_slots=spare_slots)
    d1, d2 = dev_t(W1, dev), dev_t(W2, dev)
    en = lay.expert_norm_of(d1, d2)                  # |E_i| of the experts we hold; 1 elsewhere
    full = torch.ones(cfg.E, dtype=torch.float32, device=dev)
    full[torch.tensor(list(experts), device=dev)] = en
    lay.expert_norm.copy_(full)
    for s in range(cfg.K):
        lay.set_resident(s, int(experts[s]), d1[s], d2[s])
    torch.cuda.synchronize()
    if pinned_bank:                                  # the bank the updates read from lives in host memory
        import numpy as np
        d1 = torch.from_numpy(W1.view(np.int16)).pin_memory()
        d2 = torch.from_numpy(W2.view(np.int16)).pin_memory()
    return lay, (d1, d2), (Wr, W1, W2)


def per_call(args, cfg, layers, wl, dev, T, L):
    """Median duration of every hot call on its own (events on the caller's stream around one call,
    cycling through the layers so weights come from HBM as in the throughput run), with the
    algorithmic bytes / flops of the step and the fractions of the published peaks."""
    import numpy as np
    import torch
    xs = [dev_t(wl.hidden_states(cfg, l) if cfg.period == 0 else wl.decode_stream(cfg, 1)[0], dev) for l in range(L)]
    d, f, E, K = cfg.d_model, cfg.d_ff, cfg.E, cfg.K
    for lay, x in zip(layers, xs):                       # every buffer holds a consistent state
        lay.forward(x, T, accumulate=0, residual=x)
    torch.cuda.synchronize()
    act = float(np.mean([(lay.offsets[1:] > lay.offsets[:-1]).sum().item() for lay in layers]))
    calls = {   # name: (callable(layer, x), algorithmic bytes, flops)
        "smoe_route": (lambda lay, x: lay.route(x, T), T * d * 2 + 20 * T + E * d * 4, 2.0 * T * d * E),
        "smoe_importance": (lambda lay, x: lay.importance(T, 1), 12 * T + 12 * E, 0.0),
        "smoe_permute": (lambda lay, x: lay.permute(x, T), 2 * T * d * 2 + 12 * T, 0.0),
        "smoe_expert_ffn": (lambda lay, x: lay.expert_ffn(T), act * 2 * d * f * 2 + 2 * T * d * 2, 4.0 * T * d * f),
        "smoe_combine": (lambda lay, x: lay.combine(T, residual=x), 3 * T * d * 2 + 8 * T, 0.0),
        "smoe_forward": (lambda lay, x: lay.forward_fused(x, T, accumulate=1, residual=x),
                         act * 2 * d * f * 2 + 3 * T * d * 2 + 20 * T, 4.0 * T * d * f + 2.0 * T * d * E),
    }
    one = torch.zeros(1, device=dev)
    calls["(floor: event pair around nothing)"] = (lambda lay, x: None, 0, 0.0)
    calls["(floor: event pair around a one-element fill kernel)"] = (lambda lay, x: one.zero_(), 0, 0.0)
    out = {}
    n_warm, n_iter = 10, 100
    for name, (fn, nbytes, flops) in calls.items():
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_iter)]
        for i in range(n_warm + n_iter):
            lay, x = layers[i % L], xs[i % L]
            if i >= n_warm:
                evs[i - n_warm][0].record()
            fn(lay, x)
            if i >= n_warm:
                evs[i - n_warm][1].record()
        torch.cuda.synchronize()
        us = float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e3
        out[name] = {"us": round(us, 2), "bytes": int(nbytes), "GBs": round(nbytes / us / 1e3, 1),
                     "hbm_frac": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4),
                     "TFLOPs": round(flops / us / 1e6, 1), "mfma_frac": round(flops / us / 1e6 / PEAK_BF16_MFMA_TFLOPS, 4)}
    print(json.dumps({"per_call": out, "workload": cfg.name, "tokens": T, "layers_cycled": L,
                      "mean_active_slots": round(act, 2), "iterations": n_iter, "warmup": n_warm,
                      "note": "median of per-call event pairs; bytes = algorithmic (inputs, outputs and active slots' weights once)"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--decode-layers", type=int, default=1,
                    help="c4 only: independent layers per decode step (6 exceeds the 256 MB Infinity Cache)")
    ap.add_argument("--updates", default=None, choices=["device", "sync", "async", "none"],
                    help="c4 only: how the resident set follows the scores. device (default with the bank in device "
                         "memory): smoe_update_on_device, the update rule and the slot loads run on the GPU behind the "
                         "period's last step, no read-back; sync (default otherwise): the scores are read back, the host "
                         "applies the rule and reloads the changed slots before the next step; async: "
                         "smoe_update_begin/tick, loads on a second stream into a spare slot, spread over the following "
                         "steps; none: never updated")
    ap.add_argument("--policy", default="importance", choices=["importance", "count", "static", "lru"],
                    help="c4 only: what ranks the experts at an update. importance: the Eq. 1 score; count: tokens "
                         "per expert (the 'simple scheduling' ablation); static: the K experts of largest |E_i|, "
                         "never updated (magnitude pruning); lru: load-on-miss after every step, least recently "
                         "used slot evicted ('on demand' caching; --updates sync only)")
    ap.add_argument("--graph", action="store_true",
                    help="c4 only: record one decode step of all layers into a HIP graph (one graph per value of "
                         "the accumulate flag) and replay it per step; per-kernel events are not available then")
    ap.add_argument("--period", type=int, default=None, help="c4 only: update period in steps (default 16)")
    ap.add_argument("--hit-rate", action="store_true",
                    help="c4 only: also log, per step, how many tokens found their own top-1 expert resident "
                         "(two small device copies per step inside the timed region)")
    ap.add_argument("--bank", default="device", choices=["device", "pinned"],
                    help="c4 only: where the full expert bank lives (pinned = host memory read over PCIe)")
    ap.add_argument("--spare-slots", type=int, default=1, help="c4 --updates async: spare physical slots")
    ap.add_argument("--max-ahead", type=int, default=None,
                    help="c4 only: decode steps the host may enqueue ahead of the GPU, enforced with one event "
                         "per step (default: 2 with --updates async, where unbounded run-ahead would make "
                         "'between two steps' meaningless; otherwise no pacing -- the synchronous update's "
                         "score read-back already stops the host every period, and an event per step costs "
                         "the GPU queue about 14 us per step)")
    ap.add_argument("--per-call", action="store_true",
                    help="instead of the throughput run: median time of each of the five hot calls (and of "
                         "smoe_forward) over 100 iterations after 10 warm-ups, with the bytes and flops each moves")
    ap.add_argument("--layers", type=int, default=None,
                    help="prefill workloads: number of stacked layers (default: the workload's own; 1 keeps one "
                         "layer's weights cache-resident between steps, a tuning aid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-calls", action="store_true",
                    help="drive the layer through the five per-step calls instead of smoe_forward")
    ap.add_argument("--no-events", action="store_true",
                    help="skip the second, instrumented pass (no roofline)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_2308_15030_amd import binding as b
    from paper_2308_15030_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.workload]
    decode = cfg.period > 0
    if decode and args.period:
        cfg = cfg.scaled(period=max(1, args.period))
    steps = args.steps if args.steps is not None else (cfg.steps if decode else 50)
    warmup = args.warmup if args.warmup is not None else (16 if decode else 10)
    T = cfg.T
    L = args.decode_layers if decode else (args.layers or cfg.layers)
    s2e0, e2s0 = wl.initial_resident(cfg)
    use_events = not args.no_events

    t_setup = time.time()
    experts = list(range(cfg.E)) if decode else list(s2e0)
    layers, banks, host0 = [], [], None
    for l in range(L):
        lay, bank, host = make_layer(b, wl, cfg, l, experts, dev,
                                     spare_slots=args.spare_slots if (decode and args.updates == "async") else 0,
                                     pinned_bank=decode and args.bank == "pinned")
        layers.append(lay)
        banks.append(bank if decode else None)       # prefill never reloads: free the bank copy
        if l == 0:
            host0 = host
    print(f"[bench] {cfg.name}: {L} layer(s) set up in {time.time() - t_setup:.1f}s", file=sys.stderr, flush=True)

    def fwd(lay):
        return lay.forward if args.separate_calls else lay.forward_fused

    if args.per_call:
        per_call(args, cfg, layers, wl, dev, T, L)
        return

    # Two passes over the same K steps.  The first is the throughput measurement: nothing but the
    # hot path between the two synchronisations.  The second repeats the K steps with per-kernel
    # events riding on the two grouped-GEMM dispatches of ONE layer call per sampled step (layer
    # k % L at step k; decode samples every 4th step); each pair reads the start and end of that
    # kernel's execution and feeds `roofline`.  A dispatch that carries events also carries a
    # completion signal and stalls the queue behind it (5 % at c3, 20 % on the decode step), so
    # the two measurements cannot share a pass.
    ev_stride = 4 if decode else 1
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)] if use_events else []
    ev_used = []
    active_log = []

    if not decode:
        x_host = wl.hidden_states(cfg, 0)
        x0 = dev_t(x_host, dev)

        def step(k=None):
            x = x0
            for l, lay in enumerate(layers):
                if k is not None and use_events and l == k % L:
                    b.smoe_set_profile_events(lay.handle, *evs[k])
                    ev_used.append(k)
                x = fwd(lay)(x, T, accumulate=1, residual=x)         # residual stream: next layer reads x + MoE(x)
            return x

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if use_events:
            for k in range(steps):
                step(k)
            torch.cuda.synchronize()
    else:
        xs_host = wl.decode_stream(cfg, warmup + steps)
        xs = dev_t(xs_host.reshape(-1, cfg.d_model), dev).view(warmup + steps, T, cfg.d_model)

        if args.updates is None:                     # the rule on the GPU when the bank is there, else on the host
            args.updates = "device" if (args.bank == "device" and args.policy in ("importance", "count")) else "sync"
        if args.policy == "lru" and args.updates != "sync":
            sys.exit("bench.py: --policy lru needs --updates sync")
        if args.policy == "static":                  # the K experts of largest |E_i|, chosen once by the library's policy unit
            args.updates = "none"
            for lay, (d1, d2) in zip(layers, banks):
                for sl, ex in lay.select_resident(lay.policy_rank(b.SMOE_POLICY_MAGNITUDE)):
                    lay.set_resident(sl, ex, d1[ex], d2[ex])
            torch.cuda.synchronize()
        load_stream = torch.cuda.Stream()
        oe_log = torch.zeros(steps, T, dtype=torch.int32, device=dev) if args.hit_rate else None
        e2s_log = np.zeros((steps, cfg.E), np.int32)

        graphs = {}
        x_in = torch.empty(T, cfg.d_model, dtype=xs.dtype, device=dev)
        if args.graph:
            use_events = False
            side = torch.cuda.Stream()
            for acc in (0, 1):                                 # eager once (one-off set-up work), then capture
                x = x_in
                for lay in layers:
                    x = fwd(lay)(x, T, accumulate=acc, residual=x)
            torch.cuda.synchronize()
            side.wait_stream(torch.cuda.current_stream())
            for acc in (0, 1):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        x = x_in
                        for lay in layers:
                            x = fwd(lay)(x, T, accumulate=acc, residual=x)
                graphs[acc] = g
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()

        def rank_tensor(lay):                        # asynchronous path: the ranking numbers as a device tensor
            return lay.count.to(torch.float32) if args.policy == "count" else lay.score
        lib_policy = b.SMOE_POLICY_COUNT if args.policy == "count" else b.SMOE_POLICY_IMPORTANCE
        n_samples = (steps + ev_stride - 1) // ev_stride
        offs_log = torch.zeros(n_samples, cfg.K + 1, dtype=torch.int32, device=dev)   # offsets of the timed launches
        score_host = [torch.zeros(cfg.E, dtype=torch.float32).pin_memory() for _ in layers]
        score_ev = [torch.cuda.Event() for _ in layers]
        score_due = [False] * L
        ahead = args.max_ahead if args.max_ahead is not None else (2 if args.updates == "async" else 0)
        ahead = max(0, ahead)
        step_done = [torch.cuda.Event() for _ in range(ahead + 1)]

        def run(first, n, timed, instrument=False):
            swaps = 0
            for i in range(n):
                sidx = first + i
                if args.updates == "async":                  # between two steps; never waits for the GPU
                    for l, (lay, (b1, b2)) in enumerate(zip(layers, banks)):
                        swaps += lay.update_tick(b1, b2, load_stream)
                        if score_due[l] and score_ev[l].query():
                            lay.update_begin(score_host[l].numpy())
                            score_due[l] = False
                x = xs[sidx]
                if args.graph:
                    x_in.copy_(x, non_blocking=True)
                    graphs[0 if sidx % cfg.period == 0 else 1].replay()
                for l, lay in enumerate(layers if not args.graph else []):
                    sampled = instrument and i % ev_stride == 0 and l == (i // ev_stride) % L
                    if sampled and use_events:
                        b.smoe_set_profile_events(lay.handle, *evs[i])
                        ev_used.append(i)
                    x = fwd(lay)(x, T, accumulate=0 if sidx % cfg.period == 0 else 1, residual=x)
                    if sampled:
                        offs_log[i // ev_stride].copy_(lay.offsets, non_blocking=True)
                    if timed and args.hit_rate and l == 0:
                        oe_log[i].copy_(lay.orig_expert, non_blocking=True)
                        e2s_log[i] = lay.maps()[1]
                    if args.policy == "lru":         # load on miss: the library's plan (least recently used slots go)
                        d1, d2 = banks[l]
                        for sl, ex in lay.on_demand_plan(T):
                            lay.set_resident(sl, ex, d1[ex], d2[ex])
                            swaps += 1
                if ahead > 0:
                    step_done[i % (ahead + 1)].record()
                    if i >= ahead:
                        step_done[(i - ahead) % (ahead + 1)].synchronize()
                if (sidx + 1) % cfg.period == 0 and args.updates != "none" and args.policy != "lru":
                    for l, (lay, (d1, d2)) in enumerate(zip(layers, banks)):
                        if args.updates == "async":          # scores travel to the host behind the compute stream
                            score_host[l].copy_(rank_tensor(lay), non_blocking=True)
                            score_ev[l].record()
                            score_due[l] = True
                        elif args.updates == "device":       # rule and loads on the GPU, nothing comes back
                            before = lay.maps()[0] if not timed else None   # (untimed passes count the changes)
                            lay.update_on_device(d1, d2, score=rank_tensor(lay))
                            if not timed:
                                swaps += int((lay.maps()[0] != before).sum())
                        else:
                            score = lay.policy_rank(lib_policy)      # the one host read-back per period
                            for sl, ex in lay.select_resident(score):
                                lay.set_resident(sl, ex, d1[ex], d2[ex])
                                swaps += 1
            torch.cuda.synchronize()
            return swaps

        run(0, warmup, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        swaps = run(warmup, steps, True)
        dt = time.perf_counter() - t0
        if use_events:          # the same steps again, instrumented (the resident set carries on from the first pass)
            swaps2 = run(warmup, steps, False, instrument=True)
            if args.updates == "device":
                swaps = swaps2      # counted where reading the maps back costs nothing that is timed
        active_log = (offs_log[:, 1:] > offs_log[:, :-1]).sum(dim=1).cpu().numpy().tolist()
        hit_rate = None
        if args.hit_rate:
            oe = oe_log.cpu().numpy()
            hit_rate = float(np.mean([(e2s_log[i][oe[i]] >= 0).mean() for i in range(steps)]))

    ms_per_step = dt / steps * 1e3
    value = T * L / (dt / steps)

    roof = None
    kernels_now = b.smoe_describe_ffn(layers[0].handle, T, not args.separate_calls)
    if use_events:
        g1 = np.array([evs[i][0].elapsed_time(evs[i][1]) for i in ev_used]) * 1e-3
        g2 = np.array([evs[i][2].elapsed_time(evs[i][3]) for i in ev_used]) * 1e-3
        avg = (g1.mean() + g2.mean()) / 2.0                    # mean duration of one grouped-GEMM launch
        if not decode:
            flops = 2.0 * T * cfg.d_model * cfg.d_ff           # per launch; two launches per FFN
            achieved = flops / avg / 1e12
            # algorithmic bytes per launch: the resident weights of one matrix per slot once, the
            # tokens in and the layer output out (half of each per launch); the hidden activations'
            # round trip through memory is the kernel's own doing and is listed separately
            bytes_launch = 2.0 * (cfg.K * cfg.d_model * cfg.d_ff + T * cfg.d_model)
            bytes_with_h = bytes_launch + 2.0 * T * cfg.d_ff
            default_run = (not args.separate_calls and args.layers is None)
            traffic, traffic_src = stored_traffic(args.workload, kernels_now) if default_run else (None, "non-default run")
            roof = {"bound": "mfma", "kernel": kernels_now + " (mean of the FFN's two launches)",
                    "achieved": round(achieved, 2), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_MFMA_TFLOPS, 4),
                    "traffic": traffic, "traffic_source": traffic_src,
                    "us_per_launch": round(avg * 1e6, 2), "us_gemm1": round(g1.mean() * 1e6, 2),
                    "us_gemm2": round(g2.mean() * 1e6, 2), "launches_timed": 2 * len(ev_used), "flop_per_launch": flops,
                    "hbm_bytes_per_launch_algorithmic": bytes_launch,
                    "hbm_bytes_per_launch_with_hidden_round_trip": bytes_with_h,
                    "hbm_GBs": round(bytes_launch / avg / 1e9, 1),
                    "hbm_frac": round(bytes_launch / avg / 1e9 / PEAK_HBM_GBS, 4)}
        else:
            act = float(np.mean(active_log)) if active_log else float(cfg.K)
            default_c4 = (args.workload == "c4" and args.updates == "device" and args.bank == "device"
                          and args.policy == "importance" and args.period is None and not args.separate_calls
                          and args.decode_layers == 1)
            bytes_launch = 2.0 * act * cfg.d_model * cfg.d_ff  # one weight matrix of every active slot
            achieved = bytes_launch / avg / 1e9
            traffic, traffic_src = stored_traffic(args.workload, kernels_now) if default_c4 else (None, "non-default run")
            roof = {"bound": "hbm", "kernel": kernels_now + " (mean of the FFN's two launches)",
                    "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                    "us_per_launch": round(avg * 1e6, 2), "us_gemm1": round(g1.mean() * 1e6, 2),
                    "us_gemm2": round(g2.mean() * 1e6, 2), "launches_timed": 2 * len(ev_used),
                    "mean_active_slots": round(act, 2),
                    "hbm_bytes_per_launch_algorithmic": bytes_launch}
            if kernels_now.startswith("decode_first_kernel"):
                # the first launch does not wait for the routing: it streams the first matrix of all K slots
                streamed = 2.0 * cfg.K * cfg.d_model * cfg.d_ff
                roof.update(first_launch_streams_all_slots=True, first_launch_bytes_streamed=streamed,
                            first_launch_streamed_GBs=round(streamed / g1.mean() / 1e9, 1),
                            second_launch_GBs=round(bytes_launch / g2.mean() / 1e9, 1))

    if roof is not None:
        # What a launch that only READS one product's weights costs on this GPU: the library's plain
        # streaming kernel over the K slots of each layer in turn (first matrices, then second), same
        # cache state as the step itself (one layer stays in the Infinity Cache, a stack does not).
        reps = 10
        lay0 = layers[0]
        for which in (0, 1):                                   # warm-up
            for lay in layers:
                b.smoe_profile_stream_read(lay.handle, which)
        b.smoe_profile_begin(lay0.handle)
        for _ in range(reps):
            for lay in layers:
                for which in (0, 1):
                    b.smoe_profile_stream_read(lay.handle, which)
        us = b.smoe_profile_end(lay0.handle) / (reps * len(layers) * 2)
        nbytes = 2.0 * cfg.K * cfg.d_model * cfg.d_ff
        roof["plain_read_of_all_slots"] = {"bytes_per_launch": nbytes, "us_per_launch": round(us, 2),
                                           "GBs": round(nbytes / us / 1e3, 1),
                                           "frac_of_hbm_peak": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4),
                                           "note": "smoe_profile_stream_read back to back: the time of a launch that moves one "
                                                   "product's K weight matrices and does no arithmetic"}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Wr, W1, W2 = host0
        if not decode:
            reps = 20 if args.workload != "c5" else 2       # about 10 s of host work
            t1 = time.perf_counter()
            for _ in range(reps):
                oracle.layer_forward(x_host, Wr, W1[:cfg.K], W2[:cfg.K], e2s0)
            tc = time.perf_counter() - t1
            cpu = {"value": round(T * reps / tc, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                   "cpu_model": cpu_model(), "kind": "oracle", "sample": f"{reps} x one full layer (layer 0) of {cfg.name}, all {T} tokens "
                                               f"each, {tc:.2f}s wall"}
        else:
            n = min(steps, 256)
            t1 = time.perf_counter()
            for i in range(n):
                oracle.layer_forward(xs_host[i], Wr, W1[:cfg.K], W2[:cfg.K], e2s0)
            tc = time.perf_counter() - t1
            cpu = {"value": round(T * n / tc, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                   "cpu_model": cpu_model(), "kind": "oracle", "sample": f"{n} decode steps of layer 0 of {cfg.name} on the initial "
                                               f"resident set (no updates), {tc:.2f}s wall"}

    config = {"workload": cfg.name, "E": cfg.E, "K": cfg.K, "d_model": cfg.d_model, "d_ff": cfg.d_ff,
              "tokens": T, "layers": L,
              "entry": "five separate calls" if args.separate_calls else "smoe_forward (one call: 4 launches for prefill, 2 for a decode-sized batch)",
              "step": "route+importance+permute+expert_ffn+combine over all layers"}
    if decode:
        config.update(update_period=cfg.period, experts_swapped=swaps, updates=args.updates, bank=args.bank,
                      host_steps_ahead=(ahead if ahead > 0 else "unpaced"), policy=args.policy, hip_graph=bool(args.graph),
                      hit_rate=None if hit_rate is None else round(hit_rate, 4),
                      bytes_loaded_per_step=round(swaps * 2.0 * cfg.d_model * cfg.d_ff * 2 / steps, 1),
                      spare_slots=args.spare_slots if args.updates == "async" else 0,
                      step="one decode step: route+importance+permute+expert_ffn+combine, plus score "
                           "read-back, policy and slot reloads every update_period steps")
    out = {
        "metric": "MoE-layer tokens/sec (Virtual-Expert top-1 layer forward)", "value": round(value, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": config, "us_per_layer": round(ms_per_step * 1e3 / L, 2),
        "roofline": roof, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
