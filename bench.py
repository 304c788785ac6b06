#!/usr/bin/env python3
"""Throughput of the Virtual-Expert MoE layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

One "step" is one pass of the whole hot path (route, importance, permute,
expert FFN, combine) through every stacked MoE layer of the workload, on
synthetic inputs already resident in HBM.  The default workload is the
Switch-base-64 prefill shape (E=64, K=16 resident, d_model=768, d_ff=3072,
T=4096 tokens, 6 stacked layers with independent weights, bf16), the shape the
headline metric is quoted on.  Layer l+1 reads layer l's output plus the
residual stream, so the six layers' 906 MB of resident weights are walked in
turn and no layer's weights stay cache-resident between uses.

Prints ONE JSON line.  `value` = T * layers / step time (tokens through a MoE
layer per second).  `roofline` is for the expert FFN's grouped-GEMM kernels:
their duration is measured live with HIP events recorded on the launch stream
around each of the two products of every smoe_expert_ffn call of the timed
region.  `cpu_baseline` times the CPU oracle on one full layer of the same
workload on this machine's host cores.
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true",
                    help="do not record per-kernel events inside the timed region")
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
    T, L = cfg.T, cfg.layers
    s2e, e2s = wl.initial_resident(cfg)

    def dev_t(a):
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

    t_setup = time.time()
    layers = []
    host_layer0 = None
    for l in range(L):
        Wr = wl.router_weights(cfg, l)
        W1, W2 = wl.expert_bank(cfg, l, s2e)
        if l == 0:
            host_layer0 = (Wr, W1, W2)
        lay = b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, T, cfg.dtype, router_w=torch.from_numpy(Wr),
                      device=dev)
        d1, d2 = dev_t(W1), dev_t(W2)
        en = lay.expert_norm_of(d1, d2)                  # |E_i| of the resident experts; 1 elsewhere
        full = torch.ones(cfg.E, dtype=torch.float32, device=dev)
        full[torch.from_numpy(s2e).to(dev).long()] = en
        lay.expert_norm.copy_(full)
        for s, e in enumerate(s2e):
            lay.set_resident(s, int(e), d1[s], d2[s])
        torch.cuda.synchronize()
        del d1, d2
        layers.append(lay)
    x_host = wl.hidden_states(cfg, 0)
    x0 = dev_t(x_host)
    torch.cuda.synchronize()
    print(f"[bench] {cfg.name}: {L} layers set up in {time.time() - t_setup:.1f}s", file=sys.stderr, flush=True)

    use_events = not args.no_events
    n_ev = args.steps * L
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)] if use_events else []

    def step(ev_base=None):
        x = x0
        for l, lay in enumerate(layers):
            if ev_base is not None:
                b.smoe_set_profile_events(lay.handle, *evs[ev_base + l])
            # residual stream: the next layer reads x + MoE(x)
            x = lay.forward(x, T, accumulate=1, residual=x)
        return x

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k * L if use_events else None)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    value = T * L / (dt / args.steps)

    flops_per_gemm = 2.0 * T * cfg.d_model * cfg.d_ff          # per launch; two launches per FFN
    roof = None
    if use_events:
        g1 = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e-3
        g2 = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e-3
        avg = (g1.mean() + g2.mean()) / 2.0                    # mean duration of one grouped-GEMM launch
        achieved = flops_per_gemm / avg / 1e12
        roof = {"bound": "mfma", "kernel": "grouped_gemm_bf16 (both FFN products)",
                "achieved": round(achieved, 2), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_MFMA_TFLOPS, 4), "traffic": None,
                "us_gemm1": round(g1.mean() * 1e6, 2), "us_gemm2": round(g2.mean() * 1e6, 2),
                "flop_per_launch": flops_per_gemm}
        # the same two launches against the HBM roof: resident weights once, x in, h out+in, y out
        bytes_ffn = 2.0 * (cfg.K * 2 * cfg.d_model * cfg.d_ff + 2 * T * cfg.d_model + 2 * T * cfg.d_ff)
        roof["hbm_GBs_ffn"] = round(bytes_ffn / (g1.mean() + g2.mean()) / 1e9, 1)
        roof["hbm_frac_ffn"] = round(roof["hbm_GBs_ffn"] / PEAK_HBM_GBS, 4)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Wr, W1, W2 = host_layer0
        t1 = time.perf_counter()
        oracle.layer_forward(x_host, Wr, W1, W2, e2s)
        tc = time.perf_counter() - t1
        cpu = {"value": round(T / tc, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"one full layer (layer 0) of {cfg.name}, all {T} tokens, "
                                           f"{tc:.2f}s wall"}

    out = {
        "metric": "MoE-layer tokens/sec (Virtual-Expert top-1 layer forward)", "value": round(value, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "E": cfg.E, "K": cfg.K, "d_model": cfg.d_model,
                   "d_ff": cfg.d_ff, "tokens": T, "layers": L,
                   "step": "route+importance+permute+expert_ffn+combine over all layers"},
        "us_per_layer": round(ms_per_step * 1e3 / L, 2),
        "roofline": roof, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
