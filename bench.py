#!/usr/bin/env python3
"""Benchmark of the self-speculative decoding hot path on one MI355X.

A "step" is one full ConfLayers generation cycle on the Llama-2-7B-shaped bf16 workload with the
search active: k draft steps with the current skip set, one verification pass over k+1 rows,
greedy acceptance, the per-layer confidence of the cycle's first verify row, and the host-side
search check (which may install a new skip set).  Vanilla decoding with the same library is
timed alongside.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
# HBM bytes per launch of the draft gate/up GEMV at Llama-2-7B shape: rocprofv3 FETCH_SIZE + WRITE_SIZE per
# dispatch, scaled by the factors a known-size read / copy kernel gives (FETCH_SIZE x2.000, WRITE_SIZE x1.000);
# the run and the arithmetic are in profiles/kernel_bench_llama7b_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {"llama7b": 180.76e6}


def layer_bytes(s):
    B = s.bytes_per_weight()
    return B * (2 * s.d_model * s.n_heads * s.head_dim + 2 * s.d_model * s.d_kv + 3 * s.d_model * s.d_ffn) + 2 * s.d_model * 4


def draft_step_bytes(s, n_exec_layers, pos):
    """Algorithmic HBM bytes of one single-row forward at cache position pos with n_exec_layers layers run."""
    B = s.bytes_per_weight()
    kv = 2 * (pos + 1) * s.d_kv * B + 2 * s.d_kv * B
    return n_exec_layers * (layer_bytes(s) + kv) + B * s.vocab * s.d_model + s.d_model * 4 + s.d_model * B


def verify_bytes(s, pos, rows):
    B = s.bytes_per_weight()
    kv = 2 * (pos + rows) * s.d_kv * B + 2 * rows * s.d_kv * B
    return s.n_layers * (layer_bytes(s) + kv) + B * s.vocab * s.d_model + s.d_model * 4 + rows * s.d_model * B


def gateup_kernel_bytes(s):
    """Algorithmic bytes of one launch of the draft path's gate/up GEMV: both weight matrices once, the
    residual vector and gain in, the activation vector out."""
    return 2 * s.d_ffn * s.d_model * s.bytes_per_weight() + 2 * s.d_model * 4 + s.d_ffn * 4


def cpu_baseline(shape, weights_gpu, prompt, k, mask, n_prompt=8, n_cycles=8):
    """Times the CPU oracle (as it stands) on a bounded sample of the same workload."""
    import numpy as np
    from oracle import OracleModel, OracleSSD
    w_cpu = {}
    for key, v in weights_gpu.items():
        if key.startswith("_"):
            continue
        w_cpu[key] = [t.cpu() for t in v] if isinstance(v, list) else v.cpu()
    m = OracleModel(shape, w_cpu, n_prompt + n_cycles * (k + 1) + 4)
    o = OracleSSD(m)
    o.prefill(prompt[:n_prompt])
    n0 = o.n
    t0 = time.perf_counter()
    for _ in range(n_cycles):
        d = o.draft(mask, k)
        y = o.verify(d)
        o.accept(d, y)
    dt = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    threads = min(cores, int(omp)) if omp and omp.isdigit() else cores
    return {"value": (o.n - n0) / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d-token prompt, %d SSD cycles (k=%d, %d of %d layers skipped), fp64 oracle, %.1f s"
                      % (n_prompt, n_cycles, k, int(np.sum(mask)), shape.n_layers, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="reduced depth (debugging only; marks the result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pack", action="store_true", help="keep the weights as separately allocated tensors")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (batch-1 decoding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2604_14612_amd as ssd
    from paper_2604_14612_amd.binding import KERNEL_IDS
    from synth import WORKLOADS, make_prompt, make_weights, reduced_depth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    wl = WORKLOADS[args.workload]
    shape = wl.shape if args.layers is None else reduced_depth(wl.shape, args.layers)
    k = args.k or wl.k
    K, W = args.steps, args.warmup
    L = shape.n_layers

    weights = make_weights(shape, wl.seed, device="cuda")
    w_bytes = sum(t.numel() * t.element_size() for v in weights.values() for t in (v if isinstance(v, list) else [v]))
    # Layout of the weights in HBM: the library takes the pointers it is given, and how the matrices are placed
    # matters by a few per cent (one arena in forward order is 2-3 % faster at the 7B shape, equal at the 13B
    # shape), so both are timed on a few decode steps and the faster one is kept.
    layout, packed = "separate", None
    if not args.no_pack and w_bytes < 100e9:
        def probe(wts):
            c = ssd.Context(shape, wts, wl.prompt_len + (W + K + 4) * (k + 1) + 16, max_k=k)
            c.ssd_prefill(make_prompt(shape.vocab, wl.prompt_len, wl.seed).tolist())
            for _ in range(4):
                c.ssd_decode()
            torch.cuda.synchronize(); t0 = time.perf_counter()
            for _ in range(24):
                c.ssd_decode()
            torch.cuda.synchronize(); dt = time.perf_counter() - t0
            c.close()
            return dt
        t_sep = probe(weights)
        packed = ssd.pack_weights(weights)
        t_pack = probe(packed)
        print("layout probe: separate %.2f ms, one arena %.2f ms per decode step" % (t_sep / 24 * 1e3, t_pack / 24 * 1e3),
              file=sys.stderr)
        if t_pack < t_sep:
            weights, packed, layout = packed, weights, "one arena"
    prompt = make_prompt(shape.vocab, wl.prompt_len, wl.seed).tolist()
    max_seq = wl.prompt_len + (W + K + 4) * (k + 1) + 16
    ctx = ssd.Context(shape, weights, max_seq, max_k=k)
    # the layout not chosen stays allocated until the process ends: releasing tens of GB right before the timed
    # regions slowed them by 2-5 % (the driver is still unmapping while the kernels run)
    sync = torch.cuda.synchronize

    # ---- vanilla decoding with the same library ----------------------------------------------------
    ctx.ssd_prefill(prompt)
    for _ in range(W):
        ctx.ssd_decode()
    n_van = min(K, 64)
    sync(); t0 = time.perf_counter()
    for _ in range(n_van):
        ctx.ssd_decode()
    sync(); t_van = time.perf_counter() - t0
    van_tps = n_van / t_van
    van_pos = wl.prompt_len + W + n_van // 2
    van_bytes = draft_step_bytes(shape, L, van_pos)

    # ---- SSD cycles with the search active ----------------------------------------------------------
    sel = ssd.select_defaults(protect_ends=int(wl.protect_ends), max_ratio=wl.max_skip_ratio)

    def run_cycles(n_cycles, search, timing=None):
        tokens = 0
        for _ in range(n_cycles):
            mask = search.mask()
            pos = ctx.ssd_get_stats()["n_tokens"] - 1
            ta = time.perf_counter()
            d = ctx.ssd_draft_step(mask, k)
            tb = time.perf_counter()
            y = ctx.ssd_verify(d)
            tc = time.perf_counter()
            a, _ = ctx.ssd_accept(d, y)
            conf = ctx.ssd_layer_confidence(0, 1)[0] if search.active else None
            search.observe(a, conf)
            td = time.perf_counter()
            tokens += a + 1
            if timing is not None:
                n_exec = L - int(mask.sum())
                timing["draft_s"] += tb - ta
                timing["draft_bytes"] += sum(draft_step_bytes(shape, n_exec, pos + i) for i in range(k))
                timing["verify_s"] += tc - tb
                timing["verify_bytes"] += verify_bytes(shape, pos, k + 1)
                timing["other_s"] += td - tc
                timing["accepted"] += a
                timing["skipped"] += int(mask.sum())
        return tokens

    ctx.ssd_reset()
    ctx.ssd_prefill(prompt)
    search = ssd.Search(L, ssd.search_defaults(), sel)
    run_cycles(W, search)
    timing = {"draft_s": 0.0, "draft_bytes": 0, "verify_s": 0.0, "verify_bytes": 0, "other_s": 0.0,
              "accepted": 0, "skipped": 0}
    sync(); t0 = time.perf_counter()
    tokens = run_cycles(K, search, timing)
    sync(); t_ssd = time.perf_counter() - t0
    ssd_tps = tokens / t_ssd
    rounds, best = search.status()

    # ---- roofline pass: same cycles, every launch of the dominant kernel bracketed by HIP events ------
    ctx.ssd_reset()
    ctx.ssd_prefill(prompt)
    search2 = ssd.Search(L, ssd.search_defaults(), sel)
    run_cycles(W, search2)
    ctx.ssd_profile_select(KERNEL_IDS["gemv_gateup"])
    run_cycles(min(K, 16), search2)
    n_launch, ms_total = ctx.ssd_profile_read()
    ctx.ssd_profile_select(-1)
    kern_ms = ms_total / max(n_launch, 1)
    kern_bytes = gateup_kernel_bytes(shape)
    achieved = kern_bytes / (kern_ms * 1e-3) / 1e9

    probe_ms = ssd.ssd_hbm_read_probe(weights["lm_head"], iters=20)
    probe_gbps = weights["lm_head"].numel() * weights["lm_head"].element_size() / (probe_ms * 1e-3) / 1e9

    draft_gbps = timing["draft_bytes"] / timing["draft_s"] / 1e9
    verify_gbps = timing["verify_bytes"] / timing["verify_s"] / 1e9
    out = {
        "metric": "decode tokens/s batch 1, SSD vs vanilla, 7B-shape bf16; achieved HBM GB/s",
        "value": ssd_tps, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": t_ssd / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp16": "f16", "fp32": "f32"}[shape.dtype], "data": "synthetic",
        "config": {"workload": "%s: %d layers, d_model %d, %d/%d heads, FFN %d, vocab %d, prompt %d, k=%d, "
                               "ConfLayers search active (interval 30), random-init weights"
                               % (wl.name, L, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn,
                                  shape.vocab, wl.prompt_len, k),
                   "reduced_depth": args.layers is not None, "weight_layout": layout},
        "vanilla_tokens_per_s": van_tps,
        "vanilla_GBps": van_bytes * van_tps / 1e9,
        "vanilla_frac_of_hbm_peak": van_bytes * van_tps / 1e9 / HBM_PEAK_GBPS,
        "ssd_over_vanilla": ssd_tps / van_tps,
        "acceptance": {"alpha": timing["accepted"] / (K * k), "mean_accepted_M": timing["accepted"] / K,
                       "skip_rate_beta": timing["skipped"] / (K * L), "search_rounds": rounds,
                       "search_best_score": best},
        "draft_step": {"ms": timing["draft_s"] / (K * k) * 1e3, "GBps": draft_gbps,
                       "frac_of_hbm_peak": draft_gbps / HBM_PEAK_GBPS},
        "verify": {"ms": timing["verify_s"] / K * 1e3, "GBps": verify_gbps,
                   "frac_of_hbm_peak": verify_gbps / HBM_PEAK_GBPS},
        "confidence_and_search_ms_per_cycle": timing["other_s"] / K * 1e3,
        "hbm_read_probe_GBps": probe_gbps,
        "roofline": {"bound": "hbm", "kernel": "gemv_kernel<%s, SWIGLU> (draft gate/up GEMV)" % shape.dtype,
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name) if args.layers is None else None, "avg_launch_us": kern_ms * 1e3, "launches_timed": n_launch,
                     "algorithmic_bytes_per_launch": kern_bytes},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, weights, prompt, k, search.mask())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
