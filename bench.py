#!/usr/bin/env python3
"""Benchmark of the KVCompose compression pass on one MI355X.

One "step" is one kvc_compress call (score -> head-rank -> composite -> global
select -> gather) over a synthetic Llama-3-8B-shaped bf16 cache that is already
resident in HBM.  Prints ONE JSON line: throughput in context tokens per second,
the roofline figures of the longest-running kernel (from HIP events the library
records on the launch stream) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "context tokens compressed/sec at Llama-3-8B shape, L=128k"
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBPS = 8000.0
PEAK_FP32_VALU_TFLOPS = 157.3   # 256 CUs x 4 SIMDs x 64 lanes x 2 flops x 2.4 GHz, doubled by packed issue
# HBM bytes per layer of the score kernels at the config-2 layer shape (32/8 heads, d=128,
# N=131072, M=64), from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by the copy-probe factors
# (2.000 / 1.000); source: profiles/score_mfma_config2_hbm_traffic.md
MEASURED_TRAFFIC_BYTES = {"score_mfma<stats>": 274.3e6, "score_mfma<emit>": 277.5e6}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def generate_and_upload(cfg, seed, lens, torch, workers):
    """Per-layer generation on host threads; each layer is uploaded as soon as
    it is ready so the host never holds more than `workers` layers."""
    import workloads as wl

    def to_dev(arr):
        if arr.dtype == np.uint16:
            return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(arr).cuda()

    def one_layer(l):
        qs, ks, vs = [], [], []
        for b in range(cfg.batch):
            q, k, v = wl.make_layer(cfg, seed, b, l, int(lens[b]))
            qs.append(q); ks.append(k); vs.append(v)
        return l, np.stack(qs), np.concatenate(ks, axis=1), np.concatenate(vs, axis=1)

    q_dev, k_dev, v_dev = [None] * cfg.layers, [None] * cfg.layers, [None] * cfg.layers
    t0 = time.time()
    with cf.ThreadPoolExecutor(max_workers=workers) as pool:
        futs = [pool.submit(one_layer, l) for l in range(cfg.layers)]
        for done, fut in enumerate(cf.as_completed(futs)):
            l, q, k, v = fut.result()
            q_dev[l], k_dev[l], v_dev[l] = to_dev(q), to_dev(k), to_dev(v)
            del q, k, v
            if (done + 1) % 8 == 0 or done + 1 == cfg.layers:
                log(f"generated+uploaded {done + 1}/{cfg.layers} layers ({time.time() - t0:.0f}s)")
    return q_dev, k_dev, v_dev


def cpu_baseline(cfg, seed, n, sample_layers, time_budget_s=30.0):
    """The oracle as it stands, on a bounded sample (the first `sample_layers`
    layers at full context length), scaled to the whole pass."""
    import workloads as wl
    from oracle import kvc_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    qs, ks, vs = [], [], []
    for l in range(sample_layers):
        q, k, v = wl.make_layer(cfg, seed, 0, l, n)
        qs.append(q); ks.append(k); vs.append(v)
    budget = wl.budget_for(cfg, n) * sample_layers // cfg.layers
    t0 = time.time()
    orc.compress(qs, ks, vs, budget)
    dt = time.time() - t0
    full = dt * cfg.layers / sample_layers
    return {
        "value": n / full, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{sample_layers} of {cfg.layers} layers at full N={n} (all stages), "
                  f"{dt:.1f}s measured, scaled by {cfg.layers}/{sample_layers}",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload id (2 = headline)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--n", type=int, default=None, help="override context length (debug)")
    ap.add_argument("--layers", type=int, default=None, help="override layer count (debug)")
    ap.add_argument("--batch", type=int, default=None, help="override number of sequences (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=8)
    ap.add_argument("--workers", type=int, default=min(16, os.cpu_count() or 1))
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MB",
                    help="only run the library's plain copy kernel on MB MiB (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; this build uses no second GPU (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2509_05165_amd as kv
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_probe:
        nbytes = args.copy_probe << 20
        src = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
        dst = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            kv.kvc_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes,
                              torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert bool((dst == 1).all())
        print(json.dumps({"copy_probe_bytes_read": nbytes, "copy_probe_bytes_written": nbytes,
                          "launches": 3}))
        return
    over = {}
    if args.n:
        over["n"] = args.n
    if args.layers:
        over["layers"] = args.layers
    if args.batch:
        over["batch"] = args.batch
    cfg = wl.get_config(args.config, **over)
    lens = wl.seq_lens(cfg, args.seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    total, max_n = int(cu[-1]), int(lens.max())
    budgets = [wl.budget_for(cfg, int(n)) for n in lens]
    tb = sum(budgets)
    log(f"workload {cfg.name}: batch={cfg.batch} layers={cfg.layers} hq/hkv={cfg.hq}/{cfg.hkv} "
        f"d={cfg.head_dim} N={lens.tolist()} M={cfg.window} dtype={cfg.dtype} budget={budgets}")

    q_dev, k_dev, v_dev = generate_and_upload(cfg, args.seed, lens, torch, args.workers)
    dtype = kv.KVC_BF16 if cfg.dtype == "bf16" else kv.KVC_F32
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    p = kv.KvcParams(cfg.batch, cfg.layers, cfg.hq, cfg.hkv, cfg.head_dim, cfg.window, dtype)
    ws_bytes = kv.kvc_workspace_size(p, total, max_n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    k_out = torch.empty(tb * cfg.hkv * cfg.head_dim, dtype=tdt, device="cuda")
    v_out = torch.empty_like(k_out)
    lengths = torch.empty(cfg.batch * cfg.layers, dtype=torch.int32, device="cuda")
    offsets = torch.empty(cfg.batch * cfg.layers + 1, dtype=torch.int64, device="cuda")
    qp, kp, vp = ([t.data_ptr() for t in ts] for ts in (q_dev, k_dev, v_dev))
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        kv.kvc_compress(p, qp, kp, vp, cu, budgets, k_out.data_ptr(), v_out.data_ptr(),
                        lengths.data_ptr(), offsets.data_ptr(), ws.data_ptr(), ws_bytes, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = total / (elapsed / args.steps)
    lens_out = lengths.cpu().numpy()
    assert int(lens_out.sum()) == tb, "retained count != budget"
    log(f"{ms_per_step:.3f} ms/step, {tokens_per_s / 1e6:.2f} M tokens/s; "
        f"N_l min/max = {lens_out.min()}/{lens_out.max()}")

    # ---- per-kernel durations from HIP events recorded by the library on the
    # launch stream, over the same number of steps ----
    kv.kvc_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = kv.kvc_profile_collect()
    kv.kvc_profile_enable(False)
    per_step = {k: (c // args.steps, ms / args.steps) for k, (c, ms) in prof.items()}
    for name, (c, ms) in sorted(per_step.items(), key=lambda x: -x[1][1]):
        log(f"  {name:28s} launches/step={c:4d}  ms/step={ms:8.3f}  avg_us={1e3 * ms / max(c, 1):9.1f}")

    # dominant kernel: the score contraction (one launch = window-Q x K^T of
    # cfg.layers / launches-per-step layers over all heads and tokens)
    dom = max(per_step.items(), key=lambda x: x[1][1])[0]
    roofline = None
    if dom.startswith("score_mfma"):
        c, ms = per_step[dom]
        layers_per_launch = cfg.layers / c
        flops_per_launch = 2.0 * cfg.hq * cfg.window * cfg.head_dim * total * layers_per_launch
        avg_s = ms / c * 1e-3
        achieved = flops_per_launch / avg_s / 1e12
        layer_shape = (cfg.hq, cfg.hkv, cfg.head_dim, cfg.window, total) == (32, 8, 128, 64, 131072)
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved,
                    "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_MFMA_TFLOPS,
                    "traffic": (MEASURED_TRAFFIC_BYTES[dom] * layers_per_launch
                                if layer_shape and dom in MEASURED_TRAFFIC_BYTES else None),
                    "avg_launch_us": avg_s * 1e6, "launches_per_step": c,
                    "layers_per_launch": layers_per_launch}
    elif dom == "gather_kernel":
        # per retained composite token and KV head: K and V rows read and written + one index
        c, ms = per_step[dom]
        esz_ = 2 if cfg.dtype == "bf16" else 4
        bytes_per_launch = tb * cfg.hkv * (4.0 * cfg.head_dim * esz_ + 4) / c
        avg_s = ms / c * 1e-3
        achieved = bytes_per_launch / avg_s / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": PEAK_HBM_GBPS,
                    "unit": "GB/s", "frac": achieved / PEAK_HBM_GBPS, "traffic": None,
                    "avg_launch_us": avg_s * 1e6, "launches_per_step": c}
    elif dom.startswith("score_"):
        # generic fp32 kernels (vector ALU, no matrix cores): 2*d flops per logit
        c, ms = per_step[dom]
        flops_per_launch = 2.0 * cfg.hq * cfg.window * cfg.head_dim * total * cfg.layers / c
        avg_s = ms / c * 1e-3
        achieved = flops_per_launch / avg_s / 1e12
        roofline = {"bound": "alu", "kernel": dom, "achieved": achieved, "peak": PEAK_FP32_VALU_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_VALU_TFLOPS, "traffic": None,
                    "avg_launch_us": avg_s * 1e6, "launches_per_step": c}
    stages = {
        "score_ms": sum(ms for k, (c, ms) in per_step.items() if k.startswith("score")),
        "rank_ms": sum(ms for k, (c, ms) in per_step.items() if k.startswith("head_rank")),
        "composite_ms": sum(ms for k, (c, ms) in per_step.items() if k.startswith("composite")),
        "select_ms": sum(ms for k, (c, ms) in per_step.items() if k.startswith("select")),
        "gather_ms": sum(ms for k, (c, ms) in per_step.items() if k.startswith("gather")),
    }
    esz = 2 if cfg.dtype == "bf16" else 4
    lht = cfg.layers * cfg.hkv * total
    hbm = {
        "score_algorithmic_tflops": 2.0 * cfg.layers * cfg.hq * cfg.window * cfg.head_dim * total
                                    / (stages["score_ms"] * 1e-3) / 1e12 if stages["score_ms"] else None,
        "rank_compulsory_gbps": 12.0 * lht / (stages["rank_ms"] * 1e-3) / 1e9 if stages["rank_ms"] else None,
        "gather_gbps": (tb * cfg.hkv * (4.0 * cfg.head_dim * esz + 4)) / (stages["gather_ms"] * 1e-3) / 1e9
                       if stages["gather_ms"] else None,
    }

    out = {
        "metric": METRIC, "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"config {cfg.config_id} ({cfg.name}): batch {cfg.batch}, "
                               f"{cfg.layers} layers, {cfg.hq}/{cfg.hkv} heads, d={cfg.head_dim}, "
                               f"N={max_n}, M={cfg.window}, keep {cfg.keep_percent}%",
                   "total_tokens": total, "budget": tb, "seed": args.seed},
        "roofline": roofline, "stages_ms": stages, "stage_rates": hbm,
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(cfg, args.seed, int(lens[0]), args.cpu_layers)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
