#!/usr/bin/env python3
"""Benchmark of the KVCompose compression pass on one MI355X.

One "step" is one kvc_compress call (score -> head-rank -> composite -> global
select -> gather) over a synthetic Llama-3-8B-shaped bf16 cache that is already
resident in HBM.  Prints ONE JSON line: throughput in context tokens per second,
the roofline figures of the longest-running kernel (from HIP events the library
records on the launch stream; against the published peak and against the
ceiling the library's register-resident MFMA probe reaches in the same run) and
the CPU oracle timed on a bounded sample.

Other modes (each prints one JSON line and exits):
  --sustain KIND[,KIND..] --seconds S   loop one stage (or a probe) for S seconds
        while a host thread samples shader clock and socket power; KIND is one
        of compress, score, rank, gather, mfma, mfma_stats, copy
  --graph                               the timed steps replay one kvc_compress call
        recorded in a HIP graph (for the small, launch-heavy workloads)
  --copy-probe MB                       the plain copy kernel (counter calibration)
  --record-traffic DIR                  turn rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
        csv output under DIR into profiles/hbm_traffic.json (no GPU needed)
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import csv
import glob
import hashlib
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "context tokens compressed/sec at Llama-3-8B shape, L=128k"
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBPS = 8000.0
# fp32 vector peak of the chip as published (256 CUs x 4 SIMDs x 16 lanes x 2 flops x
# 2.4 GHz x 2 for packed fp32 issue).  The library is compiled with packed fp32
# instructions off, so its plain-ALU kernels can reach half of it at most; the
# roofline object of such a kernel carries both.
PEAK_FP32_VALU_TFLOPS = 157.3
PEAK_FP32_VALU_TFLOPS_UNPACKED = PEAK_FP32_VALU_TFLOPS / 2
# Counter-derived HBM bytes per launch live in a tracked data file together with a
# digest of the kernel sources they were measured on (see load_traffic).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_DIR = os.path.join(ROOT, "paper_2509_05165_amd", "csrc")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


# --------------------------------------------------------------------------- traffic file
def kernel_source_digest() -> str:
    """sha256 over the kernel sources and the C header (names and contents, sorted)."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(KERNEL_DIR, "*")) +
                       glob.glob(os.path.join(ROOT, "include", "*.h"))):
        if os.path.isfile(path):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def load_traffic(kernel: str, shape: dict):
    """(bytes per layer, source note) for `kernel` at `shape`, or (None, why not).
    The stored figure is only handed out while the kernel sources are the ones it
    was measured on."""
    try:
        data = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None, "no profiles/hbm_traffic.json"
    if data.get("kernel_source_digest") != kernel_source_digest():
        return None, ("stale: kernel sources changed since profiles/hbm_traffic.json was "
                      f"recorded (commit {data.get('commit', '?')})")
    if data.get("layer_shape") != shape:
        return None, "recorded at another layer shape"
    ent = data.get("kernels", {}).get(kernel)
    if not ent:
        return None, "kernel not in profiles/hbm_traffic.json"
    note = (f"rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE scaled by the copy probe "
            f"(x{data['fetch_scale']:.3f} / x{data['write_scale']:.3f}), "
            f"profiles/hbm_traffic.json, commit {data.get('commit', '?')}")
    return ent["bytes_per_layer"], note


def _pmc_means(csv_path: str, counter: str) -> dict:
    acc = {}
    for r in csv.DictReader(open(csv_path)):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"].replace("kvc::(anonymous namespace)::", "").replace("void ", "")
        name = name.split("(")[0]
        acc.setdefault(name, []).append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def record_traffic(d: str, layers: int, commit: str) -> None:
    """DIR/{fetch,write,cal_fetch,cal_write}/p_counter_collection.csv -> profiles/hbm_traffic.json.
    The calibration runs are `bench.py --copy-probe 1024`, the others
    `bench.py --layers <layers>` at config 2."""
    def means(sub, counter):
        return _pmc_means(os.path.join(d, sub, "p_counter_collection.csv"), counter)
    known_kib = 1024.0 * 1024.0
    cal_f = means("cal_fetch", "FETCH_SIZE")["copy_probe_kernel"][0]
    cal_w = means("cal_write", "WRITE_SIZE")["copy_probe_kernel"][0]
    fs, ws = known_kib / cal_f, known_kib / cal_w
    fetch, write = means("fetch", "FETCH_SIZE"), means("write", "WRITE_SIZE")
    label = {"score_mfma<false, true, 4>": "score_mfma<stats>",
             "score_mfma<true, true, 4>": "score_mfma<emit>",
             "head_rank_kernel<false, false>": "head_rank_kernel",
             "head_rank_kernel<false, true>": "head_rank_kernel",
             "head_rank_kernel<true, false>": "head_rank_kernel", "gather_kernel": "gather_kernel"}
    kernels = {}
    for raw, (f, n) in fetch.items():
        key = next((v for k, v in label.items() if raw.replace(" ", "") == k.replace(" ", "")), raw)
        w = write.get(raw, (0.0, 0))[0]
        kernels[key] = {"fetch_kib_per_dispatch": f, "write_kib_per_dispatch": w, "dispatches": n,
                        "bytes_per_launch": (f * fs + w * ws) * 1024.0,
                        "bytes_per_layer": (f * fs + w * ws) * 1024.0 / layers}
    out = {"commit": commit, "kernel_source_digest": kernel_source_digest(),
           "layer_shape": {"hq": 32, "hkv": 8, "head_dim": 128, "window": 64, "tokens": 131072},
           "layers_per_launch": layers, "fetch_scale": fs, "write_scale": ws,
           "calibration": {"copy_probe_kib": known_kib, "fetch_reads": cal_f, "write_reads": cal_w},
           "kernels": kernels}
    json.dump(out, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
    print(json.dumps({"written": TRAFFIC_FILE, "kernels": sorted(kernels)}))


# --------------------------------------------------------------------------- clock / power
class GpuSampler(threading.Thread):
    """Samples socket power (hwmon power1_input / power1_average, microwatts) and
    the current shader clock (the starred line of pp_dpm_sclk) of the first GPU
    the box shows, from sysfs, every `period` seconds."""

    def __init__(self, period=0.02):
        super().__init__(daemon=True)
        self.period, self.samples, self._halt = period, [], threading.Event()
        dev = sorted(glob.glob("/sys/class/drm/card*/device"))
        self.dev = dev[0] if dev else None
        self.power_file = None
        if self.dev:
            for name in ("power1_input", "power1_average"):
                hits = glob.glob(os.path.join(self.dev, "hwmon", "hwmon*", name))
                if hits:
                    self.power_file = hits[0]
                    break
        self.sclk_file = os.path.join(self.dev, "pp_dpm_sclk") if self.dev else None

    def power_cap_w(self):
        hits = glob.glob(os.path.join(self.dev or "", "hwmon", "hwmon*", "power1_cap"))
        try:
            return int(open(hits[0]).read()) / 1e6
        except (OSError, ValueError, IndexError):
            return None

    def read_once(self):
        w = mhz = None
        try:
            w = int(open(self.power_file).read()) / 1e6
        except (OSError, ValueError, TypeError):
            pass
        try:
            for line in open(self.sclk_file):
                if "*" in line:
                    mhz = float(line.split(":")[1].lower().split("mhz")[0])
        except (OSError, ValueError, TypeError, IndexError):
            pass
        return w, mhz

    def run(self):
        while not self._halt.is_set():
            self.samples.append((time.perf_counter(),) + self.read_once())
            time.sleep(self.period)

    def stop(self):
        self._halt.set()
        self.join()

    @staticmethod
    def _summ(vals):
        vals = [v for v in vals if v is not None]
        if not vals:
            return None
        return {"min": min(vals), "median": statistics.median(vals), "max": max(vals), "n": len(vals)}

    def summary(self, t_from):
        rows = [s for s in self.samples if s[0] >= t_from]
        return {"power_w": self._summ([r[1] for r in rows]),
                "sclk_mhz": self._summ([r[2] for r in rows]),
                "source": f"sysfs {self.power_file} + {self.sclk_file}, every {self.period * 1e3:.0f} ms"}


# --------------------------------------------------------------------------- inputs
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
    orc.compress(qs, ks, vs, budget, causal_tail=bool(cfg.causal_tail))
    dt = time.time() - t0
    full = dt * cfg.layers / sample_layers
    return {
        "value": n / full, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{sample_layers} of {cfg.layers} layers at full N={n} (all stages), "
                  f"{dt:.1f}s measured, scaled by {cfg.layers}/{sample_layers}",
    }


# --------------------------------------------------------------------------- MFMA probe
class MfmaProbe:
    """The library's register-resident bf16 MFMA loop on operands drawn like the
    workload's (unit-variance normal values rounded to bf16)."""

    def __init__(self, torch, kv):
        self.torch, self.kv = torch, kv
        g = torch.Generator(device="cuda")
        g.manual_seed(1234)
        self.ops = torch.randn(kv.KVC_MFMA_PROBE_OPERAND_BYTES // 2, device="cuda",
                               generator=g).to(torch.bfloat16)
        self.sink = torch.empty(kv.KVC_MFMA_PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
        self.cycles = torch.zeros(2, dtype=torch.int64, device="cuda")

    def launch(self, iterations, mode):
        return self.kv.kvc_mfma_probe(self.ops.data_ptr(), iterations, mode, self.sink.data_ptr(),
                                      self.cycles.data_ptr(),
                                      self.torch.cuda.current_stream().cuda_stream)

    def shader_mhz(self):
        c = self.cycles.cpu().numpy()
        return float(c[0]) / (float(c[1]) / 100.0) if c[1] > 0 else None

    def measure(self, mode=0, seconds=0.3, iterations=20000):
        """TFLOP/s sustained over about `seconds` of back-to-back launches."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.launch(iterations, mode)
        torch.cuda.synchronize()
        e0.record(); flops = self.launch(iterations, mode); e1.record()
        torch.cuda.synchronize()
        one = e0.elapsed_time(e1) * 1e-3
        reps = max(2, int(seconds / max(one, 1e-6)))
        for _ in range(reps):                       # settle the clocks under this load
            self.launch(iterations, mode)
        e0.record()
        for _ in range(reps):
            self.launch(iterations, mode)
        e1.record()
        torch.cuda.synchronize()
        dt = e0.elapsed_time(e1) * 1e-3
        return {"tflops": flops * reps / dt / 1e12, "seconds": dt, "shader_mhz": self.shader_mhz()}


# --------------------------------------------------------------------------- main
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
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one kvc_compress call recorded in a HIP graph (small workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the MFMA ceiling probe")
    ap.add_argument("--cpu-layers", type=int, default=8)
    ap.add_argument("--workers", type=int, default=min(16, os.cpu_count() or 1))
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MB",
                    help="only run the library's plain copy kernel on MB MiB (counter calibration)")
    ap.add_argument("--sustain", type=str, default="",
                    help="comma-separated kinds to loop under the clock/power sampler")
    ap.add_argument("--seconds", type=float, default=3.0, help="length of each --sustain loop")
    ap.add_argument("--record-traffic", type=str, default="", metavar="DIR")
    ap.add_argument("--commit", type=str, default="?", help="commit named in the traffic file")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; this build uses no second GPU (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if args.record_traffic:
        record_traffic(args.record_traffic, args.layers or 4, args.commit)
        return

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
    p = kv.KvcParams(cfg.batch, cfg.layers, cfg.hq, cfg.hkv, cfg.head_dim, cfg.window, dtype,
                     causal_tail=cfg.causal_tail)
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

    if args.sustain:
        sustain(args, cfg, torch, kv, p, qp, kp, vp, cu, budgets, tb, total, max_n, step,
                lengths, offsets, k_out, v_out)
        return

    timed_step = step
    if args.graph:
        # the library only enqueues kernels, so a call can be recorded once and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cs = torch.cuda.current_stream().cuda_stream
            kv.kvc_compress(p, qp, kp, vp, cu, budgets, k_out.data_ptr(), v_out.data_ptr(),
                            lengths.data_ptr(), offsets.data_ptr(), ws.data_ptr(), ws_bytes, cs)
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
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
        # query rows the launch covers: all Hq*M, or, when the small last row chunk of every
        # KV head runs as a launch of its own (",rem"), the full 256-row chunks / that chunk
        rows_head = cfg.group * cfg.window
        rows = cfg.hq * cfg.window
        if any(k.endswith(",rem") for k in per_step):
            rows = cfg.hkv * (rows_head % 256 if dom.endswith(",rem") else rows_head // 256 * 256)
        flops_per_launch = 2.0 * rows * cfg.head_dim * total * layers_per_launch
        avg_s = ms / c * 1e-3
        achieved = flops_per_launch / avg_s / 1e12
        shape = {"hq": cfg.hq, "hkv": cfg.hkv, "head_dim": cfg.head_dim, "window": cfg.window,
                 "tokens": total}
        per_layer, source = load_traffic(dom, shape)
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved,
                    "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_MFMA_TFLOPS,
                    "traffic": per_layer * layers_per_launch if per_layer else None,
                    "traffic_source": source,
                    "avg_launch_us": avg_s * 1e6, "launches_per_step": c,
                    "layers_per_launch": layers_per_launch}
        if not args.no_probe:
            # measured ceiling: what the matrix cores sustain on a loop that never leaves
            # the registers, same instruction and occupancy, same run, same power limit
            probe = MfmaProbe(torch, kv)
            m0 = probe.measure(mode=0)
            m1 = probe.measure(mode=1)
            roofline.update({
                "peak_measured": m0["tflops"], "frac_measured": achieved / m0["tflops"],
                "probe": {"what": "kvc_mfma_probe: register-resident v_mfma_f32_32x32x16_bf16 loop, "
                                  "two waves per SIMD on all CUs, unit-normal bf16 operands",
                          "mfma_only_tflops": m0["tflops"], "mfma_only_shader_mhz": m0["shader_mhz"],
                          "mfma_with_softmax_valu_tflops": m1["tflops"],
                          "mfma_with_softmax_valu_shader_mhz": m1["shader_mhz"],
                          "seconds_each": round(m0["seconds"], 3)}})
            log(f"MFMA probe: {m0['tflops']:.0f} TFLOP/s at {m0['shader_mhz']:.0f} MHz (MFMA only), "
                f"{m1['tflops']:.0f} TFLOP/s at {m1['shader_mhz']:.0f} MHz (with the statistics "
                f"pass's vector work)")
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
                    "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_VALU_TFLOPS,
                    "peak_unpacked": PEAK_FP32_VALU_TFLOPS_UNPACKED,
                    "frac_unpacked": achieved / PEAK_FP32_VALU_TFLOPS_UNPACKED,
                    "note": "the library is built without packed fp32 instructions: peak_unpacked "
                            "is what its plain-ALU kernels can reach",
                    "traffic": None, "avg_launch_us": avg_s * 1e6, "launches_per_step": c}
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
                               f"N={max_n}, M={cfg.window}, keep {cfg.keep_percent}%"
                               + (", causal tail" if cfg.causal_tail else ""),
                   "total_tokens": total, "budget": tb, "seed": args.seed,
                   "launch": "hip graph replay" if args.graph else "eager"},
        "roofline": roofline, "stages_ms": stages, "stage_rates": hbm,
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(cfg, args.seed, int(lens[0]), args.cpu_layers)
    print(json.dumps(out), flush=True)


def sustain(args, cfg, torch, kv, p, qp, kp, vp, cu, budgets, tb, total, max_n, step,
            lengths, offsets, k_out, v_out):
    """Loops of one stage for --seconds each, with clock and power sampled beside."""
    stream = torch.cuda.current_stream().cuda_stream
    ws_bytes = kv.kvc_workspace_size(p, total, max_n)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    S = torch.empty((cfg.layers, cfg.hkv, total), dtype=torch.float32, device="cuda")
    idx = torch.empty((cfg.layers, cfg.hkv, total), dtype=torch.int32, device="cuda")
    ss = torch.empty_like(S)
    # one full pass with the taps on, so that every stage has valid inputs
    kv.kvc_compress(p, qp, kp, vp, cu, budgets, k_out.data_ptr(), v_out.data_ptr(),
                    lengths.data_ptr(), offsets.data_ptr(), ws.data_ptr(), ws_bytes, stream,
                    scores=S.data_ptr(), idx=idx.data_ptr(), s_sorted=ss.data_ptr())
    torch.cuda.synchronize()
    probe = MfmaProbe(torch, kv)
    copy_bytes = 1 << 30
    kinds = {
        "compress": (step, 1),
        "score": (lambda: kv.kvc_score(p, qp, kp, cu, S.data_ptr(), ws.data_ptr(), ws_bytes, stream), 1),
        "rank": (lambda: kv.kvc_head_rank(p, S.data_ptr(), cu, idx.data_ptr(), ss.data_ptr(),
                                          ws.data_ptr(), ws_bytes, stream), 1),
        "gather": (lambda: kv.kvc_gather(p, kp, vp, idx.data_ptr(), lengths.data_ptr(),
                                         offsets.data_ptr(), cu, tb, k_out.data_ptr(),
                                         v_out.data_ptr(), stream, ws.data_ptr(), ws_bytes), 1),
        "mfma": (lambda: probe.launch(20000, 0), 1),
        "mfma_stats": (lambda: probe.launch(20000, 1), 1),
    }
    if "copy" in args.sustain:
        csrc = torch.ones(copy_bytes, dtype=torch.uint8, device="cuda")
        cdst = torch.empty_like(csrc)
        kinds["copy"] = (lambda: kv.kvc_copy_probe(cdst.data_ptr(), csrc.data_ptr(), copy_bytes, stream), 1)
    sampler = GpuSampler()
    idle = sampler.read_once()
    sampler.start()
    results = {}
    for kind in [k for k in args.sustain.split(",") if k]:
        fn = kinds[kind][0]
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); fn(); e1.record(); torch.cuda.synchronize()
        one = max(e0.elapsed_time(e1) * 1e-3, 1e-5)
        batch = max(1, int(0.05 / one))              # about 50 ms of work between host syncs
        t_start = time.perf_counter()
        calls, gpu_ms = 0, 0.0
        flops = None
        while time.perf_counter() - t_start < args.seconds:
            e0.record()
            for _ in range(batch):
                r = fn()
                if isinstance(r, float):
                    flops = r
            e1.record()
            torch.cuda.synchronize()
            gpu_ms += e0.elapsed_time(e1)
            calls += batch
        # the first third of the loop is left out of the summary (clocks settling)
        summ = sampler.summary(t_start + args.seconds / 3)
        res = {"calls": calls, "ms_per_call": gpu_ms / calls, "seconds": args.seconds, **summ}
        if kind.startswith("mfma"):
            res["tflops"] = flops * calls / (gpu_ms * 1e-3) / 1e12
            res["shader_mhz_in_kernel"] = probe.shader_mhz()
        if kind == "copy":
            res["gbps_read_plus_write"] = 2 * copy_bytes * calls / (gpu_ms * 1e-3) / 1e9
        if kind == "compress":
            res["tokens_per_s"] = total * calls / (gpu_ms * 1e-3)
        results[kind] = res
        log(f"sustain {kind}: {res['ms_per_call']:.3f} ms/call over {calls} calls; "
            f"power {summ['power_w']}; sclk {summ['sclk_mhz']}")
        time.sleep(0.5)
    sampler.stop()
    print(json.dumps({"sustain": results, "idle": {"power_w": idle[0], "sclk_mhz": idle[1]},
                      "power_cap_w": sampler.power_cap_w(),
                      "workload": f"config {cfg.config_id} ({cfg.name}), {cfg.layers} layers"}),
          flush=True)


if __name__ == "__main__":
    main()
