#!/usr/bin/env python3
"""Benchmark of the routed forward pass through quantization experts on one MI355X.

A step is one moqe_forward over one batch of the workload: route -> bucket -> grouped
dequantize-GEMM gate/up with the fused SiLU gate -> grouped dequantize-GEMM down -> scatter.
Default workload: the LLaMA-7B-shaped MLP block in decode (64 sequences x 1 token, 4 experts),
synthetic seeded tensors.  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line with the throughput, the roofline of the dominant kernel (measured with HIP events on the
launch stream during the timed steps) and the CPU oracle timed on the host cores; a `workloads` array in
the same line carries the prefill-shaped, skewed and convolution workloads (step time, dominant kernel,
roofline), measured in the same run with fewer steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
MFMA_INT8_PEAK_TOPS = 5000.0    # dense int8, published

# Kernel durations from the committed rocprofv3 --kernel-trace summaries (profiles/), per workload.  The events of
# this file are handed to the kernel launch itself and read within about 5 % of the trace (2-3 us on the decode
# kernel); `frac_rocprof` is the roofline fraction with the profiler's own average duration.  Tied to the kernel
# sources like the traffic figure.
_SOURCES_AT_PROFILE = "fcee4361dc2eceee815b53fbf9630a367ad61f4fc1f5c724897bac7c85ca4a88"
ROCPROF_KERNEL_US = {
    "llama7b_mlp_decode": {"sources_sha256": _SOURCES_AT_PROFILE, "kernel_us": 49.62},
    "llama7b_mlp_prefill": {"sources_sha256": _SOURCES_AT_PROFILE, "kernel_us": 1717.04},
    "qwen_mlp_skew": {"sources_sha256": _SOURCES_AT_PROFILE, "kernel_us": 9932.68},
    "resnet50_conv": {"sources_sha256": _SOURCES_AT_PROFILE, "kernel_us": 93.47},
}


# HBM traffic of the dominant kernel from hardware counters (two rocprofv3 --pmc runs, FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB device copy; summary and
# commands are kept with the profile summaries in the repository).  Valid only for the kernel sources it was taken with: the entry carries
# their hash and is ignored (traffic = null) once they have changed.
KERNEL_SOURCES = ("qgemm_stream.hip", "qgemm_stream_lds.hip", "qgemm_tile.hip", "qgemm_device.h")       # the GEMM kernels' own sources
MEASURED_TRAFFIC = {
    "llama7b_mlp_decode": {"sources_sha256": "fcee4361dc2eceee815b53fbf9630a367ad61f4fc1f5c724897bac7c85ca4a88",
                           "bytes_per_launch": 232140493},   # fetch 230.21 MB + write 1.93 MB
}


def kernel_sources_hash():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2508_09204_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload):
    t = MEASURED_TRAFFIC.get(workload)
    if not t or not t["sources_sha256"] or t["sources_sha256"] != kernel_sources_hash():
        return None
    return t["bytes_per_launch"]


def algorithmic_weight_bytes(n, k, spec):
    """Bytes the format defines for one matrix: packed code bits + fp32 scales + u8 zero-points."""
    code = n * k * spec.bits // 8
    if spec.group:
        meta = n * (k // spec.group) * (4 + (0 if spec.symmetric else 1))
    else:
        meta = n * 4
    return code + meta


def build_device_block(cfg, n_copies):
    """Quantizes and packs the experts ON THE GPU through the library; returns `n_copies` blocks that
    share the router but own separate copies of the packed weights (rotated between steps so that a
    step never finds its weights in the last-level cache from the step before)."""
    import torch
    import workloads as wl
    from paper_2508_09204_amd import binding as mq, experts as ex

    dev = "cuda:0"
    fpw = wl.make_fp_weights(cfg)
    r = wl.make_router(cfg)
    td = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    router = mq.Router(td(r["w1"]), td(r["b1"]), td(r["w2"]), td(r["b2"]), cfg.D, cfg.router_hidden, cfg.K)
    packed = {}
    for name, w in fpw.items():
        wd = torch.from_numpy(w).to(dev)
        packed[name] = [ex.quantize_and_pack(wd, e.bits, e.group, e.symmetric, e.clip, e.act_mode) for e in cfg.experts]
        del wd
    torch.cuda.synchronize()

    def clone(qm):
        return mq.QMat(qm.qdata.clone(), None, None, qm.n, qm.k, qm.bits, qm.group, qm.symmetric, qm.act_mode, qm.layout)

    blocks = []
    for c in range(n_copies):
        pk = packed if c == 0 else {n: [clone(q) for q in v] for n, v in packed.items()}
        if cfg.kind == wl.configs.KIND_SILU_MLP:
            blocks.append(mq.Block(cfg.kind, router, pk["gate"], pk["up"], pk["down"]))
        else:
            blocks.append(mq.Block(cfg.kind, router, pk["w0"], img_h=cfg.img_h, img_w=cfg.img_w,
                                   cin=cfg.D if cfg.kind == wl.configs.KIND_CONV3X3 else 0))
    return blocks


def cpu_baseline(cfg, max_seconds_hint=30.0):
    """The oracle as it stands, timed on the host: the whole forward for the decode workload,
    a bounded number of sequences for larger ones."""
    import numpy as np
    import workloads as wl
    from oracle import moqe_oracle as oc
    from tests import oracle_blocks as ob
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    blk = ob.make_block(cfg)                      # quantization is offline work: not timed
    bits = wl.make_activations(cfg)
    x64 = oc.bf16_bits_to_f64(bits)
    if cfg.M <= 256:
        n_s, rows, sample = cfg.S, None, f"all {cfg.S} samples x {cfg.T} rows"
    elif cfg.kind == wl.configs.KIND_CONV3X3:
        n_s, rows = min(cfg.S, 32), None
        sample = f"first {n_s} images, whole images"
    else:
        n_s, rows = min(cfg.S, 16), [0, cfg.T // 2, cfg.T - 1]
        sample = f"first {n_s} samples, 3 rows each (all columns)"
    t0 = time.perf_counter()
    y, idx, _ = oc.forward(blk, x64[:n_s], rows=rows)
    dt = time.perf_counter() - t0
    units = y.shape[0] * y.shape[1] if cfg.unit == "tokens" else y.shape[0]
    return {"value": units / dt, "unit": f"{cfg.unit}/s", "cores": int(cores), "kind": "oracle",
            "sample": sample + f"; {dt:.1f} s wall, dequantization of the routed experts included"}


def rocprof_kernel_us(workload):
    t = ROCPROF_KERNEL_US.get(workload)
    if not t or t["sources_sha256"] != kernel_sources_hash():
        return None
    return t["kernel_us"]


# The paper's NLP router model at a size that matches its stated 16.7 MB of fp32 parameters for d = 4096:
# width 384, 6 heads, feed-forward 1536, MLP head 384 -> 384 -> K (4.08 M parameters).
NLP_ROUTER = {"dm": 384, "n_heads": 6, "d_ff": 1536, "head_hidden": 384}


def measure_router_nlp(cfg, x, calls=10):
    """Time of one moqe_route_nlp call on the workload's token vectors (random parameters), not part of the step."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_2508_09204_amd import binding as mq
    dev = x.device
    g = NLP_ROUTER
    p = wl.make_nlp_router(cfg.D, g["dm"], g["n_heads"], g["d_ff"], g["head_hidden"], cfg.K, cfg.seed + 77)
    t = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for k, v in p.items()}
    head = mq.Router(t["head_w1"], t["head_b1"], t["head_w2"], t["head_b2"], g["dm"], g["head_hidden"], cfg.K)
    r = mq.NlpRouter(t, head, cfg.D, g["dm"], g["n_heads"], g["d_ff"])
    idx = torch.zeros(cfg.S, dtype=torch.int32, device=dev)
    ws = torch.empty(mq.moqe_route_nlp_workspace_bytes(cfg.S, cfg.T, r), dtype=torch.uint8, device=dev)
    for _ in range(2):
        mq.moqe_route_nlp(x, cfg.S, cfg.T, r, idx, None, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        mq.moqe_route_nlp(x, cfg.S, cfg.T, r, idx, None, ws)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / calls * 1e6
    params = sum(int(v.size) for v in p.values())
    return {"us_per_call": us, "parameters": params, "fp32_megabytes": params * 4 / 1e6, **g}


# The paper's CV router model with its stated channel counts, strides and head count; MLP widths of our choosing.
CV_ROUTER = {"mlp": (64, 32, 16), "stages": (16, 32, 64), "strides": (1, 2, 2), "n_heads": 8}


def measure_router_cv(cfg, x, calls=10):
    """Time of one moqe_route_cv call on the workload's images (random parameters), not part of the step."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_2508_09204_amd import binding as mq
    dev = x.device
    g = CV_ROUTER
    p = wl.make_cv_router(cfg.D, g["mlp"], g["stages"], g["strides"], cfg.K, cfg.seed + 78)
    t = {k: torch.from_numpy(np.ascontiguousarray(v)).to(dev) for k, v in p.items()}
    r = mq.CvRouter(t, cfg.D, g["strides"], g["n_heads"], cfg.K)
    idx = torch.zeros(cfg.S, dtype=torch.int32, device=dev)
    ws = torch.empty(mq.moqe_route_cv_workspace_bytes(cfg.S, cfg.img_h, cfg.img_w, r), dtype=torch.uint8, device=dev)
    for _ in range(2):
        mq.moqe_route_cv(x, cfg.S, cfg.img_h, cfg.img_w, r, idx, None, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        mq.moqe_route_cv(x, cfg.S, cfg.img_h, cfg.img_w, r, idx, None, ws)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / calls * 1e6
    params = sum(int(v.size) for v in p.values())
    return {"us_per_call": us, "parameters": params, "fp32_megabytes": params * 4 / 1e6,
            "routing_histogram": np.bincount(idx.cpu().numpy(), minlength=cfg.K).tolist(), **{k: list(v) if isinstance(v, tuple) else v for k, v in g.items()}}


def measure(name, steps, warmup, copies=0, with_graph=False, experts=None):
    """Builds the workload on the GPU, times `steps` forwards after `warmup` untimed ones, and returns the
    step metrics and the roofline of its dominant kernel (HIP events on the launch stream, recorded by the
    library during the timed steps)."""
    import dataclasses
    import torch
    import workloads as wl
    from paper_2508_09204_amd import binding as mq

    dev = "cuda:0"
    cfg = wl.get_config(name)
    if experts is not None:
        cfg = dataclasses.replace(cfg, experts=tuple(experts))
    is_mlp = cfg.kind == wl.configs.KIND_SILU_MLP
    is_conv = cfg.kind == wl.configs.KIND_CONV3X3
    mats = cfg.matrices()
    per_expert_bytes = [sum(algorithmic_weight_bytes(n, k, e) for (n, k) in mats.values()) for e in cfg.experts]
    n_copies = copies or max(2, min(8, -(-(1 << 30) // sum(per_expert_bytes))))
    blocks = build_device_block(cfg, n_copies)
    dominant = mq.PK_GEMM_GATEUP if is_mlp else mq.PK_GEMM_PLAIN

    bits = wl.make_activations(cfg)
    x = torch.from_numpy(bits.view("int16").reshape(cfg.M, cfg.D)).to(dev).view(torch.bfloat16)
    n_out = cfg.D if is_mlp else cfg.F
    y = torch.empty((cfg.M, n_out), dtype=torch.float32, device=dev)
    counts = torch.zeros(cfg.K, dtype=torch.int32, device=dev)
    aux = mq.Aux(counts=counts)
    calls = [mq.ForwardCall(b, x, cfg.S, cfg.T, y, aux) for b in blocks]
    stream = torch.cuda.current_stream().cuda_stream
    mq.moqe_profile_enable(1 << dominant)          # warm the event pool before the timed region
    for i in range(warmup):
        calls[i % len(calls)](stream)
    torch.cuda.synchronize()
    mq.moqe_profile_enable(1 << dominant)
    t0 = time.perf_counter()
    for i in range(steps):
        calls[i % len(calls)](stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    launches, kern_ms = mq.moqe_profile_read(dominant)
    mq.moqe_profile_enable(0)
    hist = counts.cpu().tolist()

    graph_ms = None
    if with_graph:
        # the same steps replayed from captured graphs (one per weight copy): launch gaps of the eager loop removed.
        # A side figure: if capture or replay fails on a machine, the eager figures above still stand.
        try:
            graphs = []
            for c in calls:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    c(torch.cuda.current_stream().cuda_stream)
                graphs.append(g)
            for i in range(min(warmup, 10)):
                graphs[i % len(graphs)].replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                graphs[i % len(graphs)].replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t0) * 1e3 / steps
            del graphs
        except Exception as exc:       # noqa: BLE001 - reported, not hidden
            print("graph replay not timed: %r" % (exc,), file=sys.stderr, flush=True)
            graph_ms = None

    ms_per_step = dt * 1e3 / steps
    units = cfg.M if cfg.unit == "tokens" else cfg.S
    kern_us = kern_ms * 1e3 / max(launches, 1)
    launches_per_step = max(1, round(launches / steps))       # a bucket-size split may launch both GEMM kernels
    kern_us *= launches_per_step

    # algorithmic bytes / flops of the dominant launch: each non-empty expert's matrices once
    dom_mats = [mats["gate"], mats["up"]] if is_mlp else list(mats.values())
    dom_bytes = sum(sum(algorithmic_weight_bytes(n, k, e) for (n, k) in dom_mats)
                    for e, c in zip(cfg.experts, hist) if c > 0)
    flops_per_expert = [2.0 * c * cfg.T * sum(n * k for (n, k) in dom_mats) for c in hist]
    dom_flops = sum(flops_per_expert)
    # every non-empty bucket has a multiple of T rows: few rows stream the weights (bound by HBM), many rows
    # are a dense contraction on the matrix cores
    hbm_bound = (not is_conv) and cfg.T <= 32 and cfg.M <= 128
    rp_us = rocprof_kernel_us(cfg.name) if experts is None else None
    if hbm_bound:
        achieved = dom_bytes / (kern_us * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(cfg.name) if experts is None else None}
        if rp_us:
            roof["frac_rocprof"] = dom_bytes / (rp_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    else:
        # experts with int8 activations run on the int8 matrix cores: the launch's fraction of peak is the time the
        # flops would take at each expert's own peak over the measured time
        ideal_s = sum(f / ((MFMA_INT8_PEAK_TOPS if e.act_mode else MFMA_BF16_PEAK_TFLOPS) * 1e12)
                      for f, e in zip(flops_per_expert, cfg.experts))
        achieved = dom_flops / (kern_us * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ideal_s / (kern_us * 1e-6), "traffic": None}
        if any(e.act_mode for e in cfg.experts):
            roof["peak_note"] = "frac = sum over experts of flops / own peak (int8 5000 TOP/s for the W8A8 expert) over the kernel time"
        if rp_us:
            roof["frac_rocprof"] = ideal_s / (rp_us * 1e-6)
        # the same launch against the HBM roofline: weights once, activations in (bf16), results out
        k_in = cfg.D if is_conv else dom_mats[0][1]          # conv: the kernel gathers from the image
        io_bytes = cfg.M * k_in * 2 + cfg.M * dom_mats[0][0] * (2 if is_mlp else 4)
        roof["hbm_view"] = {"algorithmic_bytes_per_launch": dom_bytes + io_bytes,
                            "achieved_gbs": (dom_bytes + io_bytes) / (kern_us * 1e-6) / 1e9,
                            "frac_of_8tbs": (dom_bytes + io_bytes) / (kern_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    roof["kernel"] = ("k_qgemm_stream" if hbm_bound else "k_qgemm_tile") + ("<gate/up + SiLU>" if is_mlp else "<plain>")
    roof["kernel_us"] = kern_us
    if rp_us:
        roof["kernel_us_rocprof"] = rp_us
    roof["launches_timed"] = launches
    roof["algorithmic_bytes_per_launch"] = dom_bytes
    roof["algorithmic_flops_per_launch"] = dom_flops
    res = {"cfg": cfg, "n_copies": n_copies, "hist": hist, "ms_per_step": ms_per_step, "value": units / (dt / steps),
           "graph_ms_per_step": graph_ms, "roofline": roof, "steps": steps}
    if is_mlp and experts is None:
        res["router_nlp"] = measure_router_nlp(cfg, x)
    if is_conv and experts is None:
        res["router_cv"] = measure_router_cv(cfg, x)
    del blocks, calls
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama7b_mlp_decode")
    ap.add_argument("--copies", type=int, default=0, help="rotating weight copies (0 = pick so that they exceed 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-int4-only", action="store_true", help="skip the extra all-int4 measurement of the decode launch")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the prefill / skew / conv entries of `workloads`")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the warm-up, run a plain device copy of 1 GiB five times (a kernel of known "
                         "traffic, for scaling hardware counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU (samples would shard across GPUs with no collective); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head = measure(args.workload, args.steps, args.warmup, args.copies, with_graph=True)
    cfg, roof = head["cfg"], head["roofline"]

    # The decode target is stated for a grouped int4 GEMM: the same launch with all experts int4 g128.
    if roof["bound"] == "hbm" and cfg.kind == wl.configs.KIND_SILU_MLP and not args.no_int4_only:
        int4 = wl.configs.ExpertSpec(4, 128, False)
        r4 = measure(args.workload, max(20, args.steps // 2), min(args.warmup, 10), 0, experts=[int4] * cfg.K)
        q = r4["roofline"]
        roof["int4_only"] = {"experts": [int4.label()] * cfg.K, "kernel_us": q["kernel_us"], "launches_timed": q["launches_timed"],
                             "algorithmic_bytes_per_launch": q["algorithmic_bytes_per_launch"], "achieved": q["achieved"],
                             "frac": q["frac"]}

    def entry(r):
        c = r["cfg"]
        return {"workload": c.name, "samples": c.S, "rows_per_sample": c.T, "experts": [e.label() for e in c.experts],
                "routing_histogram": r["hist"], "steps": r["steps"], "ms_per_step": r["ms_per_step"],
                "value": r["value"], "unit": f"{c.unit}/s", "roofline": r["roofline"],
                **({"router_nlp": r["router_nlp"]} if "router_nlp" in r else {}),
                **({"router_cv": r["router_cv"]} if "router_cv" in r else {})}

    others = []
    if not args.no_other_workloads and args.workload == "llama7b_mlp_decode":
        for name, st, wu in (("llama7b_mlp_prefill", 20, 3), ("qwen_mlp_skew", 5, 2), ("resnet50_conv", 100, 10)):
            others.append(entry(measure(name, st, wu, 2)))

    out = {
        "metric": "routed qGEMM throughput (whole routed block: route + bucket + grouped qGEMMs + scatter)",
        "value": head["value"], "unit": f"{cfg.unit}/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic (seeded N(0,1) activations, N(0,0.02) weights quantized by round-to-nearest on the GPU)",
        "config": {"workload": cfg.name, "samples": cfg.S, "rows_per_sample": cfg.T, "d": cfg.D, "f": cfg.F,
                   "experts": [e.label() for e in cfg.experts], "routing_histogram": head["hist"],
                   "arithmetic": "bf16 activations x exact integer weight codes on bf16 MFMA, fp32 accumulate and scales",
                   "rotating_weight_copies": head["n_copies"],
                   "ms_per_step_graph_replay": head["graph_ms_per_step"],
                   **({"router_nlp": head["router_nlp"]} if "router_nlp" in head else {}),
                   **({"router_cv": head["router_cv"]} if "router_cv" in head else {})},
        "roofline": roof,
        "workloads": others,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
