#!/usr/bin/env python3
"""Timing of the serving mode with on-demand expert residency (Section 4.4 and the appendix on memory):
one sequence at a time, the router selects its expert, the expert's packed weights are copied in from
pinned host memory if they are not resident, the expert runs.  Prints one JSON line with the router time,
the copy time of a switch, the expert time and the overhead of routing and copying relative to the expert.

Workload: the LLaMA-7B-shaped MLP block in decode (one token per request), four experts, seeded synthetic
tensors; `--slots` experts resident at a time (each expert = its gate, up and down matrices).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=64)
    ap.add_argument("--slots", type=int, default=1, help="experts resident at a time")
    args = ap.parse_args()

    import numpy as np
    import torch
    import workloads as wl
    from paper_2508_09204_amd import binding as mq, experts as ex

    assert torch.cuda.is_available(), "needs the GPU"
    dev = "cuda:0"
    cfg = wl.get_config("llama7b_mlp_decode")
    fpw = wl.make_fp_weights(cfg)
    r = wl.make_router(cfg)
    td = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    router = mq.Router(td(r["w1"]), td(r["b1"]), td(r["w2"]), td(r["b2"]), cfg.D, cfg.router_hidden, cfg.K)
    names = ["gate", "up", "down"]
    meta, host = {}, []
    for name in names:
        wd = torch.from_numpy(fpw[name]).to(dev)
        meta[name] = []
        for e in cfg.experts:
            q = ex.quantize_and_pack(wd, e.bits, e.group, e.symmetric, e.clip, e.act_mode)
            meta[name].append(q)
        del wd
    # blob 3 * e + i = matrix i of expert e, waiting in pinned host memory
    for e in range(cfg.K):
        for name in names:
            host.append(meta[name][e].qdata.cpu().pin_memory())
    expert_bytes = [sum(host[3 * e + i].numel() for i in range(3)) for e in range(cfg.K)]
    for name in names:
        for q in meta[name]:
            q.qdata = None                                           # the device copies go away: only the cache holds weights
    torch.cuda.empty_cache()
    cache = mq.moqe_cache_create(host, 3 * args.slots)

    bits = wl.make_activations(cfg)
    x_all = torch.from_numpy(bits.view("int16").reshape(cfg.M, cfg.D)).to(dev).view(torch.bfloat16)
    S = min(args.requests, cfg.S)
    idx = torch.empty(1, dtype=torch.int32, device=dev)
    ws_route = torch.empty(max(mq.moqe_route_workspace_bytes(1, 1, router), 256), dtype=torch.uint8, device=dev)
    y = torch.empty((1, cfg.D), dtype=torch.float32, device=dev)

    def qm(proto, addr):
        return mq.QMat(addr, None, None, proto.n, proto.k, proto.bits, proto.group, proto.symmetric, proto.act_mode, proto.layout)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_route, t_copy, t_expert, switches, copied_bytes = [], [], [], 0, 0
    for rep in range(2):                                             # first pass warms up
        t_route, t_copy, t_expert, switches, copied_bytes = [], [], [], 0, 0
        for s in range(S):
            x = x_all[s:s + 1]
            e0, e1, e2, e3 = ev(), ev(), ev(), ev()
            e0.record()
            mq.moqe_route(x, 1, 1, router, idx, None, ws_route)
            e1.record()
            e = int(idx.item())                                      # the host decides what to load
            addrs, copied = mq.moqe_cache_acquire(cache, [3 * e, 3 * e + 1, 3 * e + 2])
            e2.record()
            gate = [qm(meta["gate"][k], addrs[0]) for k in range(cfg.K)]      # other experts: placeholders, never read
            up = [qm(meta["up"][k], addrs[1]) for k in range(cfg.K)]
            down = [qm(meta["down"][k], addrs[2]) for k in range(cfg.K)]
            blk = mq.Block(cfg.kind, router, gate, up, down)
            mq.ForwardCall(blk, x, 1, 1, y, mq.Aux())(torch.cuda.current_stream().cuda_stream)
            e3.record()
            torch.cuda.synchronize()
            t_route.append(e0.elapsed_time(e1))
            if copied:
                t_copy.append(e1.elapsed_time(e2))
                switches += 1
                copied_bytes += expert_bytes[e]
            t_expert.append(e2.elapsed_time(e3))
    mq.moqe_cache_destroy(cache)
    med = lambda v: float(np.median(v)) if v else 0.0
    out = {
        "workload": "llama7b_mlp_decode, one sequence per request", "requests": S, "slots": args.slots,
        "switches": switches, "router_ms": med(t_route), "switch_copy_ms": med(t_copy),
        "switch_copy_gbs": (copied_bytes / max(switches, 1)) / (med(t_copy) * 1e-3) / 1e9 if t_copy else None,
        "expert_ms": med(t_expert),
        "overhead_with_switch": (med(t_route) + med(t_copy)) / med(t_expert) if t_copy else None,
        "overhead_without_switch": med(t_route) / med(t_expert),
        "expert_bytes": expert_bytes,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
