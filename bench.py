"""Benchmark of the encoder task + embedding hand-off on one MI355X.

One step = cs_encode over one packed batch (patch embed, all transformer blocks, merger) followed
by cs_forward_embeddings into the consumer buffer, inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c4|c5|c3] [--breakdown]
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

import hashlib
import os
import re

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 2.4 GHz x 4096 flop/CU/clk, dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
ROOT = os.path.dirname(os.path.abspath(__file__))


def measured_traffic(workload: str, kernel: str, items_default: bool):
    """HBM-side bytes per launch of the dominant kernel, from the counter summary profiles/<workload>_hbm_counters.md
    (lines `dominant_kernel: ...`, `dominant_kernel_traffic_bytes: ...`, `gemm_hip_sha256: ...`).  The counters
    belong to the kernel source and launch they were taken on: None when the summary is missing, when gemm.hip
    has changed since, when the batch is not the workload's own, or when another kernel instantiation runs now."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_counters.md")
    if not items_default or not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = {k: re.search(rf"^{k}:\s*(.+)$", text, re.M) for k in ("dominant_kernel", "dominant_kernel_traffic_bytes", "gemm_hip_sha256")}
    if not all(m.values()):
        return None, None
    src = os.path.join(ROOT, "paper_2603_12118_amd", "csrc", "gemm.hip")
    if hashlib.sha256(open(src, "rb").read()).hexdigest() != m["gemm_hip_sha256"].group(1).strip():
        return None, "gemm.hip changed since profiles/%s_hbm_counters.md was taken" % workload
    if m["dominant_kernel"].group(1).strip() != kernel:
        return None, "the counters were taken on another kernel instantiation"
    return float(m["dominant_kernel_traffic_bytes"].group(1)), "profiles/%s_hbm_counters.md" % workload


def algorithmic_flops(cfg, grid_thw) -> dict:
    """FLOPs the method has to do (no padding, no masked-out attention), split by step."""
    g = np.asarray(grid_thw, np.int64)
    n_item = g.prod(1)
    N = int(n_item.sum())
    D, I, L = cfg.hidden, cfg.mlp_dim, cfg.n_layers
    f = {}
    if cfg.arch == "vit":
        M = N // 4
        f["front"] = 2 * N * cfg.patch_dim * D
        win = 0
        for (T, h, w) in g.tolist():
            hs = [cfg.window] * (h // cfg.window) + ([h % cfg.window] if h % cfg.window else []) if cfg.window > 0 else [h]
            ws = [cfg.window] * (w // cfg.window) + ([w % cfg.window] if w % cfg.window else []) if cfg.window > 0 else [w]
            win += T * sum((a * b) ** 2 for a in hs for b in ws)
        full = int((n_item ** 2).sum())
        n_full = len(cfg.full_attn_layers) if cfg.window > 0 else L
        f["attn_window"] = 4 * win * D * (L - n_full)
        f["attn_full"] = 4 * full * D * n_full
        f["mlp_up"] = 2 * N * D * 2 * I * L
        f["mlp_down"] = 2 * N * I * D * L
        f["back"] = 2 * M * 4 * D * cfg.merger_hidden + 2 * M * cfg.merger_hidden * cfg.out_hidden
    elif cfg.arch == "vit_cls":
        # tokens per tile: its patches and the class token; the projector runs on the patches only
        tok = n_item + 1
        M = N // 4
        f["front"] = 2 * N * cfg.patch_dim * D
        f["attn_window"] = 0
        f["attn_full"] = 4 * int((tok ** 2).sum()) * D * L
        N = int(tok.sum())
        f["mlp_up"] = 2 * N * D * I * L
        f["mlp_down"] = 2 * N * I * D * L
        f["back"] = 2 * M * 4 * D * cfg.merger_hidden + 2 * M * cfg.merger_hidden * cfg.out_hidden
    else:
        frames = n_item
        N = int(frames.sum()) // 2
        f["front"] = 2 * int(frames.sum()) * 3 * cfg.patch_dim * D + 2 * N * 3 * D * D
        f["attn_window"] = 0
        f["attn_full"] = 4 * int(((frames // 2) ** 2).sum()) * D * L
        f["mlp_up"] = 2 * N * D * I * L
        f["mlp_down"] = 2 * N * I * D * L
        f["back"] = 2 * (N // cfg.merge) * D * cfg.out_hidden
    f["qkv"] = 2 * N * D * 3 * D * L
    f["proj"] = 2 * N * D * D * L
    f["total"] = sum(f.values())
    return f


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "c5", "c6"])
    ap.add_argument("--items", type=int, default=0,
                    help="number of items in the batch (images, clips, tiles) instead of the workload's own")
    ap.add_argument("--breakdown", action="store_true", help="also time every step of the path separately")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step's cs_encode from a recorded HIP graph (cs_encode_graph_*; for small --items)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference reading for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; the encoder task shards by item across replicas "
              "(no collectives), so --gpus N > 1 is not measured here.", file=sys.stderr)
        return 2

    import torch
    from paper_2603_12118_amd import binding as B
    from paper_2603_12118_amd import workloads as wl

    t0 = time.time()
    make = {"c2": wl.c2_images, "c3": wl.c3_varlen, "c4": wl.c4_video, "c5": wl.c5_audio, "c6": wl.c6_tiles}[args.workload]
    size = {{"c2": "n_images", "c3": "n_images", "c4": "n_clips", "c5": "n_clips", "c6": "n_tiles"}[args.workload]: args.items} \
        if args.items > 0 else {}
    w = make(out_dtype="bf16", **size)
    weights = w.weights
    dev = "cuda:0"
    enc = B.Encoder(w.cfg, weights)
    x = torch.from_numpy(wl.to_bits_bf16(w.patches).view(np.int16)).to(dev).view(torch.bfloat16)
    n_out, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    out = torch.empty(n_out, w.cfg.out_hidden, dtype=torch.bfloat16, device=dev)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    dst = torch.from_numpy(w.consumer_buffer_bits().view(np.int16)).to(dev).view(torch.bfloat16)
    idx = torch.from_numpy(w.placeholder_index).to(dev)
    setup_s = time.time() - t0

    graph = None
    if args.graph:
        side = torch.cuda.Stream()
        graph = enc.cs_encode_graph_create(x, w.cu_seqlens, w.grid_thw, out, workspace, side)
        torch.cuda.synchronize()

    def step():
        if graph is not None:
            graph.cs_encode_graph_launch()
        else:
            enc.cs_encode(x, w.cu_seqlens, w.grid_thw, out=out, workspace=workspace)
        B.cs_forward_embeddings(out, idx, dst)

    if args.calibration_copy:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    dominant = "mlp_up"
    # every 8th launch of the dominant kernel is bracketed by a HIP event pair (4 per step): an event
    # pair idles the stream for about 5 us on either side of the launch, 0.36 ms per step if all 32 are timed
    enc.cs_encoder_time_step(B.STEPS[dominant])
    enc.cs_encoder_time_every(8)
    # the K timed steps: wall clock between two synchronisations (`value`), and beside it a HIP event between
    # every two steps on the stream the kernels run on (torch's current stream) for the median step
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    ev_raw = [evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)]
    ev_ms = sorted(ev_raw)
    dom_ms, dom_n = enc.cs_encoder_read_timing()
    enc.cs_encoder_time_step(0)
    enc.cs_encoder_time_every(1)

    # host side of one call: time of the cs_encode + cs_forward_embeddings calls themselves (plan lookup,
    # validation, launches), the stream idle before each
    host_us = []
    for _ in range(10):
        torch.cuda.synchronize()
        th = time.perf_counter()
        step()
        host_us.append((time.perf_counter() - th) * 1e6)
    torch.cuda.synchronize()
    host_us.sort()
    plan_hits, plan_misses = enc.cs_encoder_plan_cache_stats()

    fl = algorithmic_flops(w.cfg, w.grid_thw)
    n_in = int(w.cu_seqlens[-1])
    ms = dt / args.steps * 1e3
    tflops = fl["total"] / (ms * 1e-3) / 1e12
    dom_avg_ms = dom_ms / max(dom_n, 1)
    dom_flops = fl[dominant] / w.cfg.n_layers
    # (a replayed graph carries no timing events: the dominant kernel is then not timed)
    dom_tflops = dom_flops / (dom_avg_ms * 1e-3) / 1e12 if dom_n > 0 else None

    # transformer tokens of the batch: two mel frames per token; a class-token tower adds four rows per tile
    # (class token and three of padding)
    n_tokens = int(w.cu_seqlens[-1])
    if w.cfg.arch == "audio":
        n_tokens //= 2
    elif w.cfg.arch == "vit_cls":
        n_tokens += 4 * w.n_items
    kernel = enc.cs_encoder_step_kernel(B.STEPS[dominant], n_tokens)
    traffic, traffic_src = measured_traffic(w.name, kernel, args.items <= 0)
    res = {
        "metric": "encoder_patches_per_s" if w.cfg.arch != "audio" else "encoder_mel_frames_per_s",
        "value": n_in / (ms * 1e-3), "unit": "patches/s" if w.cfg.arch != "audio" else "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "ms_per_step_median_hip_events": ev_ms[len(ev_ms) // 2], "ms_per_step_min_hip_events": ev_ms[0], "ms_per_step_max_hip_events": ev_ms[-1], "slowest_step": ev_raw.index(ev_ms[-1]),
        "host_us_per_call_median": host_us[len(host_us) // 2], "plan_cache": {"hits": plan_hits, "misses": plan_misses},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "launch": "hip graph replay" if args.graph else "eager", "items": w.n_items, "input_rows": n_in, "embedding_rows": int(n_out),
                   "layers": w.cfg.n_layers, "hidden": w.cfg.hidden, "out_hidden": w.cfg.out_hidden},
        "items_per_s": w.n_items / (ms * 1e-3),
        "algorithmic_tflop_per_step": fl["total"] / 1e12,
        "achieved_tflops": tflops, "frac_of_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "roofline": {"kernel": kernel + (" (gate|up projection + SwiGLU)" if w.cfg.arch == "vit" else " (fc1 + GELU)"),
                     "bound": "mfma",
                     "achieved": dom_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": dom_tflops / PEAK_BF16_TFLOPS if dom_tflops else None, "traffic": traffic, "traffic_source": traffic_src,
                     "avg_launch_ms": dom_avg_ms, "launches_timed": dom_n, "flop_per_launch": dom_flops},
        "setup_s": setup_s,
    }

    # the hand-off on its own: HBM-bound row copy
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(50):
        B.cs_forward_embeddings(out, idx, dst)
    ev1.record()
    torch.cuda.synchronize()
    us = ev0.elapsed_time(ev1) / 50 * 1e3
    bytes_moved = n_out * (2 * w.cfg.out_hidden * 2 + 8)
    res["forward_embeddings"] = {"us_per_call": us, "algorithmic_bytes": bytes_moved,
                                 "achieved_GBs": bytes_moved / (us * 1e-6) / 1e9, "peak_GBs": PEAK_HBM_GBS}

    # what a bare MFMA loop sustains on this board, next to the path's rate: with zero operands (nominal
    # clock) and with random operands (the board at its power limit, as it is during the step)
    res["mfma_ceiling_tflops"] = {"zero_operands": B.cs_mfma_ceiling(False), "random_operands": B.cs_mfma_ceiling(True)}

    if args.breakdown:
        bd = {}
        for name, sid in B.STEPS.items():
            enc.cs_encoder_time_step(sid)
            for _ in range(3):
                step()
            torch.cuda.synchronize()
            t_ms, n = enc.cs_encoder_read_timing()
            bd[name] = {"ms_per_step": t_ms / 3, "launches_per_step": n // 3,
                        "tflops": (fl.get(name, 0) / (t_ms / 3 * 1e-3) / 1e12) if t_ms > 0 and name in fl else None}
        enc.cs_encoder_time_step(0)
        res["breakdown"] = bd

    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import encoder_oracle as O
        one = w.select_items([0, 1] if w.n_items > 1 and w.cfg.arch == "vit" and w.name == "c2_images" else [0])
        tc = time.perf_counter()
        O.encode(one.cfg, weights, one.patches, one.cu_seqlens, one.grid_thw)
        cpu_s = time.perf_counter() - tc
        cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        res["cpu_baseline"] = {"value": int(one.cu_seqlens[-1]) / cpu_s, "unit": res["unit"], "cores": cores,
                               "kind": "oracle", "seconds": cpu_s,
                               "sample": f"{one.n_items} of {w.n_items} items ({int(one.cu_seqlens[-1])} input rows), all "
                                         f"{w.cfg.n_layers} layers, numpy fp64"}
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
