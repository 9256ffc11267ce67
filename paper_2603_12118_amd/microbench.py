"""Micro-benchmarks of the path's kernels on their own, through the C ABI.

    python -m paper_2603_12118_amd.microbench [--json]

* the bare-MFMA ceiling (zero and random operands),
* every GEMM shape of the 7B-style vision layer and of the merger at M = 8192 / 2048 rows with a plain
  bf16 store (`cs_linear_bf16`; the fused epilogues are timed in place by `bench.py --breakdown`),
* `cs_forward_embeddings` at 8, 16 and 32 MB of embedding rows (the tensor sizes for which the paper
  quotes its forwarding latency, Sec. 3 "Sidecar Overhead"),
* the same sizes through `cs_channel` (producer stream -> slot -> consumer stream): the time from
  the end of the producer's last kernel to the rows being in the consumer's buffer, and the host time
  of the three calls,
* the same sizes through `cs_xchannel` (producer PROCESS -> slot in HBM -> consumer PROCESS on the same
  GPU, two child processes started here): the time from the producer's stream having finished its
  work on the slot (its host function) to the placement having finished in the consumer (its host
  function), on the clock both processes share,
* `cs_patchify` on the eight 448x448 images of the benchmark batch.

Attention on its own at segment sizes 64 / 1024 / 8192 is what `bench.py --breakdown` reports as the
window and full layers of `c2_images` (64, 1024) and the full layers of `c4_video` (8192).
Inputs are seeded random bf16 values resident in HBM; times are HIP-event means over 20 launches.
"""
from __future__ import annotations

import argparse
import json

GEMM_SHAPES = [  # (name, M, N, K)
    ("qkv", 8192, 3840, 1280), ("out projection", 8192, 1280, 1280), ("gate|up", 8192, 6912, 1280),
    ("down", 8192, 1280, 3456), ("merger fc1", 2048, 5120, 5120), ("merger fc2", 2048, 3584, 5120),
    ("square", 8192, 8192, 8192),
]


def _time(fn, n=20, warm=3):
    import torch
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n * 1e-3


def _channel(B, src, idx, dst, n=20, warm=3):
    """One tensor after the other through a two-slot channel: the producer (a copy into the slot on
    its stream) publishes, the consumer's stream places.  Returns the mean time between an event
    behind the producer's copy and an event behind the placement, and the host time of
    acquire + publish + forward."""
    import time
    import torch
    rows, hidden = src.shape
    ch = B.Channel(2, src.numel() * 2)
    prod, cons = torch.cuda.Stream(), torch.cuda.Stream()
    pairs, host = [], 0.0
    torch.cuda.synchronize()
    for i in range(warm + n):
        t0 = time.perf_counter()
        _, slot, ptr = ch.cs_channel_acquire(src.numel() * 2, prod)
        t1 = time.perf_counter()
        with torch.cuda.stream(prod):
            ch.slot_tensor(ptr, rows, hidden, torch.bfloat16).copy_(src, non_blocking=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(prod)
        t2 = time.perf_counter()
        ch.cs_channel_publish(slot, rows, hidden, B.CS_BF16, prod)
        ch.cs_channel_forward(slot, idx, dst, None, cons)
        t3 = time.perf_counter()
        e1.record(cons)
        torch.cuda.synchronize()       # one tensor in flight at a time: the latency, not the throughput
        if i >= warm:
            pairs.append(e0.elapsed_time(e1) * 1e3)
            host += (t1 - t0) + (t3 - t2)
    ch.close()
    return {"us_producer_done_to_placed": sum(pairs) / n, "host_us": host / n * 1e6}


def _xchannel(sizes_mb, hidden, n=20):
    """Two child processes (paper_2603_12118_amd.channel_peer) on this GPU, one tensor at a time."""
    import json as J
    import os
    import subprocess
    import sys
    import uuid
    import numpy as np
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    name = "mb" + uuid.uuid4().hex[:10]

    def start(role):
        p = subprocess.Popen([sys.executable, "-u", "-m", "paper_2603_12118_amd.channel_peer", role, name], cwd=root,
                             stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)
        return p

    def call(p, op=None, **kw):
        if op is not None:
            p.stdin.write(J.dumps({"op": op, **kw}) + "\n")
            p.stdin.flush()
        while True:
            line = p.stdout.readline()
            if not line:
                raise RuntimeError("channel peer ended")
            if line.strip().startswith("{"):
                return J.loads(line)

    prod, cons = start("producer"), start("consumer")
    out = []
    try:
        call(prod), call(cons)
        max_rows = max(sizes_mb) * (1 << 20) // (hidden * 2)
        call(prod, "create", n_slots=2, slot_bytes=max_rows * hidden * 2)
        call(cons, "open")
        call(cons, "buffers", count=1, rows=4 * max_rows, hidden=hidden, seed=1)
        rng = np.random.default_rng(0)
        for mb in sizes_mb:
            rows = mb * (1 << 20) // (hidden * 2)
            idx = rng.permutation(4 * max_rows)[:rows].tolist()
            call(cons, "stage_index", index=idx)      # the consumer knows its placeholder positions beforehand
            lat = []
            for i in range(n + 3):
                a = call(prod, "acquire", nbytes=rows * hidden * 2)
                assert a["st"] == 0, a
                # the consumer is already waiting when the producer publishes
                cons.stdin.write(J.dumps({"op": "wait_forward", "timeout_us": 10_000_000, "dst": 0}) + "\n")
                cons.stdin.flush()
                assert call(prod, "fill", slot=a["slot"], ptr=a["ptr"], n=rows, hidden=hidden)["st"] == 0
                w = call(cons)
                assert w["st"] == 0 and w["slot"] == a["slot"] and w["st_forward"] == 0, w
                assert call(cons, "settle", slot=w["slot"], timeout_us=10_000_000)["state"] == 0
                d = call(cons, "describe", slot=w["slot"])
                if i >= 3:
                    lat.append((d["t_placed_ns"] - d["t_ready_ns"]) / 1e3)
            lat.sort()
            out.append({"MB": mb, "rows": rows, "us_median": lat[len(lat) // 2], "us_min": lat[0], "us_max": lat[-1]})
    finally:
        for p in (cons, prod):
            try:
                p.stdin.write(J.dumps({"op": "quit"}) + "\n")
                p.stdin.flush()
                p.wait(timeout=60)
            except Exception:
                p.kill()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    import torch
    from . import binding as B
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(1)
    res = {"mfma_ceiling_tflops": {"zero_operands": B.cs_mfma_ceiling(False), "random_operands": B.cs_mfma_ceiling(True)},
           "gemm": [], "forward_embeddings": [], "channel": []}
    for name, M, N, K in GEMM_SHAPES:
        A = torch.randn(M, K, device=dev, generator=g).bfloat16()
        W = (torch.randn(N, K, device=dev, generator=g) * 0.05).bfloat16()
        out = torch.empty(M, N, device=dev, dtype=torch.bfloat16)
        s = _time(lambda: B.cs_linear_bf16(A, W, None, out))
        res["gemm"].append({"name": name, "M": M, "N": N, "K": K, "us": s * 1e6, "tflops": 2.0 * M * N * K / s / 1e12})
        del A, W, out
    hidden = 3584
    for mb in (8, 16, 32):
        rows = mb * (1 << 20) // (hidden * 2)
        src = torch.randn(rows, hidden, device=dev, generator=g).bfloat16()
        dst = torch.zeros(4 * rows, hidden, device=dev, dtype=torch.bfloat16)
        idx = (torch.randperm(4 * rows, device=dev, generator=g)[:rows]).to(torch.int64)
        s = _time(lambda: B.cs_forward_embeddings(src, idx, dst))
        nbytes = rows * (2 * hidden * 2 + 8)
        res["forward_embeddings"].append({"MB": mb, "rows": rows, "us": s * 1e6, "GBs": nbytes / s / 1e9})
        res["channel"].append({"MB": mb, "rows": rows, **_channel(B, src, idx, dst)})
        del src, dst, idx
    res["xchannel"] = _xchannel((8, 16, 32), hidden)
    px = torch.rand(8 * 3 * 448 * 448, device=dev, generator=g)
    dims = [(1, 448, 448)] * 8
    s = _time(lambda: B.cs_patchify(px, dims, temporal_patch=2))
    nbytes = px.numel() * 4 + 8192 * 1176 * 2
    res["patchify"] = {"workload": "8 x 448x448 fp32 images -> 8192 x 1176 bf16", "us": s * 1e6, "GBs": nbytes / s / 1e9}
    if args.json:
        print(json.dumps(res))
        return 0
    c = res["mfma_ceiling_tflops"]
    print(f"bare MFMA loop: {c['zero_operands']:.0f} TFLOP/s with zero operands, {c['random_operands']:.0f} with random operands")
    print("| GEMM (plain bf16 store) | M | N | K | us | TFLOP/s |\n|---|---|---|---|---|---|")
    for r in res["gemm"]:
        print(f"| {r['name']} | {r['M']} | {r['N']} | {r['K']} | {r['us']:.1f} | {r['tflops']:.0f} |")
    print("| cs_forward_embeddings | rows | us | GB/s |\n|---|---|---|---|")
    for r in res["forward_embeddings"]:
        print(f"| {r['MB']} MB | {r['rows']} | {r['us']:.1f} | {r['GBs']:.0f} |")
    print("| cs_channel (publish -> placed) | rows | us after the producer's last kernel | host us for the 3 calls |\n|---|---|---|---|")
    for r in res["channel"]:
        print(f"| {r['MB']} MB | {r['rows']} | {r['us_producer_done_to_placed']:.1f} | {r['host_us']:.1f} |")
    print("| cs_xchannel (two processes; producer's work done -> placed in the consumer) | rows | us median | min | max |\n|---|---|---|---|---|")
    for r in res["xchannel"]:
        print(f"| {r['MB']} MB | {r['rows']} | {r['us_median']:.1f} | {r['us_min']:.1f} | {r['us_max']:.1f} |")
    r = res["patchify"]
    print(f"cs_patchify, {r['workload']}: {r['us']:.1f} us, {r['GBs']:.0f} GB/s")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
