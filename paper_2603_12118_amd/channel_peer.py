"""One side of the two-process hand-off (cs_xchannel_*) as a command loop: started as a child
process (`python -m paper_2603_12118_amd.channel_peer producer|consumer <name>`), it reads one JSON
command per line on stdin and answers one JSON line on stdout.  The GPU tests and the micro-benchmark
drive a producer peer and a consumer peer with it; everything that touches the channel goes through
the C ABI (binding.XChannel), torch only provides device memory and the streams.

Producer commands: create {n_slots, slot_bytes} | acquire {nbytes} | publish {slot, n, hidden, seed, busy}
(the rows are numpy.random.default_rng(seed).integers(0, 65536, (n, hidden), uint16), copied into the slot on
the producer's stream, after `busy` rounds of unrelated work on that stream) | publish_raw {slot, n, hidden}
(publishes whatever the slot holds) | release {slot} | describe {slot} | quit.
Consumer commands: open | buffers {count, rows, hidden, seed} | wait {timeout_us} | forward {slot, dst, index}
| stage_index {index} (uploads placeholder positions ahead of the tensor, as a consumer that knows where its
placeholders are does) | wait_forward {timeout_us, dst} (waits for the next tensor and places it with the staged
index, one command: what a serving consumer does) | describe {slot} | settle {slot, timeout_us} (polls until the
slot is FREE) | dump {path} (buffers as .npy) | flag | quit.
"""
from __future__ import annotations

import json
import sys
import time

import numpy as np


def seeded_rows(seed: int, n: int, hidden: int) -> np.ndarray:
    """The rows a producer peer writes for `seed` (raw bf16 storage words)."""
    return np.random.default_rng(seed).integers(0, 1 << 16, (n, hidden), dtype=np.uint16)


def seeded_buffers(seed: int, count: int, rows: int, hidden: int):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 1 << 16, (rows, hidden), dtype=np.uint16) for _ in range(count)]


def main(role: str, name: str) -> int:
    import torch
    from . import binding as B

    dev = "cuda:0"
    stream = torch.cuda.Stream()
    ch = None
    bufs, flag = [], torch.zeros(1, dtype=torch.int32, device=dev)
    ballast = torch.randn(1024, 1024, device=dev)
    keep, staged = [], None
    torch.cuda.synchronize()
    out = sys.stdout
    print(json.dumps({"ready": role}), file=out, flush=True)
    for line in sys.stdin:
        c = json.loads(line)
        op, r = c["op"], {}
        if op == "quit":
            break
        elif op == "create":
            ch = B.XChannel(name, c["n_slots"], c["slot_bytes"], create=True)
        elif op == "open":
            ch = B.XChannel(name, create=False)
        elif op == "acquire":
            st, slot, ptr = ch.cs_xchannel_acquire(c["nbytes"])
            r = {"st": st, "slot": slot, "ptr": ptr}
        elif op in ("publish", "publish_raw"):
            n, hidden = c["n"], c["hidden"]
            if op == "publish" and n > 0 and c.get("write", True):
                src = torch.from_numpy(seeded_rows(c["seed"], n, hidden).view(np.int16)).to(dev).view(torch.bfloat16)
                torch.cuda.current_stream().synchronize()
                keep.append(src)
                with torch.cuda.stream(stream):
                    x = ballast
                    for _ in range(c.get("busy", 0)):
                        x = x @ x
                        x = x / x.abs().max().clamp_min(1.0)
                    ch.slot_tensor(c["ptr"], n, hidden, torch.bfloat16).copy_(src, non_blocking=True)
            r = {"st": ch.cs_xchannel_publish(c["slot"], n, hidden, B.CS_BF16, stream)}
        elif op == "fill":       # micro-benchmark: a device copy of n rows into the slot, then publish
            n, hidden = c["n"], c["hidden"]
            if not keep or keep[-1].shape != (n, hidden):
                keep.append(torch.randn(n, hidden, device=dev).to(torch.bfloat16))
                torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                ch.slot_tensor(c["ptr"], n, hidden, torch.bfloat16).copy_(keep[-1], non_blocking=True)
            r = {"st": ch.cs_xchannel_publish(c["slot"], n, hidden, B.CS_BF16, stream)}
        elif op == "release":
            r = {"st": ch.cs_xchannel_release(c["slot"])}
        elif op == "describe":
            r = ch.cs_xchannel_describe(c["slot"])
        elif op == "buffers":
            bufs = [torch.from_numpy(b.view(np.int16)).to(dev).view(torch.bfloat16)
                    for b in seeded_buffers(c["seed"], c["count"], c["rows"], c["hidden"])]
            torch.cuda.synchronize()
        elif op == "wait":
            st, slot, rows, hidden, dtype = ch.cs_xchannel_wait(c["timeout_us"])
            r = {"st": st, "slot": slot, "n": rows, "hidden": hidden, "dtype": dtype}
        elif op == "forward":
            idx = torch.tensor(c["index"], dtype=torch.int64, device=dev)
            torch.cuda.current_stream().synchronize()
            keep.append(idx)
            r = {"st": ch.cs_xchannel_forward(c["slot"], idx, bufs[c["dst"]], flag, stream)}
        elif op == "stage_index":
            staged = torch.tensor(c["index"], dtype=torch.int64, device=dev)
            torch.cuda.synchronize()
        elif op == "wait_forward":
            st, slot, rows, hidden, dtype = ch.cs_xchannel_wait(c["timeout_us"])
            r = {"st": st, "slot": slot, "n": rows}
            if st == 0:
                r["st_forward"] = ch.cs_xchannel_forward(slot, staged[:rows], bufs[c["dst"]], flag, stream)
        elif op == "settle":
            t0, state = time.perf_counter(), -1
            while (time.perf_counter() - t0) * 1e6 < c["timeout_us"]:
                state = ch.cs_xchannel_describe(c["slot"])["state"]
                if state == B.CS_XSLOT_FREE:
                    break
                time.sleep(0.0002)
            r = {"state": state}
        elif op == "dump":
            torch.cuda.synchronize()
            np.save(c["path"], np.stack([b.view(torch.int16).cpu().numpy().view(np.uint16) for b in bufs]))
        elif op == "flag":
            torch.cuda.synchronize()
            r = {"flag": int(flag.item())}
        else:
            r = {"error": f"unknown op {op}"}
        print(json.dumps(r), file=out, flush=True)
    torch.cuda.synchronize()
    if ch is not None:
        ch.close()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1], sys.argv[2]))
