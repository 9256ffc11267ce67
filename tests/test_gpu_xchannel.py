"""GPU test of the two-process hand-off (cs_xchannel_*): a producer process and a consumer process on
the one GPU, each a fresh child that imports the library and talks to it through the C ABI
(paper_2603_12118_amd/channel_peer.py); this test drives them with a seeded sequence of calls and
compares every status and slot number, and at the end every bit of the consumer's buffers, with the
sequential model in the oracle (oracle.ChannelModel).

The model is sequential: a call's effect is complete when it returns.  Across processes the slot
becomes READY when the producer's GPU work is done and FREE when the consumer's scatter is done, so
the driver lets the consumer wait for the notification after every publish (with the producer's
stream kept busy before some of them: the tensor has then not arrived when the wait starts) and
lets a placement settle before the next call."""
import json
import os
import subprocess
import sys
import uuid

import numpy as np
import pytest

from oracle import encoder_oracle as O
from paper_2603_12118_amd import channel_peer as P

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
STATUS = {0: "ok", 1: "invalid", 2: "shape", 3: "workspace", 8: "busy", 10: "timeout"}
WAIT_US = 20_000_000


class Peer:
    def __init__(self, role, name):
        self.p = subprocess.Popen([sys.executable, "-u", "-m", "paper_2603_12118_amd.channel_peer", role, name],
                                  cwd=ROOT, stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True)
        assert self._read()["ready"] == role

    def _read(self):
        while True:
            line = self.p.stdout.readline()
            assert line, "peer process ended"
            line = line.strip()
            if line.startswith("{"):
                return json.loads(line)

    def __call__(self, op, **kw):
        self.p.stdin.write(json.dumps({"op": op, **kw}) + "\n")
        self.p.stdin.flush()
        return self._read()

    def quit(self):
        try:
            self.p.stdin.write(json.dumps({"op": "quit"}) + "\n")
            self.p.stdin.flush()
            self.p.wait(timeout=60)
        finally:
            if self.p.poll() is None:
                self.p.kill()


@pytest.mark.parametrize("seed", [0, 1])
def test_two_processes_replay_the_sequential_model(seed, tmp_path):
    rng = np.random.default_rng(100 + seed)
    hidden, max_rows, n_slots, n_dst, dst_rows = 256, 96, 3, 4, 400
    slot_bytes = max_rows * hidden * 2
    name = "t" + uuid.uuid4().hex[:12]
    model = O.ChannelModel(n_slots, slot_bytes)
    dst = P.seeded_buffers(7 + seed, n_dst, dst_rows, hidden)
    prod, cons = Peer("producer", name), Peer("consumer", name)
    try:
        prod("create", n_slots=n_slots, slot_bytes=slot_bytes)
        cons("open")
        cons("buffers", count=n_dst, rows=dst_rows, hidden=hidden, seed=7 + seed)
        held = {}        # slot -> [state, device address, reserved bytes, rows published]
        n_forwards = 0
        for step in range(70):
            op = rng.choice(["acquire", "publish", "forward", "release", "bad"], p=[0.3, 0.3, 0.3, 0.05, 0.05])
            if op == "acquire":
                nbytes = int(rng.integers(1, max_rows + 1)) * hidden * 2 if rng.random() < 0.9 else slot_bytes + 1
                r = prod("acquire", nbytes=nbytes)
                want = model.acquire(nbytes)
                assert (STATUS[r["st"]], r["slot"]) == want, (step, op)
                if r["st"] == 0:
                    held[r["slot"]] = ["writing", r["ptr"], nbytes, 0]
            elif op == "publish":
                cands = [s for s, h in held.items() if h[0] == "writing"]
                if not cands:
                    continue
                slot = int(rng.choice(cands))
                cap = held[slot][2] // (hidden * 2)
                n = int(rng.integers(0, cap + 1)) if rng.random() < 0.9 else cap + 1
                rows_seed = 1000 * seed + step
                want = model.publish(slot, P.seeded_rows(rows_seed, n, hidden))
                r = prod("publish", slot=slot, ptr=held[slot][1], n=n, hidden=hidden, seed=rows_seed,
                         write=(want == "ok"), busy=int(rng.integers(0, 3)) * 8)
                assert STATUS[r["st"]] == want, (step, op)
                if r["st"] == 0:
                    # the consumer waits for the tensor to arrive, and is told which slot and what it holds
                    w = cons("wait", timeout_us=WAIT_US)
                    assert (STATUS[w["st"]], w["slot"], w["n"], w["hidden"]) == ("ok", slot, n, hidden), (step, w)
                    held[slot][0], held[slot][3] = "ready", n
            elif op == "forward":
                cands = [s for s, h in held.items() if h[0] == "ready"]
                if not cands:
                    continue
                slot = int(rng.choice(cands))
                n, j = held[slot][3], int(rng.integers(0, n_dst))
                idx = rng.permutation(dst_rows)[:n].astype(np.int64)
                idx[rng.random(n) < 0.1] = -1
                r = cons("forward", slot=slot, dst=j, index=idx.tolist())
                want, dst[j] = model.forward(slot, idx, dst[j])
                assert STATUS[r["st"]] == want == "ok", (step, op)
                assert cons("settle", slot=slot, timeout_us=WAIT_US)["state"] == 0
                del held[slot]
                n_forwards += 1
            elif op == "release":
                cands = [s for s, h in held.items() if h[0] == "writing"]
                slot = int(rng.choice(cands)) if cands else int(rng.integers(0, n_slots))
                if slot in held and held[slot][0] == "ready":
                    continue
                r = prod("release", slot=slot)
                assert STATUS[r["st"]] == model.release(slot), (step, op)
                held.pop(slot, None)
            else:
                # calls on slots in the wrong state or that do not exist change nothing
                slot = int(rng.integers(-1, n_slots + 1))
                if slot in held and held[slot][0] == "ready":
                    continue
                idx = [0]
                r = cons("forward", slot=slot, dst=0, index=idx)
                want, _ = model.forward(slot, np.asarray(idx), dst[0])
                assert STATUS[r["st"]] == want == "invalid", (step, op)
        assert n_forwards >= 5
        assert cons("wait", timeout_us=0)["st"] == 10          # nothing is queued any more
        assert cons("flag")["flag"] == 0
        path = str(tmp_path / "bufs.npy")
        cons("dump", path=path)
        got = np.load(path)
        for j in range(n_dst):
            assert np.array_equal(got[j], dst[j]), f"consumer buffer {j} differs from the model"
    finally:
        cons.quit()
        prod.quit()
