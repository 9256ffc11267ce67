"""Writes the expected embeddings used by the full-size GPU parity tests: EVERY output row of the
items it runs.

Calls only the CPU checker (oracle/) and the seeded workload generators; nothing here touches the
GPU library.  The encoder treats every item of a batch independently (block-diagonal attention in
every layer; the paper's shared encoders rest on the same independence, Sec. 2.2 "Component
Sharing"), so the checker is run on single items of the full-size workloads; the GPU tests run the
whole batch and compare all rows of those items.

    python tests/golden/make_expected.py [c2 c3 c4 c5 c6] [--force]

Items: c2 images 0 and 5; c3 the smallest, the largest and the median image plus four drawn with
numpy.random.default_rng(7); c4 clip 1; c5 clip 3; c6 tiles 0 and 6.

Output: tests/golden/<workload>_item<i>.npz with
    q        int16 [rows, hidden]  checker output (fp64) in fixed point: value = q * STEP, STEP = 2^-11;
                                   rounding to the nearest step moves a value by at most STEP/2 =
                                   2.44e-4, which the tests subtract from their bar (fp32 would double
                                   the size of these files to no purpose: the bar is 3e-2)
    step     float                 STEP
    max_abs  float                 largest |value| of the item
A file that exists is kept unless --force is given.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import encoder_oracle as O                      # noqa: E402
from paper_2603_12118_amd import workloads as wl            # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
STEP = 2.0 ** -11
ITEMS = {"c2": [0, 5], "c3": None, "c4": [1], "c5": [3], "c6": [0, 6]}


def c3_items(w) -> list:
    """Smallest, largest and median item by patch count, and four more drawn without replacement."""
    n = w.grid_thw.prod(1)
    order = np.argsort(n, kind="stable")
    fixed = [int(order[0]), int(order[-1]), int(order[len(order) // 2])]
    rest = [i for i in range(len(n)) if i not in fixed]
    extra = np.random.default_rng(7).choice(rest, size=4, replace=False)
    return fixed + sorted(int(i) for i in extra)


def main(names, force):
    for name in names:
        w = {"c2": wl.c2_images, "c3": wl.c3_varlen, "c4": wl.c4_video, "c5": wl.c5_audio,
             "c6": wl.c6_tiles}[name]()
        items = ITEMS[name] if ITEMS[name] is not None else c3_items(w)
        print(f"{name}: items {items}", flush=True)
        W = None
        for it in items:
            path = os.path.join(HERE, f"{name}_item{it}.npz")
            if os.path.exists(path) and not force:
                print(f"{name} item {it}: kept {path}", flush=True)
                continue
            if W is None:
                W = w.weights
            one = w.select_items([it])
            t = time.time()
            y = O.encode(one.cfg, W, one.patches, one.cu_seqlens, one.grid_thw)
            m = float(np.abs(y).max())
            assert m * (1.0 / STEP) < 32767, f"|y| = {m} does not fit the fixed-point range"
            q = np.rint(y / STEP).astype(np.int16)
            assert np.abs(q * STEP - y).max() <= STEP / 2 + 1e-12
            np.savez_compressed(path, q=q, step=STEP, max_abs=m)
            print(f"{name} item {it}: {one.patches.shape[0]} input rows -> {y.shape}, max|y|={m:.3f}, "
                  f"{time.time() - t:.1f}s -> {path}", flush=True)


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--force"]
    main(args or ["c2", "c3", "c4", "c5", "c6"], "--force" in sys.argv[1:])
