"""Writes the expected embedding rows used by the full-size GPU parity tests.

Calls only the CPU checker (oracle/) and the seeded workload generators; nothing here touches the
GPU library.  The encoder treats every item of a batch independently (block-diagonal attention),
so the checker is run on single items of the full-size workloads and a sample of their output
rows is stored; the GPU tests run the whole batch and compare those rows.

    python tests/golden/make_expected.py [c2 c3 c4 c5 c6]

Output: tests/golden/<workload>_item<i>.npz with
    rows   int64 [R]            row numbers inside the item's embedding tensor
    values float32 [R, hidden]  checker output (fp64) rounded to fp32
    max_abs float               largest |value| over the whole item (not only the sample)
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
# workload -> items whose embeddings are stored (c3: the smallest image and a mid-sized one)
ITEMS = {"c2": [0, 5], "c3": None, "c4": [1], "c5": [3], "c6": [0, 6]}
N_ROWS = 12


def sample_rows(n_rows: int, item: int) -> np.ndarray:
    rng = np.random.default_rng(1000 + item)
    extra = rng.choice(n_rows, size=min(N_ROWS - 2, n_rows), replace=False)
    return np.unique(np.concatenate([[0, n_rows - 1], extra])).astype(np.int64)


def c3_items(w) -> list:
    n = w.grid_thw.prod(1)
    order = np.argsort(n)
    return [int(order[0]), int(order[len(order) // 3])]


def main(names):
    for name in names:
        w = {"c2": wl.c2_images, "c3": wl.c3_varlen, "c4": wl.c4_video, "c5": wl.c5_audio,
             "c6": wl.c6_tiles}[name]()
        items = ITEMS[name] if ITEMS[name] is not None else c3_items(w)
        W = w.weights
        for it in items:
            one = w.select_items([it])
            t = time.time()
            y = O.encode(one.cfg, W, one.patches, one.cu_seqlens, one.grid_thw)
            rows = sample_rows(y.shape[0], it)
            path = os.path.join(HERE, f"{name}_item{it}.npz")
            np.savez_compressed(path, rows=rows, values=y[rows].astype(np.float32), max_abs=np.abs(y).max())
            print(f"{name} item {it}: {one.patches.shape[0]} input rows -> {y.shape}, max|y|={np.abs(y).max():.3f}, "
                  f"{time.time() - t:.1f}s -> {path}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or ["c2", "c3", "c4", "c5", "c6"])
