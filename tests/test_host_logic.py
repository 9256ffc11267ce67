"""CPU-only tests of the library's host side: the shared object loads and exports every entry point the
header declares, and the batch planner (internal token order, windows, output rows, validation) agrees
with brute-force enumeration written here.  No compute call is made (no GPU needed)."""
import ctypes as C
import os
import re
from dataclasses import replace

import numpy as np
import pytest

from oracle import encoder_oracle as O
from paper_2603_12118_amd import binding as B
from paper_2603_12118_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "cornenc.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(cs_[a-z_0-9]+)\s*\(", hdr))
    assert {"cs_encoder_create", "cs_encode", "cs_forward_embeddings", "cs_encoder_query", "cs_encoder_destroy",
            "cs_plan_tokens", "cs_linear_bf16", "cs_attention_varlen", "cs_status_string", "cs_last_error",
            "cs_encoder_time_step", "cs_encoder_read_timing", "cs_mfma_ceiling", "cs_patchify", "cs_pack_batch",
            "cs_encoder_time_every", "cs_channel_create", "cs_channel_destroy", "cs_channel_acquire",
            "cs_channel_publish", "cs_channel_forward", "cs_channel_release", "cs_channel_describe"} <= names
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in cornenc.h but not exported"
    assert B.lib().cs_status_string(0) == b"ok"
    assert C.sizeof(B.cs_encoder_config) == 96


def brute_plan(grid, window, merge=2):
    """Internal order by definition: item, frame, window (row-major), 2x2 group (row-major), patch."""
    src, out_row, win_cu = [], [], [0]
    base = obase = 0
    for (T, h, w) in grid:
        for t in range(T):
            for r0 in range(0, h, window):
                for c0 in range(0, w, window):
                    for R in range(r0, min(r0 + window, h), merge):
                        for Cc in range(c0, min(c0 + window, w), merge):
                            out_row.append(obase + (t * (h // merge) + R // merge) * (w // merge) + Cc // merge)
                            for dr in range(merge):
                                for dc in range(merge):
                                    src.append(base + (t * h + R + dr) * w + Cc + dc)
                    win_cu.append(len(src))
        base += T * h * w
        obase += T * (h // merge) * (w // merge)
    return np.array(src), np.array(out_row), np.array(win_cu)


@pytest.mark.parametrize("grid", [[(1, 4, 4)], [(1, 6, 10)], [(1, 18, 34)], [(3, 10, 12)], [(1, 32, 32)] * 2,
                                  [(1, 84, 36), (1, 24, 40), (2, 2, 2)]])
def test_plan_matches_brute_force_and_checker_geometry(grid):
    cfg = wl.vit_7b_config()
    g = np.array(grid, np.int32)
    cu = np.concatenate([[0], np.cumsum(g.prod(1))]).astype(np.int32)
    src, out_row, win_cu = B.cs_plan_tokens(cfg, cu, g)
    bs, bo, bw = brute_plan(grid, 8)
    assert np.array_equal(src, bs) and np.array_equal(out_row, bo) and np.array_equal(win_cu, bw)
    n = int(cu[-1])
    assert sorted(src.tolist()) == list(range(n))                      # a permutation
    assert sorted(out_row.tolist()) == list(range(n // 4))
    # windows of the plan are exactly the checker's attention classes
    item, pos = O.token_coords(g)
    allowed = O.attention_allowed(item, pos, 8)
    for a, b in zip(win_cu[:-1], win_cu[1:]):
        members = np.sort(src[a:b])
        assert np.array_equal(np.flatnonzero(allowed[members[0]]), members)
    # four consecutive internal tokens feed one merged token, in the checker's concat order
    mi = O.merge_index(g, 2)
    assert np.array_equal(src.reshape(-1, 4), mi[out_row])


def test_plan_random_batches_against_brute_force():
    """Sixty seeded random batches (1-5 items, 1-3 frames, even sides up to 44, window 4 or 8)."""
    from dataclasses import replace
    rng = np.random.default_rng(17)
    for _ in range(60):
        n = int(rng.integers(1, 6))
        grid = [(int(rng.integers(1, 4)), 2 * int(rng.integers(1, 23)), 2 * int(rng.integers(1, 23))) for _ in range(n)]
        win = int(rng.choice([4, 8]))
        g = np.array(grid, np.int32)
        cu = np.concatenate([[0], np.cumsum(g.prod(1))]).astype(np.int32)
        src, out_row, win_cu = B.cs_plan_tokens(replace(wl.vit_7b_config(), window=win), cu, g)
        bs, bo, bw = brute_plan(grid, win)
        assert np.array_equal(src, bs) and np.array_equal(out_row, bo) and np.array_equal(win_cu, bw), (grid, win)


def test_plan_merge_major_input_order():
    """With merge-major input the planner's source rows are the checker's permutation undone: internal
    token i reads input row j where perm[j] is the raster row it would read otherwise."""
    from dataclasses import replace
    grid = [(1, 18, 34), (3, 10, 12), (1, 2, 2)]
    g = np.array(grid, np.int32)
    cu = np.concatenate([[0], np.cumsum(g.prod(1))]).astype(np.int32)
    src_r, out_r, win_r = B.cs_plan_tokens(wl.vit_7b_config(), cu, g)
    src_m, out_m, win_m = B.cs_plan_tokens(replace(wl.vit_7b_config(), input_order="merge_major"), cu, g)
    perm = O.merge_major_order(g, 2)
    assert np.array_equal(perm[src_m], src_r)
    assert np.array_equal(out_m, out_r) and np.array_equal(win_m, win_r)
    bad = replace(wl.audio_config(), input_order="merge_major")
    with pytest.raises(B.CsError):
        B.cs_plan_tokens(bad, [0, 16], [[1, 4, 4]])


def test_plan_full_attention_config_keeps_merge_groups():
    cfg = wl.vit_tiny_config()
    src, out_row, win_cu = B.cs_plan_tokens(cfg, [0, 256], [[1, 16, 16]])
    assert len(win_cu) == 1                                            # no windows
    assert np.array_equal(src.reshape(-1, 4), O.merge_index(np.array([[1, 16, 16]]), 2)[out_row])


def test_plan_of_a_class_token_tower_by_definition():
    """Tiles of 4x6 and 6x4 patches (25 positions each): per tile the patches merge group by merge
    group, then four rows without a source (class token, padding); merged row j feeds output row
    (R, C) of its tile and the row made of the class token and the padding feeds none."""
    cfg = replace(wl.vit_cls_config(2), tile_patches=(4, 6))
    grid = np.array([[1, 4, 6], [1, 6, 4], [1, 4, 6]], np.int32)
    cu = np.array([0, 24, 48, 72], np.int32)
    src, out_row, win_cu = B.cs_plan_tokens(cfg, cu, grid)
    want_src, want_out, base, obase = [], [], 0, 0
    for (_, h, w) in grid.tolist():
        for R in range(h // 2):
            for Cc in range(w // 2):
                want_out.append(obase + R * (w // 2) + Cc)
                want_src += [base + (2 * R + dr) * w + 2 * Cc + dc for dr in (0, 1) for dc in (0, 1)]
        want_src += [-1] * 4
        want_out.append(-1)
        base += h * w
        obase += h * w // 4
    assert src.tolist() == want_src and out_row.tolist() == want_out and len(win_cu) == 1
    # the same groups the checker concatenates: its merge index, tile by tile
    groups = np.array([r for r in src.tolist() if r >= 0]).reshape(-1, 4)
    assert np.array_equal(groups[np.argsort([o for o in out_row.tolist() if o >= 0])],
                          O.merge_index(grid, 2).reshape(-1, 4))
    for bad_grid, bad_cu in (([[1, 4, 6], [1, 4, 4]], [0, 24, 40]),      # a tile that does not fit the position table
                             ([[2, 4, 6]], [0, 48]),                     # t != 1
                             ([[1, 5, 5]], [0, 25])):                    # odd sides
        with pytest.raises(B.CsError):
            B.cs_plan_tokens(cfg, np.array(bad_cu, np.int32), np.array(bad_grid, np.int32))


@pytest.mark.parametrize("cu,grid,status", [
    ([0, 17], [[1, 4, 4]], 2),            # token count does not match the grid
    ([1, 17], [[1, 4, 4]], 2),            # does not start at 0
    ([0, 15], [[1, 3, 5]], 2),            # odd grid
    ([0, 0], [[0, 4, 4]], 2),             # empty item
])
def test_plan_rejects_inconsistent_batches(cu, grid, status):
    with pytest.raises(B.CsError) as e:
        B.cs_plan_tokens(wl.vit_7b_config(), cu, grid)
    assert e.value.status == status and B.last_error()


def test_config_validation_on_host():
    from dataclasses import replace
    bad = replace(wl.vit_7b_config(), head_dim=72, n_heads=16, hidden=1152)
    with pytest.raises(B.CsError) as e:
        B.cs_plan_tokens(bad, [0, 16], [[1, 4, 4]])
    assert e.value.status == 5
    bad = replace(wl.vit_7b_config(), rope_sections=(0, 20, 19))
    with pytest.raises(B.CsError):
        B.cs_plan_tokens(bad, [0, 16], [[1, 4, 4]])


def test_forward_embeddings_argument_errors_need_no_gpu():
    assert B.cs_forward_embeddings_raw(16, 16, 16, -1, 4, 8, B.CS_BF16) == 1       # negative size
    assert B.cs_forward_embeddings_raw(16, 16, 16, 4, 4, 7, B.CS_BF16) == 5        # 14-byte rows
    assert B.cs_forward_embeddings_raw(16, 16, 16, 4, 4, 8, 9) == 1                # bad dtype
    assert B.cs_forward_embeddings_raw(8, 16, 16, 4, 4, 8, B.CS_BF16) == 1         # misaligned src
    assert B.cs_forward_embeddings_raw(0, 0, 0, 0, 4, 8, B.CS_BF16) == 0           # empty: no-op


def test_channel_argument_errors_need_no_gpu():
    L, h, slot, ptr = B.lib(), C.c_void_p(), C.c_int32(7), C.c_void_p(5)
    assert L.cs_channel_create(0, 1 << 20, C.byref(h)) == B.CS_ERR_INVALID_ARG          # no slots
    assert L.cs_channel_create(1025, 1 << 20, C.byref(h)) == B.CS_ERR_INVALID_ARG       # too many slots
    assert L.cs_channel_create(2, 0, C.byref(h)) == B.CS_ERR_INVALID_ARG                # empty slots
    assert L.cs_channel_create(2, 1 << 20, None) == B.CS_ERR_INVALID_ARG
    assert not h.value
    assert L.cs_channel_acquire(None, 16, None, C.byref(slot), C.byref(ptr)) == B.CS_ERR_INVALID_ARG
    assert L.cs_channel_publish(None, 0, 1, 8, B.CS_BF16, None) == B.CS_ERR_INVALID_ARG
    assert L.cs_channel_forward(None, 0, None, None, 4, None, None) == B.CS_ERR_INVALID_ARG
    assert L.cs_channel_release(None, 0, None) == B.CS_ERR_INVALID_ARG
    assert L.cs_channel_describe(None, 0, None, None, None, None, None, None) == B.CS_ERR_INVALID_ARG
    assert b"NULL channel" in L.cs_last_error()
    L.cs_channel_destroy(None)                                                           # a no-op
    assert L.cs_status_string(B.CS_ERR_BUSY) == b"busy"


def test_pack_batch_matches_the_checker_and_feeds_the_planner():
    rng = np.random.default_rng(9)
    for _ in range(100):
        n = int(rng.integers(1, 10))
        grid = np.stack([rng.integers(1, 3, n), 2 * rng.integers(1, 12, n), 2 * rng.integers(1, 12, n)], 1).astype(np.int32)
        rows = grid.prod(1).tolist()
        budget, cap = int(rng.integers(1, 600)), int(rng.integers(1, 6))
        sel, cu, pg = B.cs_pack_batch(grid, budget, cap)
        assert sel.tolist() == O.pack_batch(rows, budget, cap)
        assert np.array_equal(pg, grid[sel]) and cu.tolist() == [0] + np.cumsum(grid[sel].prod(1)).tolist()
        src, out_row, win_cu = B.cs_plan_tokens(wl.vit_7b_config(), cu, pg)          # a batch cs_encode accepts
        assert len(src) == cu[-1]
    with pytest.raises(B.CsError):
        B.cs_pack_batch([[1, 0, 4]], 100)
    with pytest.raises(B.CsError):
        B.cs_pack_batch([[1, 4, 4]], 0)


def test_patchify_argument_errors_need_no_gpu():
    L = B.lib()
    i32p = C.POINTER(C.c_int32)
    def dims(*d):
        a = np.array(d, np.int32)
        return a, a.ctypes.data_as(i32p)
    a, p = dims(1, 30, 28)
    assert L.cs_patchify(16, B.CS_F32, p, 1, 2, 14, 32, B.CS_BF16, None, None, None) == 2           # side not a multiple of 14
    a, p = dims(3, 28, 28)
    assert L.cs_patchify(16, B.CS_F32, p, 1, 2, 14, 32, B.CS_BF16, None, None, None) == 2           # 3 frames, temporal patch 2
    a, p = dims(1, 28, 28)
    assert L.cs_patchify(16, 7, p, 1, 2, 14, 32, B.CS_BF16, None, None, None) == 1                  # dtype
    assert L.cs_patchify(8, B.CS_F32, p, 1, 2, 14, 32, B.CS_BF16, None, None, None) == 1            # misaligned frames
    assert L.cs_patchify(16, B.CS_F32, p, 1, 2, 13, 32, B.CS_BF16, None, None, None) == 1           # odd patch size
    assert L.cs_patchify(16, B.CS_F32, p, 0, 2, 14, 32, B.CS_BF16, None, None, None) == 1           # no items
    assert "cs_patchify" in B.last_error()


def test_mfma_ceiling_argument_errors_need_no_gpu():
    out = C.c_double(0.0)
    assert B.lib().cs_mfma_ceiling(None, 1 << 20, 0, 10, C.byref(out), None) == 1       # no scratch
    assert B.lib().cs_mfma_ceiling(16, 1024, 0, 10, C.byref(out), None) == 1             # scratch too small
    assert B.lib().cs_mfma_ceiling(16, 1 << 20, 0, 0, C.byref(out), None) == 1           # no iterations


def test_flop_model_matches_hand_count():
    import bench
    f = bench.algorithmic_flops(wl.vit_7b_config(), np.array([[1, 32, 32]] * 8))
    n, d, i = 8192, 1280, 3420
    lin = 2 * n * 1176 * d + 32 * (2 * n * d * 3 * d + 2 * n * d * d + 3 * 2 * n * d * i) + \
        2 * 2048 * 5120 * 5120 + 2 * 2048 * 5120 * 3584
    att = 28 * 4 * (8 * 16 * 64 ** 2) * d + 4 * 4 * (8 * 1024 ** 2) * d
    assert f["total"] == lin + att
    assert abs(f["total"] / 1e12 - 10.78) < 0.01
