"""Pins for the CPU checker: every operator of oracle/encoder_oracle.py is compared with
something other than itself -- a CPU PyTorch library routine, a closed form, an
invariant, a brute-force loop, or indices worked out by hand.  The paper prints no
worked numeric example for the encoder task (it fixes only the task boundary, Sec. 2.2
and Listing 1), so none of these values comes from the paper.
"""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import encoder_oracle as O
from paper_2603_12118_amd import workloads as wl

RNG = np.random.default_rng(1234)
T64 = lambda a: torch.tensor(np.asarray(a, np.float64))


# ------------------------------------------------------------------ elementwise / norms
def test_linear_matches_loop():
    x, W, b = RNG.standard_normal((3, 5)), RNG.standard_normal((4, 5)), RNG.standard_normal(4)
    y = O.linear(x, W, b)
    for i in range(3):
        for o in range(4):
            assert abs(y[i, o] - (sum(x[i, k] * W[o, k] for k in range(5)) + b[o])) < 1e-12


def test_silu_gelu_scalar_forms():
    z = np.linspace(-6, 6, 41)
    assert np.allclose(O.gelu(z), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in z], atol=1e-15)
    assert np.allclose(O.silu(z), F.silu(T64(z)).numpy(), atol=1e-15)
    assert np.allclose(O.gelu(z), F.gelu(T64(z)).numpy(), atol=1e-14)
    assert O.gelu(np.array([0.0]))[0] == 0 and abs(O.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15


def test_rmsnorm_invariants_and_library():
    x, g = RNG.standard_normal((7, 48)), 1 + 0.1 * RNG.standard_normal(48)
    y1 = O.rmsnorm(x, np.ones(48), 0.0)
    assert np.allclose((y1 ** 2).mean(1), 1.0, atol=1e-12)            # unit mean square
    assert np.allclose(O.rmsnorm(3.7 * x, g, 0.0), O.rmsnorm(x, g, 0.0), atol=1e-12)  # scale invariance
    assert np.allclose(O.rmsnorm(x, g, 1e-6), F.rms_norm(T64(x), (48,), T64(g), 1e-6).numpy(), atol=1e-12)
    # eps matters on a tiny row: closed form
    xr = np.full((1, 4), 1e-3)
    assert np.allclose(O.rmsnorm(xr, np.ones(4), 1e-6), 1e-3 / math.sqrt(1e-6 + 1e-6), atol=1e-12)


def test_layernorm_library():
    x, g, b = RNG.standard_normal((5, 32)) * 3 + 1, RNG.standard_normal(32), RNG.standard_normal(32)
    assert np.allclose(O.layernorm(x, g, b, 1e-5), F.layer_norm(T64(x), (32,), T64(g), T64(b), 1e-5).numpy(),
                       atol=1e-12)


# ------------------------------------------------------------------ geometry
def test_token_coords_raster_by_hand():
    item, pos = O.token_coords(np.array([[1, 2, 3], [2, 2, 2]]))
    assert item.tolist() == [0] * 6 + [1] * 8
    assert pos[:6].tolist() == [[0, 0, 0], [0, 0, 1], [0, 0, 2], [0, 1, 0], [0, 1, 1], [0, 1, 2]]
    assert pos[6:].tolist() == [[0, 0, 0], [0, 0, 1], [0, 1, 0], [0, 1, 1],
                                [1, 0, 0], [1, 0, 1], [1, 1, 0], [1, 1, 1]]


@pytest.mark.parametrize("grid", [[[1, 4, 4]], [[1, 6, 10]], [[1, 18, 34]], [[3, 10, 12]], [[1, 4, 6], [2, 10, 4]]])
def test_window_mask_is_a_partition_with_hand_sizes(grid):
    g = np.array(grid)
    item, pos = O.token_coords(g)
    A = O.attention_allowed(item, pos, 8)
    n = len(item)
    assert (A == A.T).all() and A.diagonal().all()
    # equivalence relation: rows are either identical or disjoint
    classes = {tuple(np.flatnonzero(A[i])) for i in range(n)}
    assert sum(len(c) for c in classes) == n
    sizes = sorted(len(c) for c in classes)
    expect = []
    for (T, h, w) in grid:
        hs = [8] * (h // 8) + ([h % 8] if h % 8 else [])
        ws = [8] * (w // 8) + ([w % 8] if w % 8 else [])
        expect += [a * b for a in hs for b in ws] * T
    assert sizes == sorted(expect)
    # brute-force predicate
    for i in range(0, n, max(1, n // 37)):
        for j in range(0, n, max(1, n // 41)):
            ok = (item[i] == item[j] and pos[i, 0] == pos[j, 0] and pos[i, 1] // 8 == pos[j, 1] // 8
                  and pos[i, 2] // 8 == pos[j, 2] // 8)
            assert A[i, j] == ok


def test_window_covering_grid_equals_full():
    item, pos = O.token_coords(np.array([[1, 6, 8], [1, 4, 4]]))
    assert (O.attention_allowed(item, pos, 8) == O.attention_allowed(item, pos, 0)).all()
    # ... but not across frames of a clip
    item, pos = O.token_coords(np.array([[2, 4, 4]]))
    assert O.attention_allowed(item, pos, 8).sum() == 2 * 16 * 16
    assert O.attention_allowed(item, pos, 0).sum() == 32 * 32


def test_edge_window_sizes_18x34_by_hand():
    # 18 rows -> windows of 8, 8, 2 rows; 34 cols -> 8, 8, 8, 8, 2
    item, pos = O.token_coords(np.array([[1, 18, 34]]))
    A = O.attention_allowed(item, pos, 8)
    assert A[0].sum() == 64                     # top-left window
    assert A[33].sum() == 8 * 2                 # (0,33): last column strip, 8 rows x 2 cols
    assert A[17 * 34].sum() == 2 * 8            # (17,0): last row strip
    assert A[17 * 34 + 33].sum() == 4           # bottom-right corner 2x2


# ------------------------------------------------------------------ rotary
def test_rotary_angle_table_by_hand():
    pos = np.array([[3, 5, 7]])
    ang = O.rotary_angles(pos, (2, 2, 4), 100.0)
    expect = [3, 3 * 100 ** -0.5, 5, 5 * 100 ** -0.5, 7, 7 * 100 ** -0.25, 7 * 100 ** -0.5, 7 * 100 ** -0.75]
    assert np.allclose(ang[0], expect, atol=1e-12)


def test_rotary_identity_norm_and_shift_invariance():
    nh, dh = 2, 16
    q, k = RNG.standard_normal((6, nh, dh)), RNG.standard_normal((6, nh, dh))
    pos = RNG.integers(0, 30, (6, 3))
    sec = (2, 3, 3)
    a0 = O.rotary_angles(np.zeros((6, 3), int), sec, 10000.0)
    assert np.array_equal(O.apply_rotary(q, a0), q)                       # position 0 = identity
    a = O.rotary_angles(pos, sec, 10000.0)
    qr, kr = O.apply_rotary(q, a), O.apply_rotary(k, a)
    half = dh // 2
    assert np.allclose(qr[..., :half] ** 2 + qr[..., half:] ** 2, q[..., :half] ** 2 + q[..., half:] ** 2)
    a2 = O.rotary_angles(pos + np.array([4, 9, 2]), sec, 10000.0)        # shift every token alike
    qr2, kr2 = O.apply_rotary(q, a2), O.apply_rotary(k, a2)
    s1 = np.einsum("ihd,jhd->hij", qr, kr)
    s2 = np.einsum("ihd,jhd->hij", qr2, kr2)
    assert np.allclose(s1, s2, atol=1e-9)
    # temporal section untouched when t == 0
    pos0 = pos.copy(); pos0[:, 0] = 0
    q0 = O.apply_rotary(q, O.rotary_angles(pos0, sec, 10000.0))
    assert np.array_equal(q0[..., :2], q[..., :2]) and np.array_equal(q0[..., half:half + 2], q[..., half:half + 2])


def test_rotary_matches_complex_rotation():
    # pair (x_j, x_{j+dh/2}) is the complex number x_j + i x_{j+dh/2} multiplied by e^{i angle}
    dh = 8
    x = RNG.standard_normal((5, 1, dh))
    ang = RNG.standard_normal((5, dh // 2))
    z = (x[:, 0, :4] + 1j * x[:, 0, 4:]) * np.exp(1j * ang)
    y = O.apply_rotary(x, ang)[:, 0]
    assert np.allclose(y[:, :4], z.real) and np.allclose(y[:, 4:], z.imag)


# ------------------------------------------------------------------ attention
def test_attention_matches_sdpa_with_mask():
    item, pos = O.token_coords(np.array([[1, 10, 12], [1, 4, 6]]))
    n = len(item)
    q, k, v = (RNG.standard_normal((n, 3, 16)) for _ in range(3))
    for win in (0, 8):
        A = O.attention_allowed(item, pos, win)
        mine = O.attention(q, k, v, A)
        ref = F.scaled_dot_product_attention(T64(q).permute(1, 0, 2)[None], T64(k).permute(1, 0, 2)[None],
                                             T64(v).permute(1, 0, 2)[None], attn_mask=torch.tensor(A)[None, None])
        assert np.allclose(mine, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_attention_brute_force_and_constant_v():
    n, dh = 9, 4
    q, k, v = (RNG.standard_normal((n, 1, dh)) for _ in range(3))
    A = RNG.random((n, n)) < 0.5
    A |= np.eye(n, dtype=bool)
    out = O.attention(q, k, v, A)
    for i in range(n):
        w = np.array([math.exp(float(q[i, 0] @ k[j, 0]) / math.sqrt(dh)) if A[i, j] else 0.0 for j in range(n)])
        w /= w.sum()
        assert np.allclose(out[i, 0], sum(w[j] * v[j, 0] for j in range(n)), atol=1e-12)
    vc = np.tile(np.array([1.0, -2.0, 3.0, 0.5]), (n, 1, 1))
    assert np.allclose(O.attention(q, k, vc, A), vc, atol=1e-12)


def test_window_attention_equals_per_window_sdpa():
    """A grid that is a multiple of the window: cut it into windows by reshaping (no mask) and
    run the library attention on each window separately."""
    h, w, nh, dh = 16, 24, 2, 8
    item, pos = O.token_coords(np.array([[1, h, w]]))
    q, k, v = (RNG.standard_normal((h * w, nh, dh)) for _ in range(3))
    mine = O.attention(q, k, v, O.attention_allowed(item, pos, 8))

    def cut(a):  # [h*w, nh, dh] -> [windows, nh, 64, dh]
        a = T64(a).reshape(h // 8, 8, w // 8, 8, nh, dh).permute(0, 2, 4, 1, 3, 5)
        return a.reshape(-1, nh, 64, dh)

    ref = F.scaled_dot_product_attention(cut(q), cut(k), cut(v))
    ref = ref.reshape(h // 8, w // 8, nh, 8, 8, dh).permute(0, 3, 1, 4, 2, 5).reshape(h * w, nh, dh)
    assert np.allclose(mine, ref.numpy(), atol=1e-12)


# ------------------------------------------------------------------ patches, merger
def test_patchify_element_order_by_hand():
    img = np.arange(3 * 28 * 28, dtype=np.float32).reshape(1, 3, 28, 28)
    p, grid = wl.patchify(img, 1)
    assert grid == (1, 2, 2) and p.shape == (4, 588)
    # patch (r=1,c=0), channel 2, py=3, px=5 -> pixel (2, 14+3, 5)
    assert p[2, 2 * 196 + 3 * 14 + 5] == img[0, 2, 17, 5]
    p2, _ = wl.patchify(img, 2)                     # single frame shown twice
    assert p2.shape == (4, 1176)
    assert p2[3, 1 * 392 + 0 * 196 + 13 * 14 + 13] == img[0, 1, 27, 27]
    assert p2[3, 1 * 392 + 1 * 196 + 13 * 14 + 13] == img[0, 1, 27, 27]


def test_oracle_patchify_by_hand_brute_force_and_against_the_input_recipe():
    """oracle.patchify: hand-computed elements, an element-by-element loop written here, and the
    reshape/transposition the input generator uses (a different construction of the same layout)."""
    img = np.arange(3 * 28 * 42, dtype=np.float32).reshape(1, 3, 28, 42)
    p, grid = O.patchify(img, 1)
    assert grid == (1, 2, 3) and p.shape == (6, 588)
    assert p[3, 2 * 196 + 3 * 14 + 5] == img[0, 2, 14 + 3, 5]            # patch (r=1,c=0)
    assert p[5, 0 * 196 + 13 * 14 + 13] == img[0, 0, 27, 41]             # last pixel of channel 0
    p2, _ = O.patchify(img, 2)                                           # single frame shown twice
    assert p2[4, 1 * 392 + 0 * 196 + 2 * 14 + 1] == p2[4, 1 * 392 + 1 * 196 + 2 * 14 + 1] == img[0, 1, 16, 15]
    clip = RNG.random((4, 3, 28, 28)).astype(np.float32)                 # two temporal patches
    pc, g = O.patchify(clip, 2)
    assert g == (2, 2, 2)
    for t in range(2):
        for r in range(2):
            for c in range(2):
                for ch in range(3):
                    for tt in range(2):
                        for py in (0, 7, 13):
                            for px in (0, 6, 13):
                                assert pc[(t * 2 + r) * 2 + c, ((ch * 2 + tt) * 14 + py) * 14 + px] == \
                                    clip[2 * t + tt, ch, 14 * r + py, 14 * c + px]
    for fr, tp in ((img, 1), (img, 2), (clip, 2), (clip, 1)):
        a, ga = O.patchify(fr, tp)
        b, gb = wl.patchify(fr, tp)
        assert ga == gb and np.array_equal(a, b)
    # every pixel appears exactly once per temporal slot it is shown in
    assert np.array_equal(np.sort(O.patchify(img, 1)[0].ravel()), np.sort(img.ravel()))


def test_merge_major_order_is_the_merge_index_flattened_and_by_hand():
    g = np.array([[1, 4, 6], [2, 2, 4]])
    perm = O.merge_major_order(g, 2)
    assert sorted(perm.tolist()) == list(range(24 + 16))                     # a permutation
    assert perm[:8].tolist() == [0, 1, 6, 7, 2, 3, 8, 9]                     # first two groups of a 4x6 grid
    assert perm[24:32].tolist() == [24, 25, 28, 29, 26, 27, 30, 31]          # second item, frame 0
    # the merged token m of the merger reads exactly the four consecutive merge-major rows 4m..4m+3
    assert np.array_equal(perm.reshape(-1, 4), O.merge_index(g, 2))
    # numpy view construction of the same order
    for (T, h, w), off in ((g[0], 0), (g[1], 24)):
        idx = np.arange(T * h * w).reshape(T, h // 2, 2, w // 2, 2).transpose(0, 1, 3, 2, 4).ravel() + off
        assert np.array_equal(perm[off:off + T * h * w], idx)


def test_audio_chunk_mask_by_loops_and_per_chunk_sdpa():
    """Chunked audio attention: the mask against a double loop written here, its class sizes by hand,
    and attention under it against PyTorch SDPA run chunk by chunk."""
    lens, chunk = [20, 12], 8
    m = O.audio_attention_allowed(lens, chunk)
    starts = [0, 20]
    for p in range(32):
        for q in range(32):
            ip, iq = int(p >= 20), int(q >= 20)
            want = ip == iq and (p - starts[ip]) // chunk == (q - starts[iq]) // chunk
            assert m[p, q] == want
    assert m.sum(1).tolist() == [8] * 16 + [4] * 4 + [8] * 8 + [4] * 4       # chunks 8,8,4 | 8,4
    assert np.array_equal(O.audio_attention_allowed(lens, 0), O.audio_attention_allowed(lens, 64))
    q, k, v = (RNG.standard_normal((32, 3, 16)) for _ in range(3))
    mine = O.attention(q, k, v, m)
    for a, b in ((0, 8), (8, 16), (16, 20), (20, 28), (28, 32)):
        ref = F.scaled_dot_product_attention(T64(q[a:b]).transpose(0, 1), T64(k[a:b]).transpose(0, 1),
                                             T64(v[a:b]).transpose(0, 1)).transpose(0, 1)
        assert np.allclose(mine[a:b], ref.numpy(), atol=1e-12)


def test_pack_batch_by_hand_and_by_its_defining_properties():
    assert O.pack_batch([100, 900, 50, 60, 10], 200, 10) == [0, 2, 4]        # 900 and then 60 do not fit
    assert O.pack_batch([500, 10], 200, 10) == [0]                           # oldest alone over budget; 10 would exceed it further
    assert O.pack_batch([10, 10, 10, 10], 1000, 2) == [0, 1]                 # item limit
    assert O.pack_batch([200], 200, 1) == [0]
    rng = np.random.default_rng(5)
    for _ in range(200):
        rows = rng.integers(1, 400, size=rng.integers(1, 12)).tolist()
        budget, cap = int(rng.integers(1, 900)), int(rng.integers(1, 8))
        sel = O.pack_batch(rows, budget, cap)
        assert sel[0] == 0 and sel == sorted(set(sel)) and len(sel) <= cap
        tot = 0
        for i in range(len(rows)):                     # replay: an item is left out only if it did not fit then, or the cap was reached
            if i in sel:
                tot += rows[i]
                assert i == 0 or tot <= budget
            elif sum(1 for j in sel if j < i) < cap:
                assert tot + rows[i] > budget


def test_duplicated_frame_patch_embed_collapses():
    """With both temporal slots showing the same frame, the 1176-wide patch embedding equals a
    588-wide one whose weight is the sum over the temporal axis."""
    img = RNG.random((1, 3, 28, 42)).astype(np.float32)
    p2, _ = wl.patchify(img, 2)
    p1, _ = wl.patchify(img, 1)
    W = RNG.standard_normal((6, 1176))
    Wsum = W.reshape(6, 3, 2, 196).sum(2).reshape(6, 588)
    assert np.allclose(O.linear(p2, W), O.linear(p1, Wsum), atol=1e-9)


def test_merge_index_by_hand():
    mi = O.merge_index(np.array([[1, 16, 16]]), 2)
    assert mi.shape == (64, 4)
    assert mi[0].tolist() == [0, 1, 16, 17]
    assert mi[7].tolist() == [14, 15, 30, 31]
    assert mi[63].tolist() == [238, 239, 254, 255]
    mi = O.merge_index(np.array([[1, 4, 6], [2, 2, 2]]), 2)     # non-square, then a 2-frame clip
    assert mi[4].tolist() == [14, 15, 20, 21]                   # (R=1, C=1)
    assert mi[6].tolist() == [24, 25, 26, 27] and mi[7].tolist() == [28, 29, 30, 31]


# ------------------------------------------------------------------ audio front end
def test_conv1d_and_pool_library():
    x, W, b = RNG.standard_normal((5, 22)), RNG.standard_normal((7, 5, 3)), RNG.standard_normal(7)
    for stride in (1, 2):
        ref = F.conv1d(T64(x)[None], T64(W), T64(b), stride=stride, padding=1)[0].numpy()
        assert np.allclose(O.conv1d(x, W, b, stride, 1), ref, atol=1e-12)
    assert O.conv1d(np.zeros((128, 3000)), np.zeros((4, 128, 3)), np.zeros(4), 1, 1).shape == (4, 3000)
    assert O.conv1d(np.zeros((4, 3000)), np.zeros((4, 4, 3)), np.zeros(4), 2, 1).shape == (4, 1500)


def test_sinusoid_positions_closed_form():
    pe = O.sinusoid_positions(10, 8)
    assert np.array_equal(pe[0], [0, 0, 0, 0, 1, 1, 1, 1])
    assert np.allclose(pe[3, 0], math.sin(3.0)) and np.allclose(pe[3, 4], math.cos(3.0))
    assert np.allclose(pe[3, 3], math.sin(3.0 * 1e-4)) and np.allclose(pe[5, 7], math.cos(5.0 * 1e-4))
    assert np.allclose(pe[2, 1], math.sin(2.0 * 10000 ** (-1 / 3)))


# ------------------------------------------------------------------ whole towers: an independent composition
class _TorchViT:
    """Second write-up of the vision tower from PyTorch pieces, organised differently from the
    checker: windows are cut out by index lists and attended one by one with the library
    attention (no mask), rotary goes through complex multiplication, the merger gathers by
    explicit (t, R, C) loops."""

    def __init__(self, cfg, W):
        self.cfg, self.W = cfg, {k: T64(v) for k, v in W.items()}

    def groups(self, grid, window):
        out, base = [], 0
        for (T, h, w) in grid:
            if window <= 0:
                out.append(list(range(base, base + T * h * w)))
            else:
                for t in range(T):
                    for r0 in range(0, h, window):
                        for c0 in range(0, w, window):
                            out.append([base + (t * h + r) * w + c for r in range(r0, min(r0 + window, h))
                                        for c in range(c0, min(c0 + window, w))])
            base += T * h * w
        return out

    def rope(self, x, pos):
        cfg = self.cfg
        half = cfg.head_dim // 2
        freqs = []
        for a, n in enumerate(cfg.rope_sections):
            inv = torch.tensor([cfg.rope_theta ** (-i / n) for i in range(n)], dtype=torch.float64)
            freqs.append(pos[:, a:a + 1].double() * inv[None])
        ang = torch.cat(freqs, 1)
        z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], -1)

    def run(self, patches, grid):
        cfg, W = self.cfg, self.W
        D, nh, dh = cfg.hidden, cfg.n_heads, cfg.head_dim
        pos = torch.tensor([[t, r, c] for (T, h, w) in grid for t in range(T) for r in range(h) for c in range(w)])
        x = F.linear(T64(patches), W["patch_embed.weight"])
        N = x.shape[0]
        for l in range(cfg.n_layers):
            p = f"blocks.{l}."
            u = F.rms_norm(x, (D,), W[p + "norm1.weight"], cfg.norm_eps)
            q, k, v = F.linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"]).reshape(N, 3, nh, dh).unbind(1)
            q, k = self.rope(q, pos), self.rope(k, pos)
            win = 0 if (cfg.window <= 0 or l in cfg.full_attn_layers) else cfg.window
            a = torch.empty(N, nh, dh, dtype=torch.float64)
            for idx in self.groups(grid, win):
                o = F.scaled_dot_product_attention(q[idx].transpose(0, 1), k[idx].transpose(0, 1),
                                                   v[idx].transpose(0, 1))
                a[idx] = o.transpose(0, 1)
            x = x + F.linear(a.reshape(N, D), W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
            u = F.rms_norm(x, (D,), W[p + "norm2.weight"], cfg.norm_eps)
            m = F.silu(F.linear(u, W[p + "mlp.gate.weight"], W[p + "mlp.gate.bias"])) * \
                F.linear(u, W[p + "mlp.up.weight"], W[p + "mlp.up.bias"])
            x = x + F.linear(m, W[p + "mlp.down.weight"], W[p + "mlp.down.bias"])
        z = F.rms_norm(x, (D,), W["merger.norm.weight"], cfg.norm_eps)
        rows, base = [], 0
        for (T, h, w) in grid:
            for t in range(T):
                for R in range(h // 2):
                    for C in range(w // 2):
                        f = lambda r, c: z[base + (t * h + r) * w + c]
                        rows.append(torch.cat([f(2 * R, 2 * C), f(2 * R, 2 * C + 1), f(2 * R + 1, 2 * C),
                                               f(2 * R + 1, 2 * C + 1)]))
            base += T * h * w
        y = F.gelu(F.linear(torch.stack(rows), W["merger.fc1.weight"], W["merger.fc1.bias"]))
        return F.linear(y, W["merger.fc2.weight"], W["merger.fc2.bias"]).numpy()


def _mini_vit_cfg(**kw):
    base = dict(arch="vit", dtype="f32", patch_dim=24, temporal_patch=1, hidden=32, n_heads=2, head_dim=16,
                n_layers=3, mlp_dim=40, merge=2, merger_hidden=48, out_hidden=20, window=8,
                full_attn_layers=(1,), rope_sections=(0, 4, 4))
    base.update(kw)
    return wl.EncoderConfig(**base)


@pytest.mark.parametrize("sections,grid", [((0, 4, 4), [(1, 10, 12), (1, 4, 6)]), ((2, 3, 3), [(3, 10, 4), (1, 2, 2)])])
def test_vit_tower_matches_independent_composition(sections, grid):
    cfg = _mini_vit_cfg(rope_sections=sections)
    W = wl.make_weights(cfg, seed=5, std=0.2)
    n = sum(t * h * w for t, h, w in grid)
    patches = RNG.standard_normal((n, cfg.patch_dim))
    mine = O.vit_encode(cfg, W, patches, np.array(grid))
    ref = _TorchViT(cfg, W).run(patches, grid)
    assert mine.shape == (n // 4, cfg.out_hidden)
    assert np.allclose(mine, ref, atol=1e-9)


def test_vit_identity_layers_closed_form():
    """Zero output projections and zero down projections make every block the identity, so
    the tower is merger(patch_embed(x)) in closed form."""
    cfg = _mini_vit_cfg()
    W = wl.make_weights(cfg, seed=6, std=0.2)
    for l in range(cfg.n_layers):
        for nme in ("attn.proj.weight", "attn.proj.bias", "mlp.down.weight", "mlp.down.bias"):
            W[f"blocks.{l}.{nme}"] = np.zeros_like(W[f"blocks.{l}.{nme}"])
    grid = np.array([[1, 4, 6]])
    patches = RNG.standard_normal((24, cfg.patch_dim))
    x = patches @ W["patch_embed.weight"].astype(np.float64).T
    z = x / np.sqrt((x * x).mean(1, keepdims=True) + cfg.norm_eps) * W["merger.norm.weight"]
    zc = np.stack([np.concatenate([z[(2 * R + dr) * 6 + 2 * C + dc] for dr in (0, 1) for dc in (0, 1)])
                   for R in range(2) for C in range(3)])
    hid = zc @ W["merger.fc1.weight"].astype(np.float64).T + W["merger.fc1.bias"]
    hid = F.gelu(T64(hid)).numpy()
    y = hid @ W["merger.fc2.weight"].astype(np.float64).T + W["merger.fc2.bias"]
    assert np.allclose(O.vit_encode(cfg, W, patches, grid), y, atol=1e-10)


def test_vit_batch_invariance_bitwise():
    cfg = _mini_vit_cfg()
    W = wl.make_weights(cfg, seed=7, std=0.2)
    g = np.array([[1, 10, 12], [1, 4, 6]])
    patches = RNG.standard_normal((144, cfg.patch_dim))
    both = O.vit_encode(cfg, W, patches, g)
    a = O.vit_encode(cfg, W, patches[:120], g[:1])
    b = O.vit_encode(cfg, W, patches[120:], g[1:])
    assert np.allclose(both, np.concatenate([a, b]), atol=1e-12)


# ------------------------------------------------------------------ class-token tower
def _mini_cls_cfg(**kw):
    base = dict(arch="vit_cls", dtype="f32", patch_dim=24, temporal_patch=1, hidden=32, n_heads=2, head_dim=16,
                n_layers=3, mlp_dim=40, merge=2, merger_hidden=48, out_hidden=20, window=0, full_attn_layers=(),
                rope_sections=(0, 0, 0), tile_patches=(4, 6))
    base.update(kw)
    return wl.EncoderConfig(**base)


def _torch_cls_tower(cfg, W, patches, n_tiles):
    """Second write-up from PyTorch pieces, organised differently from the checker: all tiles as one
    batched tensor [B, 1 + h*w, D], library LayerNorm / attention / GELU, the 2x2 grouping by a
    view + permute instead of explicit indices."""
    W = {k: T64(v) for k, v in W.items()}
    h, w = cfg.tile_patches
    D, nh, dh = cfg.hidden, cfg.n_heads, cfg.head_dim
    x = F.linear(T64(patches).reshape(n_tiles, h * w, -1), W["patch_embed.weight"], W["patch_embed.bias"])
    x = torch.cat([W["cls_token"].expand(n_tiles, 1, D), x], 1) + W["pos_embed"][None]
    for l in range(cfg.n_layers):
        p = f"blocks.{l}."
        u = F.layer_norm(x, (D,), W[p + "norm1.weight"], W[p + "norm1.bias"], cfg.norm_eps)
        q, k, v = F.linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"]).reshape(n_tiles, -1, 3, nh, dh).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(n_tiles, -1, D)
        x = x + W[p + "ls1"] * F.linear(a, W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
        u = F.layer_norm(x, (D,), W[p + "norm2.weight"], W[p + "norm2.bias"], cfg.norm_eps)
        m = F.gelu(F.linear(u, W[p + "mlp.fc1.weight"], W[p + "mlp.fc1.bias"]))
        x = x + W[p + "ls2"] * F.linear(m, W[p + "mlp.fc2.weight"], W[p + "mlp.fc2.bias"])
    z = x[:, 1:].reshape(n_tiles, h // 2, 2, w // 2, 2, D).permute(0, 1, 3, 2, 4, 5).reshape(-1, 4 * D)
    z = F.layer_norm(z, (4 * D,), W["merger.norm.weight"], W["merger.norm.bias"], cfg.norm_eps)
    y = F.gelu(F.linear(z, W["merger.fc1.weight"], W["merger.fc1.bias"]))
    return F.linear(y, W["merger.fc2.weight"], W["merger.fc2.bias"]).numpy()


@pytest.mark.parametrize("tile", [(4, 6), (2, 2), (6, 4)])
def test_cls_tower_matches_independent_composition(tile):
    cfg = _mini_cls_cfg(tile_patches=tile)
    W = wl.make_weights(cfg, seed=11, std=0.2)
    n = tile[0] * tile[1]
    patches = RNG.standard_normal((3 * n, cfg.patch_dim))
    mine = O.cls_encode(cfg, W, patches, np.array([(1, *tile)] * 3))
    assert mine.shape == (3 * n // 4, cfg.out_hidden)
    assert np.allclose(mine, _torch_cls_tower(cfg, W, patches, 3), atol=1e-9)


def test_cls_tower_with_zero_branch_scales_in_closed_form():
    """ls1 = ls2 = 0 switches every block off: the output is the projector applied to
    patch_embed + position, written out here with explicit indices (a 4 x 6 tile: group (R, C) is
    patches (2R, 2C), (2R, 2C+1), (2R+1, 2C), (2R+1, 2C+1); patch (r, c) takes position row
    1 + 6 r + c); the class token and position row 0 do not reach the output at all."""
    cfg = _mini_cls_cfg()
    W = wl.make_weights(cfg, seed=12, std=0.2)
    for l in range(cfg.n_layers):
        W[f"blocks.{l}.ls1"] = np.zeros(cfg.hidden, np.float32)
        W[f"blocks.{l}.ls2"] = np.zeros(cfg.hidden, np.float32)
    patches = RNG.standard_normal((24, cfg.patch_dim))
    grid = np.array([[1, 4, 6]])
    e = patches @ W["patch_embed.weight"].astype(np.float64).T + W["patch_embed.bias"]
    rows = []
    for R in range(2):
        for C in range(3):
            rows.append(np.concatenate([e[6 * r + c] + W["pos_embed"][1 + 6 * r + c].astype(np.float64)
                                        for r, c in ((2 * R, 2 * C), (2 * R, 2 * C + 1), (2 * R + 1, 2 * C), (2 * R + 1, 2 * C + 1))]))
    z = np.stack(rows)
    z = (z - z.mean(1, keepdims=True)) / np.sqrt(z.var(1, keepdims=True) + cfg.norm_eps)
    z = z * W["merger.norm.weight"] + W["merger.norm.bias"]
    hid = z @ W["merger.fc1.weight"].astype(np.float64).T + W["merger.fc1.bias"]
    hid = np.array([[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in row] for row in hid])
    want = hid @ W["merger.fc2.weight"].astype(np.float64).T + W["merger.fc2.bias"]
    got = O.cls_encode(cfg, W, patches, grid)
    assert np.allclose(got, want, atol=1e-10)
    W2 = dict(W)
    W2["cls_token"] = W["cls_token"] + 1.0
    W2["pos_embed"] = W["pos_embed"].copy()
    W2["pos_embed"][0] += 3.0
    assert np.array_equal(O.cls_encode(cfg, W2, patches, grid), got)


def test_cls_tower_class_token_is_attended_and_tiles_are_independent():
    cfg = _mini_cls_cfg()
    W = wl.make_weights(cfg, seed=13, std=0.2)
    patches = RNG.standard_normal((48, cfg.patch_dim))
    g = np.array([[1, 4, 6], [1, 4, 6]])
    both = O.cls_encode(cfg, W, patches, g)
    a, b = O.cls_encode(cfg, W, patches[:24], g[:1]), O.cls_encode(cfg, W, patches[24:], g[1:])
    assert np.allclose(both, np.concatenate([a, b]), atol=1e-12)
    W2 = dict(W)
    # with the blocks on, the class token is a key for every patch (a change that LayerNorm does not
    # remove: not a common offset of all channels)
    W2["cls_token"] = W["cls_token"] + np.linspace(-1, 1, cfg.hidden).astype(np.float32)
    assert np.abs(O.cls_encode(cfg, W2, patches[:24], g[:1]) - a).max() > 1e-4
    assert np.allclose(O.encode(cfg, W, patches, np.array([0, 24, 48]), g), both, atol=0)


def test_audio_tower_matches_independent_composition():
    cfg = wl.EncoderConfig(arch="audio", dtype="f32", patch_dim=6, temporal_patch=1, hidden=16, n_heads=2,
                           head_dim=8, n_layers=2, mlp_dim=24, merge=2, merger_hidden=0, out_hidden=10,
                           window=0, full_attn_layers=(), rope_sections=(0, 0, 0), norm_eps=1e-5)
    Wn = wl.make_weights(cfg, seed=8, std=0.3)
    W = {k: T64(v) for k, v in Wn.items()}
    frames = RNG.standard_normal((20 + 12, 6))
    cu = np.array([0, 20, 32])
    mine = O.audio_encode(cfg, Wn, frames, cu)
    outs = []
    for i in range(2):
        mel = T64(frames[cu[i]:cu[i + 1]]).T[None]
        c = F.gelu(F.conv1d(mel, W["conv1.weight"], W["conv1.bias"], padding=1))
        c = F.gelu(F.conv1d(c, W["conv2.weight"], W["conv2.bias"], stride=2, padding=1))[0].T
        T = c.shape[0]
        inv = torch.exp(-math.log(10000.0) / 7 * torch.arange(8, dtype=torch.float64))
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None]
        x = c + torch.cat([ang.sin(), ang.cos()], 1)
        for l in range(2):
            p = f"blocks.{l}."
            u = F.layer_norm(x, (16,), W[p + "norm1.weight"], W[p + "norm1.bias"], 1e-5)
            q, k, v = F.linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"]).reshape(T, 3, 2, 8).unbind(1)
            a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1))
            x = x + F.linear(a.transpose(0, 1).reshape(T, 16), W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
            u = F.layer_norm(x, (16,), W[p + "norm2.weight"], W[p + "norm2.bias"], 1e-5)
            x = x + F.linear(F.gelu(F.linear(u, W[p + "mlp.fc1.weight"], W[p + "mlp.fc1.bias"])),
                             W[p + "mlp.fc2.weight"], W[p + "mlp.fc2.bias"])
        pooled = F.avg_pool1d(x.T[None], 2)[0].T
        z = F.layer_norm(pooled, (16,), W["post.norm.weight"], W["post.norm.bias"], 1e-5)
        outs.append(F.linear(z, W["post.proj.weight"], W["post.proj.bias"]).numpy())
    ref = np.concatenate(outs)
    assert mine.shape == (5 + 3, 10)
    assert np.allclose(mine, ref, atol=1e-10)
    assert np.all(Wn["blocks.0.attn.qkv.bias"][16:32] == 0)        # the key projection carries no bias


# ------------------------------------------------------------------ hand-off
def test_forward_embeddings_c1_layout():
    w = wl.c1_tiny()
    assert w.placeholder_index.tolist() == list(range(32, 96))
    dst = w.consumer_buffer_bits()
    src = np.random.default_rng(0).integers(0, 1 << 32, size=(64, 512), dtype=np.uint32)
    out = O.forward_embeddings(src, w.placeholder_index, dst)
    assert np.array_equal(out[32:96], src)
    assert np.array_equal(out[:32], dst[:32]) and np.array_equal(out[96:], dst[96:])


def test_forward_embeddings_identity_skip_and_order():
    src = np.arange(12, dtype=np.uint16).reshape(4, 3)
    dst = np.full((6, 3), 999, np.uint16)
    assert np.array_equal(O.forward_embeddings(src, np.arange(4), dst)[:4], src)      # identity = memcpy
    out = O.forward_embeddings(src, np.array([5, -1, 0, 2]), dst)
    assert out.tolist() == [[6, 7, 8], [999] * 3, [9, 10, 11], [999] * 3, [999] * 3, [0, 1, 2]]


# ------------------------------------------------------------------ workloads (shapes the configs name)
def test_workload_shapes():
    w = wl.c1_tiny()
    assert w.patches.shape == (256, 588) and w.out_rows.tolist() == [64]
    sizes = wl.varlen_image_sizes()
    assert len(sizes) == 32 and all(224 <= s <= 1344 and s % 28 == 0 for hw in sizes for s in hw)
    x = np.array([1.0, 1.00390625, 1.005859375, -3.14159], np.float32)
    r = wl.round_to_bf16(x)
    assert r.tolist() == torch.tensor(x).to(torch.bfloat16).float().tolist()
    assert np.array_equal(wl.from_bits_bf16(wl.to_bits_bf16(r)), r)


# ------------------------------------------------------------------ hand-off channel (sequential model)
def test_channel_model_follows_a_hand_written_trace():
    """Two slots of 64 bytes, rows of 4 uint32 (16 bytes).  Every status, slot number and buffer
    content below is written out by hand from the rules: lowest free slot; WRITING -> READY ->
    FREE; a placement copies row i to the row its index names, -1 skips."""
    m = O.ChannelModel(2, 64)
    rows_a = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], np.uint32)
    rows_b = np.array([[9, 9, 9, 9]], np.uint32)
    dst = np.zeros((4, 4), np.uint32) + np.arange(100, 104, dtype=np.uint32)[:, None]
    assert m.acquire(0) == ("workspace", -1) and m.acquire(65) == ("workspace", -1)
    assert m.acquire(32) == ("ok", 0)
    assert m.acquire(64) == ("ok", 1)
    assert m.acquire(16) == ("busy", -1)
    assert m.publish(0, np.zeros((3, 4), np.uint32)) == "shape"        # 48 bytes into 32 reserved
    assert m.forward(0, np.array([0]), dst)[0] == "invalid"            # acquired, nothing published
    assert m.publish(1, rows_b) == "ok"
    assert m.publish(1, rows_b) == "invalid"                           # already published
    st, d1 = m.forward(1, np.array([2]), dst)
    assert st == "ok" and d1.tolist() == [[100] * 4, [101] * 4, [9] * 4, [103] * 4]
    assert dst.tolist() == [[100] * 4, [101] * 4, [102] * 4, [103] * 4]  # the argument is not modified
    assert m.forward(1, np.array([2]), dst)[0] == "invalid"            # consumed: the slot is free again
    assert m.acquire(16) == ("ok", 1)                                  # slot 0 is still being written
    assert m.publish(0, rows_a) == "ok"
    st, d2 = m.forward(0, np.array([3, -1]), d1)
    assert st == "ok" and d2.tolist() == [[100] * 4, [101] * 4, [9] * 4, [1, 2, 3, 4]]
    assert m.release(0) == "invalid" and m.release(2) == "invalid" and m.release(-1) == "invalid"
    assert m.release(1) == "ok" and m.state == [m.FREE, m.FREE]
    assert m.acquire(64) == ("ok", 0)
    assert m.publish(0, np.zeros((0, 4), np.uint32)) == "ok"           # an empty tensor may be handed over
    st, d3 = m.forward(0, np.zeros(0, np.int64), d2)
    assert st == "ok" and np.array_equal(d3, d2)


def test_channel_model_keeps_what_was_published_not_what_the_array_holds_later():
    m = O.ChannelModel(1, 16)
    rows = np.array([[1, 2, 3, 4]], np.uint32)
    assert m.acquire(16) == ("ok", 0) and m.publish(0, rows) == "ok"
    rows[:] = 0
    assert m.forward(0, np.array([0]), np.zeros((1, 4), np.uint32))[1].tolist() == [[1, 2, 3, 4]]
