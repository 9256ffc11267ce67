"""GPU parity over batch sizes: shallow towers of the full layer shapes on seeded random batches whose
token counts straddle the launcher's choices (split-K below 2560 tokens, 128 x 128 / 256 x 256 / narrow
tiles, 64-row tail tiles, half tiles of a last round, folded or separate normalisation).  The whole batch
runs through the C ABI; the largest items and the last one are compared with the CPU checker run on them
alone (items are independent in every layer), element by element, at the bars used everywhere."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import encoder_oracle as O
from paper_2603_12118_amd import binding as B
from paper_2603_12118_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MAX_ABS, MIN_COS = 3e-2, 0.999
_weights = {}


def dev_bf16(x32: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(wl.to_bits_bf16(x32).view(np.int16)).to(DEV).view(torch.bfloat16)


def shared_weights(key, w: wl.Workload):
    """One set of weights per tower shape (same seed, same shapes for every batch of that tower)."""
    if key not in _weights:
        _weights[key] = w.weights
    w._weights = _weights[key]
    return _weights[key]


def check_items(tag, w: wl.Workload, W, items):
    enc = B.Encoder(w.cfg, W)
    out, _ = enc.cs_encode(dev_bf16(w.patches), w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    g = out.double().cpu().numpy()
    assert np.isfinite(g).all(), tag
    ocu = np.concatenate([[0], np.cumsum(w.out_rows)])
    for it in items:
        one = w.select_items([it])
        ref = O.encode(one.cfg, W, one.patches, one.cu_seqlens, one.grid_thw)
        gi = g[ocu[it]:ocu[it + 1]]
        err = float(np.abs(gi - ref).max())
        cos = float(((gi * ref).sum(1) / (np.linalg.norm(gi, axis=1) * np.linalg.norm(ref, axis=1))).min())
        print(f"{tag} item {it}: rows={ref.shape[0]} max_abs_err={err:.4g} min_cos={cos:.6f}", flush=True)
        assert err <= MAX_ABS and cos >= MIN_COS, (tag, it, err, cos)


@pytest.mark.parametrize("target", [900, 1500, 2560, 2700, 4100, 6700, 9100, 21000])
def test_image_batches_of_many_sizes(target):
    rng = np.random.default_rng(target)
    cfg = replace(wl.vit_7b_config(2), dtype="bf16", full_attn_layers=(1,))
    sizes, total = [], 0
    while total < target:
        h, w_ = 28 * int(rng.integers(2, 34)), 28 * int(rng.integers(2, 34))
        n = (h // 14) * (w_ // 14)
        if sizes and total + n > 1.15 * target:
            break
        sizes.append((h, w_))
        total += n
    w = wl.images_workload(f"images_{target}", cfg, sizes, seq_len=8192, data_seed=target)
    W = shared_weights("vit", w)
    order = np.argsort(-w.out_rows)
    check_items(f"images {int(w.cu_seqlens[-1])} tokens", w, W, sorted({int(order[0]), len(sizes) - 1}))


@pytest.mark.parametrize("n_tiles", [3, 11])
def test_class_token_tower_tile_counts(n_tiles):
    w = wl.images_workload(f"tiles_{n_tiles}", wl.vit_cls_config(2), [(448, 448)] * n_tiles, seq_len=2048, data_seed=n_tiles)
    W = shared_weights("cls", w)
    check_items(f"class-token tower, {n_tiles} tiles", w, W, sorted({0, n_tiles - 1}))


@pytest.mark.parametrize("n_clips,frames", [(3, 1960), (11, 1208)])
def test_audio_clip_lengths(n_clips, frames):
    w = wl.audio_workload(f"audio_{n_clips}x{frames}", wl.audio_config(2), n_clips, frames, seq_len=2048, data_seed=frames)
    W = shared_weights("audio", w)
    check_items(f"audio {n_clips} clips of {frames} frames", w, W, sorted({0, n_clips - 1}))


def test_tile_choice_by_batch_size():
    """The launcher's choices the batches above straddle, by name: which instantiation the four GEMMs of a block
    run for a number of tokens (`gemm_kernel<BM, BN, waves along M, waves along N, epilogue, tail>`)."""
    import os
    if any(k.startswith("CS_GEMM_") or k == "CS_NO_NORM_FOLD" for k in os.environ):
        pytest.skip("a measurement switch in the environment changes the choices this test names")
    w = wl.images_workload("tiles_by_size", replace(wl.vit_7b_config(2), dtype="bf16", full_attn_layers=(1,)),
                           [(56, 56)], seq_len=8192, data_seed=1)
    enc = B.Encoder(w.cfg, shared_weights("vit", w))
    name = lambda step, n: enc.cs_encoder_step_kernel(B.STEPS[step], n).split(">")[0] + ">"
    # gate|up: 128 x 128 below a round of 256 x 256 tiles (short of 5/8 of it), 256 x 256 from 160 tiles on, with half
    # tiles in a last round that is at most half full
    assert name("mlp_up", 1024) == "gemm_kernel<128, 128, 2, 2, 5, 0>"
    assert name("mlp_up", 2048) == "gemm_kernel<256, 256, 2, 4, 5, 0>"      # 216 tiles: one round
    assert name("mlp_up", 3072) == "gemm_kernel<256, 256, 2, 4, 5, 2>"      # 324 tiles: a round and 68
    assert name("mlp_up", 8192) == "gemm_kernel<256, 256, 2, 4, 5, 2>"      # 864 tiles: three rounds and 96
    # residual GEMMs with N = 1280: 128 x 160 (eight waves up to one tile per CU, then two four-wave workgroups per
    # CU), 256 x 160 from 192 of those on, 256 x 256 from a round and a half on
    assert name("proj", 3072) == "gemm_kernel<128, 160, 4, 2, 4, 0>"
    assert name("proj", 5120) == "gemm_kernel<128, 160, 2, 2, 4, 0>"
    assert name("proj", 8192) == "gemm_kernel<256, 160, 4, 2, 4, 0>"
    assert name("mlp_down", 8192) == "gemm_kernel<256, 160, 4, 2, 4, 0>"
    assert name("proj", 24576) == "gemm_kernel<256, 256, 2, 4, 4, 0>"        # 480 tiles: a round and 224
    assert name("proj", 32768) == "gemm_kernel<256, 256, 2, 4, 4, 2>"        # 640 tiles: two rounds and 128
    assert name("qkv", 8192) == "gemm_kernel<256, 256, 2, 4, 6, 0>"
