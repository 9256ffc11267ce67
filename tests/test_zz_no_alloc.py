"""cs_encode_static (the entry point that allocates nothing: its workspace is a static array on the GPU)
against cs_encode, through the C ABI: two calls in a row, the second with a smaller batch, each compared
bit for bit with cs_encode on the same input (the same kernels run in the same launch configuration, so
the embedding tolerance collapses to equality); and the refusal of a batch that does not fit the array."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2603_12118_amd import binding as B
from paper_2603_12118_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_bf16(x32: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(wl.to_bits_bf16(x32).view(np.int16)).to(DEV).view(torch.bfloat16)


def test_static_scratch_matches_workspace_call():
    # a shallow tower of the 7B shape; one 448 x 448 image (1024 patches: most of the array), then a
    # smaller ragged pair whose buffers lie differently in it
    cfg = replace(wl.vit_7b_config(3), dtype="bf16", full_attn_layers=(1,))
    big = wl.images_workload("one_image", cfg, [(448, 448)], seq_len=1024)
    small = wl.images_workload("two_small", cfg, [(84, 140), (252, 196)], seq_len=1024, data_seed=5)
    enc = B.Encoder(cfg, big.weights)
    for w in (big, small):
        n_out, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
        assert ws_bytes <= 64 << 20
        x = dev_bf16(w.patches)
        ref, _ = enc.cs_encode(x, w.cu_seqlens, w.grid_thw)
        out = torch.full((n_out, cfg.out_hidden), float("nan"), dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        enc.cs_encode_static(x, w.cu_seqlens, w.grid_thw, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.isfinite(out).all()
        assert torch.equal(out, ref), (w.name, (out - ref).abs().max().item())
    # the first batch once more: nothing of the smaller call's leftovers in the array shows
    x = dev_bf16(big.patches)
    ref, _ = enc.cs_encode(x, big.cu_seqlens, big.grid_thw)
    out = enc.cs_encode_static(x, big.cu_seqlens, big.grid_thw)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_static_scratch_refuses_what_does_not_fit():
    cfg = replace(wl.vit_7b_config(1), dtype="bf16", full_attn_layers=())
    w = wl.images_workload("four_images", cfg, [(448, 448)] * 4, seq_len=1024)
    enc = B.Encoder(cfg, w.weights)
    _, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    assert ws_bytes > 64 << 20
    x = dev_bf16(w.patches)
    out = torch.zeros(int(w.out_rows.sum()), cfg.out_hidden, dtype=torch.float32, device=DEV)
    with pytest.raises(B.CsError) as ei:
        enc.cs_encode_static(x, w.cu_seqlens, w.grid_thw, out=out)
    assert ei.value.status == B.CS_ERR_WORKSPACE and "static scratch" in str(ei.value)
    torch.cuda.synchronize()
    assert not out.any()          # refused before anything was enqueued
