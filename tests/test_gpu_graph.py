"""cs_encode_graph_*: the launches of one small batch recorded into a HIP graph and replayed.  Every replay
is compared bit for bit with the eager cs_encode on the same inputs, with the program's own eager work and
synchronisations between the replays (another batch through another workspace), and once with new pixel
data written into the bound input buffer."""
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


@pytest.mark.parametrize("sizes", [[(448, 448)], [(84, 140), (252, 196), (56, 56)]])
def test_graph_replays_give_the_eager_bits(sizes):
    cfg = replace(wl.vit_7b_config(4), dtype="bf16", full_attn_layers=(1, 3))
    w = wl.images_workload("graph_batch", cfg, sizes, seq_len=2048)
    other = wl.images_workload("other_batch", cfg, [(140, 84)], seq_len=2048, data_seed=9)
    enc = B.Encoder(cfg, w.weights)
    x = dev_bf16(w.patches)
    ref, _ = enc.cs_encode(x, w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    n_out, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    out = torch.full_like(ref, float("nan"))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    g = enc.cs_encode_graph_create(x, w.cu_seqlens, w.grid_thw, out, ws, side)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)                      # the eager call inside create
    xo = dev_bf16(other.patches)
    for k in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.cs_encode_graph_launch(side if k % 2 else None)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {k}"
        # eager work of the same encoder in between (its own workspace), then a synchronisation
        o2, _ = enc.cs_encode(xo, other.cu_seqlens, other.grid_thw)
        torch.cuda.synchronize()
        assert torch.isfinite(o2).all()
    # new data in the bound input buffer
    w2 = wl.images_workload("graph_batch2", cfg, sizes, seq_len=2048, data_seed=4)
    x2 = dev_bf16(w2.patches)
    ref2, _ = enc.cs_encode(x2, w2.cu_seqlens, w2.grid_thw)
    x.copy_(x2)
    torch.cuda.synchronize()
    g.cs_encode_graph_launch()
    torch.cuda.synchronize()
    assert torch.equal(out, ref2) and not torch.equal(ref2, ref)
    g.close()


def test_graph_create_rejects_the_default_stream():
    cfg = replace(wl.vit_7b_config(1), dtype="bf16", full_attn_layers=())
    w = wl.images_workload("b", cfg, [(56, 56)], seq_len=64)
    enc = B.Encoder(cfg, w.weights)
    x = dev_bf16(w.patches)
    n_out, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    out = torch.zeros(n_out, cfg.out_hidden, device=DEV)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)

    class Null:
        cuda_stream = 0
    with pytest.raises(B.CsError):
        enc.cs_encode_graph_create(x, w.cu_seqlens, w.grid_thw, out, ws, Null())
