"""GPU parity tests: the HIP path, called through the C ABI, against the CPU checker on the same
seeded inputs.  Bars: bit-exact for the embedding hand-off and all index work; for embeddings
max |gpu - oracle| <= 3e-2 and per-row cosine >= 0.999 (bf16 arithmetic against the fp64 checker
fed the same bf16-rounded weights and inputs)."""
import math
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


def dev_bf16(x32: np.ndarray) -> torch.Tensor:
    """fp32 array of bf16-representable values -> device bf16 tensor with the same bits."""
    return torch.from_numpy(wl.to_bits_bf16(x32).view(np.int16)).to(DEV).view(torch.bfloat16)


def dev_input(w: wl.Workload) -> torch.Tensor:
    return dev_bf16(w.patches) if w.cfg.dtype == "bf16" else torch.from_numpy(w.patches).to(DEV)


def check_embeddings(gpu: torch.Tensor, ref: np.ndarray, what: str):
    g = gpu.float().cpu().numpy().astype(np.float64)
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - ref).max()
    cos = (g * ref).sum(1) / (np.linalg.norm(g, axis=1) * np.linalg.norm(ref, axis=1))
    print(f"{what}: max_abs_err={err:.4g} min_cos={cos.min():.6f} max|ref|={np.abs(ref).max():.3f}", flush=True)
    assert err <= MAX_ABS, f"{what}: max abs error {err}"
    assert cos.min() >= MIN_COS, f"{what}: min cosine {cos.min()}"


# ------------------------------------------------------------------ embedding hand-off (bit-exact)
def _scatter_case(rows, hidden, dst_rows, dtype, idx, seed=0):
    rng = np.random.default_rng(seed)
    if dtype == "bf16":
        src = rng.integers(0, 1 << 16, (rows, hidden), dtype=np.uint16)
        dst = rng.integers(0, 1 << 16, (dst_rows, hidden), dtype=np.uint16)
        tv = lambda a: torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
        back = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    else:
        src = rng.integers(0, 1 << 32, (rows, hidden), dtype=np.uint32)
        dst = rng.integers(0, 1 << 32, (dst_rows, hidden), dtype=np.uint32)
        tv = lambda a: torch.from_numpy(a.view(np.int32)).to(DEV).view(torch.float32)
        back = lambda t: t.view(torch.int32).cpu().numpy().view(np.uint32)
    d = tv(dst)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.cs_forward_embeddings(tv(src), torch.from_numpy(np.asarray(idx, np.int64)).to(DEV), d, err_flag=flag)
    torch.cuda.synchronize()
    return src, dst, back(d), int(flag.item())


def test_forward_embeddings_c1_positions():
    w = wl.c1_tiny()
    src, dst, got, flag = _scatter_case(64, 512, 128, "f32", w.placeholder_index)
    assert np.array_equal(got, O.forward_embeddings(src, w.placeholder_index, dst)) and flag == 0
    assert np.array_equal(got[32:96], src) and np.array_equal(got[:32], dst[:32]) and np.array_equal(got[96:], dst[96:])


@pytest.mark.parametrize("rows", [1170, 2340, 4681])       # 8, 16, 32 MB of bf16 rows, the sizes of the paper's Sec. 3 "Sidecar Overhead"
def test_forward_embeddings_random_spans_bf16(rows):
    rng = np.random.default_rng(rows)
    dst_rows = 3 * rows + 17
    idx = rng.permutation(dst_rows)[:rows].astype(np.int64)
    idx[rng.integers(0, rows, 5)] = -1
    src, dst, got, flag = _scatter_case(rows, 3584, dst_rows, "bf16", idx)
    assert np.array_equal(got, O.forward_embeddings(src, idx, dst)) and flag == 0


def test_forward_embeddings_edge_cases():
    # identity index = plain copy; empty input; out-of-range index raises the flag and writes nothing
    src, dst, got, flag = _scatter_case(33, 8, 33, "bf16", np.arange(33))
    assert np.array_equal(got, src) and flag == 0
    idx = np.array([2, 7, -5, 1], np.int64)
    src, dst, got, flag = _scatter_case(4, 8, 7, "f32", idx)
    ok = np.array([2, -1, -1, 1])
    assert np.array_equal(got, O.forward_embeddings(src, ok, dst)) and flag == 1
    d = torch.zeros(4, 8, device=DEV)
    B.cs_forward_embeddings(torch.zeros(0, 8, device=DEV), torch.zeros(0, dtype=torch.int64, device=DEV), d)
    assert B.cs_forward_embeddings_raw(1, 8, 16, 4, 4, 7, B.CS_BF16) != 0        # 14-byte rows are refused


def test_forward_embeddings_workload_spans():
    w = wl.c2_images(n_layers=1)
    rows = int(w.out_rows.sum())
    src, dst, got, flag = _scatter_case(rows, 3584, w.n_sequences * w.seq_len, "bf16", w.placeholder_index)
    assert np.array_equal(got, O.forward_embeddings(src, w.placeholder_index, dst)) and flag == 0


# ------------------------------------------------------------------ contraction kernels on their own
# one K slice; one row; N a multiple of 4 only; ragged tails of every tile shape; the layer shapes; 256 x 256
# tiles that fill one round of the chip (180 of them), with and without 64-row tail tiles behind the full
# tile rows (3000 = 11 x 256 + 184); 256 x 128 tiles with one tail tile row (8224 = 32 x 256 + 32)
@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (1, 8, 64), (100, 36, 192), (300, 200, 128), (1000, 520, 1216),
                                   (257, 3840, 1280), (2048, 1280, 3456), (3000, 1280, 256), (3072, 3840, 128),
                                   (3000, 3840, 192), (8224, 1024, 256),
                                   (4096, 4352, 128),      # 272 tiles of 256 x 256: the last 16 run as half tiles
                                   (16500, 2048, 64)])     # 520 tiles, a ragged last tile row among the 8 split ones
def test_linear_matches_oracle(M, N, K):
    rng = np.random.default_rng(M + N)
    A = wl.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    W = wl.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    b = rng.standard_normal(N).astype(np.float32)
    ref = O.linear(A, W, b)
    out = torch.empty(M, N, device=DEV)
    B.cs_linear_bf16(dev_bf16(A), dev_bf16(W), torch.from_numpy(b).to(DEV), out)
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy() - ref).max()
    print(f"linear {M}x{N}x{K}: max err {err:.3g}, max|ref| {np.abs(ref).max():.3g}", flush=True)
    assert err <= 2e-5 * math.sqrt(K) * np.abs(ref).max()       # fp32 accumulation of exact bf16 products
    outb = torch.empty(M, N, device=DEV, dtype=torch.bfloat16)
    B.cs_linear_bf16(dev_bf16(A), dev_bf16(W), None, outb)
    torch.cuda.synchronize()
    refb = O.linear(A, W)
    assert np.abs(outb.float().cpu().numpy() - refb).max() <= 2 ** -8 * np.abs(refb).max() + 1e-6


# sharp > 1: queries scaled up and keys growing along the sequence, so that the largest score of a query
# keeps rising from key tile to key tile by more than the kernel lets its running maximum lag behind
@pytest.mark.parametrize("dh,nh,segs,sharp", [(80, 2, [64, 16, 32, 4, 60, 64, 12], 1.0), (80, 3, [300, 1028, 64, 516], 1.0),
                                              (64, 2, [256, 40], 1.0), (64, 1, [1500], 1.0),
                                              (80, 2, [1028, 200, 64], 6.0), (64, 2, [1500, 70], 6.0)])
def test_attention_matches_oracle(dh, nh, segs, sharp):
    rng = np.random.default_rng(dh + len(segs))
    cu = np.concatenate([[0], np.cumsum(segs)])
    n, D = int(cu[-1]), nh * dh
    qs = wl.round_to_bf16(rng.standard_normal((n, D), dtype=np.float32) * np.float32(sharp * 1.4426950408889634 / math.sqrt(dh)))
    k = rng.standard_normal((n, D), dtype=np.float32)
    if sharp > 1.0:
        k *= (1.0 + np.arange(n, dtype=np.float32) / np.float32(n))[:, None]
    k = wl.round_to_bf16(k)
    v = wl.round_to_bf16(rng.standard_normal((n, D), dtype=np.float32))
    item = np.repeat(np.arange(len(segs)), segs)
    q = qs.astype(np.float64) * math.sqrt(dh) * math.log(2.0)        # undo the folded scale for the checker
    ref = O.attention(q.reshape(n, nh, dh), k.reshape(n, nh, dh).astype(np.float64),
                      v.reshape(n, nh, dh).astype(np.float64), item[:, None] == item[None, :]).reshape(n, D)
    qk = dev_bf16(np.concatenate([qs, k], 1))
    ld = (n + 7) // 8 * 8
    vt = torch.zeros(D, ld, device=DEV, dtype=torch.bfloat16)
    vt[:, :n] = dev_bf16(np.ascontiguousarray(v.T))
    out = torch.zeros(n, D, device=DEV, dtype=torch.bfloat16)
    B.cs_attention_varlen(qk, vt, out, cu, nh, dh)
    torch.cuda.synchronize()
    err = np.abs(out.float().cpu().numpy() - ref).max()
    print(f"attention dh={dh} segs={segs} sharp={sharp}: max err {err:.3g}", flush=True)
    assert err <= 2e-2        # probabilities and outputs are rounded to bf16 (2^-9 relative), |v| up to ~4


# ------------------------------------------------------------------ whole encoder task
def run_encode(w: wl.Workload):
    enc = B.Encoder(w.cfg, w.weights)
    out, _ = enc.cs_encode(dev_input(w), w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    return enc, out


def test_encode_c1_tiny_and_forward():
    """One 224x224 image through the tiny fp32 tower; rows land at positions 32..95."""
    w = wl.c1_tiny()
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, "c1")
    dst_bits = w.consumer_buffer_bits()
    dst = torch.from_numpy(dst_bits.view(np.int32)).to(DEV).view(torch.float32)
    B.cs_forward_embeddings(out, torch.from_numpy(w.placeholder_index).to(DEV), dst)
    torch.cuda.synchronize()
    got = dst.view(torch.int32).cpu().numpy().view(np.uint32)
    want = O.forward_embeddings(ref.astype(np.float32).view(np.uint32), w.placeholder_index, dst_bits)
    placed = np.zeros(len(dst_bits), bool)
    placed[w.placeholder_index] = True
    assert np.array_equal(got[~placed], want[~placed])                    # untouched rows keep their bits
    check_embeddings(torch.from_numpy(got[placed].view(np.float32)), want[placed].view(np.float32).astype(np.float64),
                     "c1 rows in the consumer buffer")


@pytest.mark.parametrize("sections", [(0, 20, 20), (8, 16, 16)])
def test_encode_small_ragged_vit(sections):
    """7B-shaped layers (hidden 1280, 16x80 heads, MLP 3420, merger 5120->3584) on three small images whose
    grids are not multiples of the window: truncated edge windows, window and full layers."""
    w = wl.small_vit(rope_sections=sections)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, f"small_vit{sections}")
    # bf16 output rows: the same values rounded once more
    w2 = replace(w, cfg=replace(w.cfg, out_dtype="bf16"))
    enc2, out2 = run_encode(w2)
    assert out2.dtype == torch.bfloat16
    assert torch.equal(out2, out.to(torch.bfloat16))
    # determinism and batch invariance
    out3, _ = enc.cs_encode(dev_input(w), w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    assert torch.equal(out3, out)
    one = w.select_items([1])
    o1, _ = enc.cs_encode(dev_input(one), one.cu_seqlens, one.grid_thw)
    torch.cuda.synchronize()
    a = int(w.out_rows[0])
    assert (o1 - out[a:a + int(w.out_rows[1])]).abs().max().item() <= 1e-2


def test_encode_smallest_items():
    """The degenerate sizes: a single 2x2-patch image (one embedding row), and a batch that mixes it
    with a one-window image and a one-merge-row strip."""
    for sizes in ([(28, 28)], [(28, 28), (112, 112), (28, 224)]):
        w = wl.small_vit(sizes_px=tuple(sizes), n_layers=2)
        ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
        enc, out = run_encode(w)
        assert out.shape[0] == sum((a // 28) * (b // 28) for a, b in sizes)
        check_embeddings(out, ref, f"tiny items {sizes}")


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_encode_random_small_batches(seed):
    """Seeded random batches of 1-4 images with sides of 2..12 patches (even), one window layer and
    one full layer: ragged windows of every size, items smaller than a window, mixed into one call."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 5))
    sizes = tuple((28 * int(rng.integers(1, 7)), 28 * int(rng.integers(1, 7))) for _ in range(n))
    w = wl.small_vit(sizes_px=sizes, n_layers=2)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, f"random batch {sizes}")


@pytest.mark.parametrize("window", [4, 16])
def test_encode_other_window_sizes(window):
    """Windows of 16 tokens, and of up to 256 tokens (four key tiles per 64-query work item)."""
    w = wl.small_vit(sizes_px=((252, 476), (84, 140)), n_layers=2)
    w = replace(w, cfg=replace(w.cfg, window=window))
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, f"window {window}")


def test_encode_video_clip_small():
    cfg = wl.vit_7b_config(2, rope_sections=(8, 16, 16))
    w = wl.video_workload("small_video", replace(cfg, full_attn_layers=(1,)), 1, 6, (140, 196), seq_len=512)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, "small_video")


def test_encode_small_audio():
    w = wl.audio_workload("small_audio", wl.audio_config(n_layers=2), n_clips=2, n_frames=400, seq_len=256)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, "small_audio")


@pytest.mark.parametrize("chunk", [8, 52, 100, 160])
def test_encode_small_audio_chunked_attention(chunk):
    """Block-diagonal attention over chunks of a clip: one-tile chunks (8, 52), two-tile chunks in
    64-query workgroups (100), and 256-query workgroups (160); 200 tokens per clip, so the last
    chunk is shorter in every case."""
    from dataclasses import replace
    w = wl.audio_workload("small_audio", replace(wl.audio_config(n_layers=2), attn_chunk=chunk), n_clips=2,
                          n_frames=400, seq_len=256)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    check_embeddings(out, ref, f"small_audio chunk {chunk}")
    whole = O.encode(replace(w.cfg, attn_chunk=0), w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    assert np.abs(whole - ref).max() > 1e-3          # the chunking does change the result


def test_encode_rejects_bad_batches():
    w = wl.small_vit(n_layers=1, full_layers=())
    enc = B.Encoder(w.cfg, w.weights)
    x = dev_input(w)
    bad_cu = w.cu_seqlens.copy(); bad_cu[1] += 4
    with pytest.raises(B.CsError) as e:
        enc.cs_encode(x, bad_cu, w.grid_thw)
    assert e.value.status == 2
    odd = w.grid_thw.copy(); odd[0] = (1, 3, 20)
    with pytest.raises(B.CsError):
        enc.cs_encode(x, w.cu_seqlens, odd)
    n_out, ws = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    out = torch.empty(n_out, w.cfg.out_hidden, device=DEV)
    small = torch.empty(ws - 256, dtype=torch.uint8, device=DEV)
    st = B.lib().cs_encode(enc._h, x.data_ptr(), B._i32p(B._i32(w.cu_seqlens)), B._i32p(B._i32(w.grid_thw)),
                           w.n_items, out.data_ptr(), small.data_ptr(), small.numel(), 0)
    assert st == 3
    torch.cuda.synchronize()


def test_mfma_ceiling_probe_reports_a_plausible_rate():
    """The bare MFMA loop: between a fifth of the nominal bf16 peak and the peak itself, and not
    faster with random operands (power-limited) than with zeros."""
    zero = B.cs_mfma_ceiling(False, iters=2000)
    rnd = B.cs_mfma_ceiling(True, iters=2000)
    assert 500.0 < rnd <= zero * 1.02 and zero < 2516.6 * 1.02, (zero, rnd)


# ------------------------------------------------------------------ pixels -> patch rows
@pytest.mark.parametrize("in_dtype,out_dtype", [(torch.float32, torch.bfloat16), (torch.float32, torch.float32),
                                                (torch.bfloat16, torch.bfloat16)])
def test_patchify_is_bit_exact(in_dtype, out_dtype):
    """Three items back to back (a still image, a non-square image, a 4-frame clip); every output word
    against the checker's explicit loops on the same stored values."""
    rng = np.random.default_rng(11)
    dims = [(1, 28, 42), (1, 56, 28), (4, 28, 28)]
    frames = [rng.random((F, 3, H, W)).astype(np.float32) for F, H, W in dims]
    if in_dtype == torch.bfloat16:
        frames = [wl.round_to_bf16(f) for f in frames]
    flat = torch.from_numpy(np.concatenate([f.ravel() for f in frames])).to(DEV).to(in_dtype)
    out, cu, grid = B.cs_patchify(flat, dims, temporal_patch=2, out_dtype=out_dtype)
    torch.cuda.synchronize()
    ref = [O.patchify(f, 2) for f in frames]
    assert grid.tolist() == [list(g) for _, g in ref]
    assert cu.tolist() == np.concatenate([[0], np.cumsum([p.shape[0] for p, _ in ref])]).tolist()
    want = np.concatenate([p for p, _ in ref])
    if out_dtype == torch.bfloat16:
        got = out.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, wl.to_bits_bf16(wl.round_to_bf16(want)))     # fp32 -> bf16: nearest even
    else:
        assert np.array_equal(out.cpu().numpy(), want)


def test_patchify_full_size_batch_and_into_the_encoder():
    """Eight 448x448 images: patch rows bit-exact against the checker, and the same bits as the
    benchmark workload's input, so cs_patchify -> cs_encode is the measured path fed from pixels."""
    w = wl.c2_images(n_layers=1)
    rng = np.random.default_rng(1)
    frames = [rng.random((1, 3, 448, 448), dtype=np.float32) for _ in range(8)]          # the workload's own recipe
    flat = torch.from_numpy(np.concatenate([f.ravel() for f in frames])).to(DEV)
    out, cu, grid = B.cs_patchify(flat, [(1, 448, 448)] * 8, temporal_patch=2)
    torch.cuda.synchronize()
    want = np.concatenate([O.patchify(f, 2)[0] for f in frames])
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, wl.to_bits_bf16(wl.round_to_bf16(want)))
    assert np.array_equal(cu, w.cu_seqlens) and np.array_equal(grid, w.grid_thw)
    assert np.array_equal(wl.to_bits_bf16(w.patches), got)
    enc = B.Encoder(w.cfg, w.weights)
    a, _ = enc.cs_encode(out, cu, grid)
    b, _ = enc.cs_encode(torch.from_numpy(wl.to_bits_bf16(w.patches).view(np.int16)).to(DEV).view(torch.bfloat16),
                         w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_merge_major_input_order_gives_the_same_embeddings():
    """The same ragged batch handed over merge group by merge group (the checker's permutation applied
    to the rows): identical bits out, since only the gather at the front of the path changes."""
    from dataclasses import replace
    w = wl.small_vit(n_layers=2)
    perm = O.merge_major_order(w.grid_thw, w.cfg.merge)
    x = torch.from_numpy(wl.to_bits_bf16(w.patches).view(np.int16)).to(DEV).view(torch.bfloat16)
    xm = x[torch.from_numpy(perm).to(DEV)].contiguous()
    a, _ = B.Encoder(w.cfg, w.weights).cs_encode(x, w.cu_seqlens, w.grid_thw)
    b, _ = B.Encoder(replace(w.cfg, input_order="merge_major"), w.weights).cs_encode(xm, w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and not torch.equal(x, xm)


def test_outputs_that_do_not_start_on_a_128_byte_line():
    """The kernels write through the L2 only where whole 128-byte lines are theirs; a destination that
    is merely 16-byte aligned must take the plain path and give the same bits."""
    rng = np.random.default_rng(31)
    # hand-off into a buffer that starts 16 bytes into an allocation
    rows, hidden, n_dst = 300, 512, 900
    src_bits = rng.integers(0, 1 << 16, size=(rows, hidden), dtype=np.uint16)
    dst_bits = rng.integers(0, 1 << 16, size=(n_dst, hidden), dtype=np.uint16)
    idx = rng.permutation(n_dst)[:rows].astype(np.int64)
    raw = torch.zeros(n_dst * hidden * 2 + 64, dtype=torch.uint8, device=DEV)
    dst = raw[16:16 + n_dst * hidden * 2].view(torch.bfloat16).view(n_dst, hidden)
    dst.copy_(torch.from_numpy(dst_bits.view(np.int16)).to(DEV).view(torch.bfloat16))
    assert dst.data_ptr() % 128 == 16
    src = torch.from_numpy(src_bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    B.cs_forward_embeddings(src, torch.from_numpy(idx).to(DEV), dst)
    torch.cuda.synchronize()
    got = dst.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, O.forward_embeddings(src_bits, idx, dst_bits))
    # GEMM output 16 bytes into an allocation, rows a multiple of 128 bytes
    M, N, K = 600, 512, 256
    A = wl.round_to_bf16(rng.standard_normal((M, K), dtype=np.float32))
    W = wl.round_to_bf16(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    raw2 = torch.zeros(M * N * 2 + 64, dtype=torch.uint8, device=DEV)
    out = raw2[16:16 + M * N * 2].view(torch.bfloat16).view(M, N)
    ref_out = torch.empty(M, N, device=DEV, dtype=torch.bfloat16)
    B.cs_linear_bf16(dev_bf16(A), dev_bf16(W), None, out)
    B.cs_linear_bf16(dev_bf16(A), dev_bf16(W), None, ref_out)
    torch.cuda.synchronize()
    assert out.data_ptr() % 128 == 16 and ref_out.data_ptr() % 128 == 0
    assert torch.equal(out, ref_out)
    assert np.abs(out.float().cpu().numpy() - O.linear(A, W)).max() <= 2 ** -8 * 12 + 1e-6


@pytest.mark.parametrize("tower", ["vit", "audio", "vit_cls"])
def test_encode_with_workspace_and_output_16_bytes_into_an_allocation(tower):
    """Every buffer of the path then starts 16 bytes past a 128-byte line, so every kernel takes its plain
    stores instead of the write-through ones: the embeddings must come out with the same bits."""
    if tower == "vit":
        w = wl.small_vit(n_layers=2)
    elif tower == "audio":
        w = wl.audio_workload("small_audio", wl.audio_config(n_layers=2), n_clips=2, n_frames=400, seq_len=256)
    else:
        w = wl.small_cls(n_layers=2)
    enc = B.Encoder(w.cfg, w.weights)
    x = dev_input(w)
    n_out, ws_bytes = enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)
    out, _ = enc.cs_encode(x, w.cu_seqlens, w.grid_thw)
    raw_ws = torch.empty(ws_bytes + 64, dtype=torch.uint8, device=DEV)
    raw_out = torch.empty(n_out * w.cfg.out_hidden * 4 + 64, dtype=torch.uint8, device=DEV)
    ws2 = raw_ws[16:16 + ws_bytes]
    out2 = raw_out[16:16 + n_out * w.cfg.out_hidden * 4].view(torch.float32).view(n_out, w.cfg.out_hidden)
    assert ws2.data_ptr() % 128 == 16 and out2.data_ptr() % 128 == 16 and out.data_ptr() % 128 == 0
    enc.cs_encode(x, w.cu_seqlens, w.grid_thw, out=out2, workspace=ws2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_calls_of_one_encoder_overlapping_on_two_streams():
    """Six calls of one encoder alternating between two streams, each stream with its own workspace and
    outputs, nothing synchronised in between (the per-batch index tables go through two pinned
    staging slots that are reused while earlier calls are still running): every result has the bits
    of the same batch run alone."""
    wa = wl.small_vit(n_layers=2)
    wb = wl.small_vit(sizes_px=((112, 56), (56, 280)), n_layers=2)
    enc = B.Encoder(wa.cfg, wa.weights)
    xa, xb = dev_input(wa), dev_input(wb)
    alone_a, _ = enc.cs_encode(xa, wa.cu_seqlens, wa.grid_thw)
    alone_b, _ = enc.cs_encode(xb, wb.cu_seqlens, wb.grid_thw)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    # all memory is allocated before the first call, so that nothing is handed out again while a call still uses it
    need = max(enc.cs_encoder_query(w.cu_seqlens, w.grid_thw)[1] for w in (wa, wb))
    ws = [torch.empty(need, dtype=torch.uint8, device=DEV) for _ in range(2)]
    plan = [(wa, xa, alone_a) if i % 3 != 1 else (wb, xb, alone_b) for i in range(6)]
    outs = [torch.empty_like(want) for (_, _, want) in plan]
    torch.cuda.synchronize()
    for i, (w, x, _) in enumerate(plan):
        enc.cs_encode(x, w.cu_seqlens, w.grid_thw, out=outs[i], workspace=ws[i % 2], stream=streams[i % 2])
    torch.cuda.synchronize()
    outs = [(o, want) for o, (_, _, want) in zip(outs, plan)]
    for i, (o, want) in enumerate(outs):
        assert torch.equal(o, want), f"call {i}"


# ------------------------------------------------------------------ class-token tower
@pytest.mark.parametrize("tile,n_tiles", [((6, 10), 3), ((2, 2), 1), ((16, 18), 2), ((32, 32), 1)])
def test_encode_class_token_tower(tile, n_tiles):
    """Tiles of 61, 5, 289 and 1025 tokens (none a multiple of what the kernels tile by): class token,
    learned positions, LayerNorm, full attention with the class token as a key, scaled branches,
    LayerNorm(4D) projector; several tiles per call."""
    w = wl.small_cls(tile_patches=tile, n_tiles=n_tiles, n_layers=2)
    ref = O.encode(w.cfg, w.weights, w.patches, w.cu_seqlens, w.grid_thw)
    enc, out = run_encode(w)
    assert out.shape == (n_tiles * tile[0] * tile[1] // 4, w.cfg.out_hidden)
    check_embeddings(out, ref, f"class-token tower, tiles {tile} x {n_tiles}")
    out2, _ = enc.cs_encode(dev_input(w), w.cu_seqlens, w.grid_thw)
    torch.cuda.synchronize()
    assert torch.equal(out2, out)
    if n_tiles > 1:                                   # a tile alone gives what it gives inside the batch
        one = w.select_items([n_tiles - 1])
        o1, _ = enc.cs_encode(dev_input(one), one.cu_seqlens, one.grid_thw)
        torch.cuda.synchronize()
        assert (o1 - out[-o1.shape[0]:]).abs().max().item() <= 1e-2


def test_class_token_tower_rejects_what_it_cannot_run():
    w = wl.small_cls(tile_patches=(6, 10), n_tiles=1, n_layers=1)
    enc = B.Encoder(w.cfg, w.weights)
    x = dev_input(w)
    with pytest.raises(B.CsError):                    # a tile that does not fit the position table
        enc.cs_encode(x[:48], np.array([0, 48], np.int32), np.array([[1, 6, 8]], np.int32))
    with pytest.raises(B.CsError):                    # window attention is not part of this tower
        B.Encoder(replace(w.cfg, window=8), w.weights)
    no_scale = {k: v for k, v in w.weights.items() if not k.endswith("ls1")}
    with pytest.raises(B.CsError):
        B.Encoder(w.cfg, no_scale)
