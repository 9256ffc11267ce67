"""Seeded synthetic workloads for the encoder task and the embedding hand-off.

This module only *draws and arranges numbers*: encoder configurations, random
weights, random images / clips / log-mel inputs, the patch extraction that a
preprocessor would do in front of the encoder, the consumer LLM's embedding
buffer and the placeholder positions.  It holds none of the encoder's
arithmetic, and both the GPU library's tests and the CPU checker's tests draw
their inputs from here so that the two sides read identical bytes.

The paper (Sec. 2.1 "Data Plane", Listing 1) fixes only the split into an
encoder task that yields one embedding tensor per multimodal item and an LLM
task that receives those tensors; it evaluates on a request trace that is not
reproduced here.  The five workloads below stand in for it: synthetic images,
video clips and audio with the shapes of a Qwen2.5-VL-style vision tower and a
Whisper-style audio tower.

Conventions
-----------
* every Linear weight is ``[out_features, in_features]``;
* values are drawn in fp32 and, for bf16 workloads, rounded to bf16
  (round-to-nearest-even); arrays keep the rounded values widened to fp32, and
  ``to_bits_bf16`` gives the 16-bit patterns a bf16 consumer stores;
* generators: weights seed 0, input data seed 1, shapes / placeholders seed 2.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

PATCH = 14  # pixels per patch side


# --------------------------------------------------------------------------
# bf16 rounding (storage format only)
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest bf16 value (ties to even), returned widened to fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def to_bits_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def from_bits_bf16(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# configuration
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class EncoderConfig:
    arch: str = "vit"            # "vit" | "audio" | "vit_cls" (class token, learned positions, LayerNorm, GELU)
    dtype: str = "bf16"          # storage type of weights and inputs: "bf16" | "f32"
    out_dtype: str = "f32"       # type of the embedding rows the encoder emits
    patch_dim: int = 1176        # vit: 3*tp*14*14 ; audio: n_mels
    temporal_patch: int = 2
    hidden: int = 1280
    n_heads: int = 16
    head_dim: int = 80
    n_layers: int = 32
    mlp_dim: int = 3420
    merge: int = 2               # vit: spatial merge side ; audio: frames pooled
    merger_hidden: int = 5120
    out_hidden: int = 3584
    window: int = 8              # in patches; <= 0: every layer attends over the whole item
    full_attn_layers: Tuple[int, ...] = (7, 15, 23, 31)
    rope_sections: Tuple[int, int, int] = (0, 20, 20)   # rotary pairs for (t, row, col)
    rope_theta: float = 10000.0
    norm_eps: float = 1e-6
    conv_kernel: int = 3         # audio only
    input_order: str = "raster"  # vit: "raster" or "merge_major" rows inside an item
    attn_chunk: int = 0          # audio: tokens per attention chunk (0: whole clip)
    tile_patches: Tuple[int, int] = (32, 32)   # vit_cls: patch grid of a tile (sizes the position table)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


def vit_tiny_config() -> EncoderConfig:
    return EncoderConfig(arch="vit", dtype="f32", out_dtype="f32", patch_dim=588, temporal_patch=1,
                         hidden=256, n_heads=4, head_dim=64, n_layers=2, mlp_dim=1024, merge=2,
                         merger_hidden=512, out_hidden=512, window=0, full_attn_layers=(),
                         rope_sections=(0, 16, 16))


def vit_7b_config(n_layers: int = 32, rope_sections=(0, 20, 20), out_dtype: str = "f32") -> EncoderConfig:
    full = tuple(l for l in (7, 15, 23, 31) if l < n_layers)
    return EncoderConfig(arch="vit", dtype="bf16", out_dtype=out_dtype, n_layers=n_layers,
                         full_attn_layers=full, rope_sections=tuple(rope_sections))


def vit_cls_config(n_layers: int = 24, out_dtype: str = "f32") -> EncoderConfig:
    """A 0.3B-class class-token tower (InternVL-style): 448x448 tiles of 32x32 patches, hidden 1024,
    16 heads of 64, MLP 4096, projector LayerNorm(4096) -> 4096 -> GELU -> 4096."""
    return EncoderConfig(arch="vit_cls", dtype="bf16", out_dtype=out_dtype, patch_dim=588, temporal_patch=1,
                         hidden=1024, n_heads=16, head_dim=64, n_layers=n_layers, mlp_dim=4096, merge=2,
                         merger_hidden=4096, out_hidden=4096, window=0, full_attn_layers=(),
                         rope_sections=(0, 0, 0), norm_eps=1e-6)


def audio_config(n_layers: int = 32, out_dtype: str = "f32") -> EncoderConfig:
    return EncoderConfig(arch="audio", dtype="bf16", out_dtype=out_dtype, patch_dim=128, temporal_patch=1,
                         hidden=1280, n_heads=20, head_dim=64, n_layers=n_layers, mlp_dim=5120, merge=2,
                         merger_hidden=0, out_hidden=3584, window=0, full_attn_layers=(),
                         rope_sections=(0, 0, 0), norm_eps=1e-5)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def weight_shapes(cfg: EncoderConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) in a fixed order; kind in {"w", "b", "g"} =
    matrix / bias / norm gain."""
    D, I, L = cfg.hidden, cfg.mlp_dim, cfg.n_layers
    out: List[Tuple[str, Tuple[int, ...], str]] = []
    if cfg.arch == "vit":
        out.append(("patch_embed.weight", (D, cfg.patch_dim), "w"))
        for l in range(L):
            p = f"blocks.{l}."
            out += [(p + "norm1.weight", (D,), "g"),
                    (p + "attn.qkv.weight", (3 * D, D), "w"), (p + "attn.qkv.bias", (3 * D,), "b"),
                    (p + "attn.proj.weight", (D, D), "w"), (p + "attn.proj.bias", (D,), "b"),
                    (p + "norm2.weight", (D,), "g"),
                    (p + "mlp.gate.weight", (I, D), "w"), (p + "mlp.gate.bias", (I,), "b"),
                    (p + "mlp.up.weight", (I, D), "w"), (p + "mlp.up.bias", (I,), "b"),
                    (p + "mlp.down.weight", (D, I), "w"), (p + "mlp.down.bias", (D,), "b")]
        g = cfg.merge * cfg.merge * D
        out += [("merger.norm.weight", (D,), "g"),
                ("merger.fc1.weight", (cfg.merger_hidden, g), "w"), ("merger.fc1.bias", (cfg.merger_hidden,), "b"),
                ("merger.fc2.weight", (cfg.out_hidden, cfg.merger_hidden), "w"),
                ("merger.fc2.bias", (cfg.out_hidden,), "b")]
    elif cfg.arch == "audio":
        k = cfg.conv_kernel
        out += [("conv1.weight", (D, cfg.patch_dim, k), "w"), ("conv1.bias", (D,), "b"),
                ("conv2.weight", (D, D, k), "w"), ("conv2.bias", (D,), "b")]
        for l in range(L):
            p = f"blocks.{l}."
            out += [(p + "norm1.weight", (D,), "g"), (p + "norm1.bias", (D,), "b"),
                    (p + "attn.qkv.weight", (3 * D, D), "w"), (p + "attn.qkv.bias", (3 * D,), "kb"),
                    (p + "attn.proj.weight", (D, D), "w"), (p + "attn.proj.bias", (D,), "b"),
                    (p + "norm2.weight", (D,), "g"), (p + "norm2.bias", (D,), "b"),
                    (p + "mlp.fc1.weight", (I, D), "w"), (p + "mlp.fc1.bias", (I,), "b"),
                    (p + "mlp.fc2.weight", (D, I), "w"), (p + "mlp.fc2.bias", (D,), "b")]
        out += [("post.norm.weight", (D,), "g"), ("post.norm.bias", (D,), "b"),
                ("post.proj.weight", (cfg.out_hidden, D), "w"), ("post.proj.bias", (cfg.out_hidden,), "b")]
    elif cfg.arch == "vit_cls":
        out += [("patch_embed.weight", (D, cfg.patch_dim), "w"), ("patch_embed.bias", (D,), "b"),
                ("cls_token", (D,), "b"), ("pos_embed", (1 + n_positions_grid(cfg), D), "b")]
        for l in range(L):
            p = f"blocks.{l}."
            out += [(p + "norm1.weight", (D,), "g"), (p + "norm1.bias", (D,), "b"),
                    (p + "attn.qkv.weight", (3 * D, D), "w"), (p + "attn.qkv.bias", (3 * D,), "b"),
                    (p + "attn.proj.weight", (D, D), "w"), (p + "attn.proj.bias", (D,), "b"), (p + "ls1", (D,), "s"),
                    (p + "norm2.weight", (D,), "g"), (p + "norm2.bias", (D,), "b"),
                    (p + "mlp.fc1.weight", (I, D), "w"), (p + "mlp.fc1.bias", (I,), "b"),
                    (p + "mlp.fc2.weight", (D, I), "w"), (p + "mlp.fc2.bias", (D,), "b"), (p + "ls2", (D,), "s")]
        g = cfg.merge * cfg.merge * D
        out += [("merger.norm.weight", (g,), "g"), ("merger.norm.bias", (g,), "b"),
                ("merger.fc1.weight", (cfg.merger_hidden, g), "w"), ("merger.fc1.bias", (cfg.merger_hidden,), "b"),
                ("merger.fc2.weight", (cfg.out_hidden, cfg.merger_hidden), "w"),
                ("merger.fc2.bias", (cfg.out_hidden,), "b")]
    else:
        raise ValueError(cfg.arch)
    return out


def n_positions_grid(cfg: EncoderConfig) -> int:
    """Patches per tile of a class-token tower (its position table has one more row)."""
    return cfg.tile_patches[0] * cfg.tile_patches[1]


def make_weights(cfg: EncoderConfig, seed: int = 0, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Random-init weights: matrices and biases ~ N(0, std); norm gains 1 + N(0, std); the
    branch scales of the class-token tower 0.1 + N(0, std) (such towers start them at 0.1).
    The key-projection third of the audio qkv bias is zero (that tower has no key bias)."""
    rng = np.random.default_rng(seed)
    W: Dict[str, np.ndarray] = {}
    for name, shape, kind in weight_shapes(cfg):
        a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if kind == "g":
            a = a + np.float32(1.0)
        if kind == "s":
            a = a + np.float32(0.1)
        if kind == "kb":
            a[cfg.hidden:2 * cfg.hidden] = 0.0
        if cfg.dtype == "bf16":
            a = round_to_bf16(a)
        W[name] = a
    return W


# --------------------------------------------------------------------------
# patch extraction (what the preprocessor in front of the encoder does)
# --------------------------------------------------------------------------
def patchify(frames: np.ndarray, temporal_patch: int) -> Tuple[np.ndarray, Tuple[int, int, int]]:
    """frames ``[F, 3, Hpix, Wpix]`` -> patches ``[T*h*w, 3*tp*14*14]`` in raster order
    (t, row, col); inside one patch the element order is (channel, temporal, py, px).
    A single frame with temporal_patch 2 is shown twice."""
    F, C, Hp, Wp = frames.shape
    tp = temporal_patch
    if F == 1 and tp > 1:
        frames = np.repeat(frames, tp, axis=0)
        F = tp
    assert F % tp == 0 and Hp % PATCH == 0 and Wp % PATCH == 0
    T, h, w = F // tp, Hp // PATCH, Wp // PATCH
    x = frames.reshape(T, tp, C, h, PATCH, w, PATCH)
    x = x.transpose(0, 3, 5, 2, 1, 4, 6)          # T h w C tp py px
    return np.ascontiguousarray(x.reshape(T * h * w, C * tp * PATCH * PATCH)), (T, h, w)


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    cfg: EncoderConfig
    patches: np.ndarray          # [N, patch_dim] fp32 (rounded to cfg.dtype); audio: [sum frames, n_mels]
    cu_seqlens: np.ndarray       # int32 [B+1]
    grid_thw: np.ndarray         # int32 [B,3]; audio items are (1, 1, frames)
    out_rows: np.ndarray         # int64 [B] embedding rows each item yields
    seq_len: int                 # tokens per consumer sequence
    placeholder_index: np.ndarray  # int64 [sum out_rows] flat row in the consumer buffer
    weight_seed: int = 0
    _weights: Optional[Dict[str, np.ndarray]] = field(default=None, repr=False)

    @property
    def weights(self) -> Dict[str, np.ndarray]:
        if self._weights is None:
            self._weights = make_weights(self.cfg, self.weight_seed)
        return self._weights

    @property
    def n_items(self) -> int:
        return int(self.grid_thw.shape[0])

    @property
    def n_sequences(self) -> int:
        return self.n_items

    def consumer_buffer_bits(self, seed: int = 3) -> np.ndarray:
        """The consumer LLM's input-embedding buffer before the hand-off, as raw storage
        words (uint16 for bf16 rows, uint32 for fp32 rows) filled with seeded random bits."""
        rng = np.random.default_rng(seed)
        rows = self.n_sequences * self.seq_len
        if self.cfg.out_dtype == "bf16":
            return rng.integers(0, 1 << 16, size=(rows, self.cfg.out_hidden), dtype=np.uint16)
        return rng.integers(0, 1 << 32, size=(rows, self.cfg.out_hidden), dtype=np.uint32)

    def select_items(self, items: List[int]) -> "Workload":
        """The same workload restricted to some items (items are independent)."""
        cu = [0]
        parts = []
        for i in items:
            a, b = int(self.cu_seqlens[i]), int(self.cu_seqlens[i + 1])
            parts.append(self.patches[a:b])
            cu.append(cu[-1] + b - a)
        out_rows = self.out_rows[items]
        ocu = np.concatenate([[0], np.cumsum(self.out_rows)])
        idx = []
        for j, i in enumerate(items):
            seg = self.placeholder_index[ocu[i]:ocu[i + 1]]
            idx.append(seg - i * self.seq_len + j * self.seq_len)
        return Workload(name=f"{self.name}[{','.join(map(str, items))}]", cfg=self.cfg,
                        patches=np.concatenate(parts, 0), cu_seqlens=np.asarray(cu, np.int32),
                        grid_thw=self.grid_thw[items].copy(), out_rows=out_rows, seq_len=self.seq_len,
                        placeholder_index=np.concatenate(idx), weight_seed=self.weight_seed,
                        _weights=self._weights)


def _spans(out_rows: np.ndarray, seq_len: int, rng: np.random.Generator) -> np.ndarray:
    """One contiguous span of placeholder positions per sequence, at a random start."""
    idx = []
    for b, m in enumerate(out_rows):
        start = int(rng.integers(0, seq_len - int(m) + 1))
        idx.append(b * seq_len + start + np.arange(int(m), dtype=np.int64))
    return np.concatenate(idx)


def _finish_inputs(cfg: EncoderConfig, parts: List[np.ndarray]) -> np.ndarray:
    x = np.concatenate(parts, 0).astype(np.float32)
    return round_to_bf16(x) if cfg.dtype == "bf16" else x


def _vit_workload(name, cfg, frame_sets, seq_len, fixed_start=None) -> Workload:
    parts, grids = [], []
    for fr in frame_sets:
        p, g = patchify(fr, cfg.temporal_patch)
        parts.append(p)
        grids.append(g)
    grid = np.asarray(grids, np.int32)
    n = grid.prod(1)
    cu = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    out_rows = (n // (cfg.merge * cfg.merge)).astype(np.int64)
    if fixed_start is None:
        idx = _spans(out_rows, seq_len, np.random.default_rng(2))
    else:
        idx = np.concatenate([b * seq_len + fixed_start + np.arange(int(m), dtype=np.int64)
                              for b, m in enumerate(out_rows)])
    return Workload(name, cfg, _finish_inputs(cfg, parts), cu, grid, out_rows, seq_len, idx)


def images_workload(name: str, cfg: EncoderConfig, sizes_px: List[Tuple[int, int]], seq_len: int,
                    data_seed: int = 1, fixed_start=None) -> Workload:
    rng = np.random.default_rng(data_seed)
    frames = [rng.random((1, 3, hp, wp), dtype=np.float32) for hp, wp in sizes_px]
    return _vit_workload(name, cfg, frames, seq_len, fixed_start)


def video_workload(name: str, cfg: EncoderConfig, n_clips: int, n_frames: int, size_px: Tuple[int, int],
                   seq_len: int, data_seed: int = 1) -> Workload:
    rng = np.random.default_rng(data_seed)
    frames = [rng.random((n_frames, 3, size_px[0], size_px[1]), dtype=np.float32) for _ in range(n_clips)]
    return _vit_workload(name, cfg, frames, seq_len)


def audio_workload(name: str, cfg: EncoderConfig, n_clips: int, n_frames: int, seq_len: int,
                   data_seed: int = 1) -> Workload:
    """Log-mel inputs ~ N(0,1), handed over frame-major: rows are mel frames, columns mel bins."""
    rng = np.random.default_rng(data_seed)
    parts = [np.ascontiguousarray(rng.standard_normal((cfg.patch_dim, n_frames), dtype=np.float32).T)
             for _ in range(n_clips)]
    grid = np.asarray([(1, 1, n_frames)] * n_clips, np.int32)
    cu = (np.arange(n_clips + 1) * n_frames).astype(np.int32)
    out_rows = np.full(n_clips, n_frames // 2 // cfg.merge, np.int64)
    idx = _spans(out_rows, seq_len, np.random.default_rng(2))
    return Workload(name, cfg, _finish_inputs(cfg, parts), cu, grid, out_rows, seq_len, idx)


def varlen_image_sizes(n_images: int = 32, seed: int = 2) -> List[Tuple[int, int]]:
    """Height and width drawn independently and uniformly from the multiples of 28 in [224, 1344]."""
    rng = np.random.default_rng(seed)
    k = rng.integers(8, 49, size=(n_images, 2))
    return [(int(a) * 28, int(b) * 28) for a, b in k]


def c1_tiny() -> Workload:
    """One 224x224 image through the tiny fp32 tower; 64 rows land at positions 32..95 of a
    128-token sequence."""
    return images_workload("c1_tiny", vit_tiny_config(), [(224, 224)], seq_len=128, fixed_start=32)


def c2_images(n_layers: int = 32, n_images: int = 8, out_dtype: str = "f32") -> Workload:
    """Eight 448x448 images (1024 patches each) through the 7B-style tower."""
    return images_workload("c2_images", vit_7b_config(n_layers, out_dtype=out_dtype),
                           [(448, 448)] * n_images, seq_len=2048)


def c3_varlen(n_layers: int = 32, n_images: int = 32, out_dtype: str = "f32") -> Workload:
    """Thirty-two images of mixed sizes packed into one variable-length batch."""
    return images_workload("c3_varlen", vit_7b_config(n_layers, out_dtype=out_dtype),
                           varlen_image_sizes(n_images), seq_len=4096)


def c4_video(n_layers: int = 32, n_clips: int = 2, n_frames: int = 16, out_dtype: str = "f32") -> Workload:
    """Two 16-frame 448x448 clips; rotary over (t, row, col)."""
    return video_workload("c4_video", vit_7b_config(n_layers, rope_sections=(8, 16, 16), out_dtype=out_dtype),
                          n_clips, n_frames, (448, 448), seq_len=16384)


def c5_audio(n_layers: int = 32, n_clips: int = 16, n_frames: int = 3000, out_dtype: str = "f32") -> Workload:
    """Sixteen 30 s log-mel clips through the Whisper-style tower."""
    return audio_workload("c5_audio", audio_config(n_layers, out_dtype=out_dtype), n_clips, n_frames,
                          seq_len=2048)


def small_vit(sizes_px=((84, 140), (252, 476), (56, 56)), n_layers: int = 3, dtype: str = "bf16",
              rope_sections=(0, 20, 20), full_layers=(1,), hidden_scale: int = 1) -> Workload:
    """A shallow 7B-shaped tower on a few small ragged images: grids that are not multiples of the
    window, so edge windows are truncated, yet cheap enough for the checker to run in seconds."""
    cfg = replace(vit_7b_config(n_layers, rope_sections=rope_sections), dtype=dtype,
                  full_attn_layers=tuple(full_layers))
    return images_workload("small_vit", cfg, list(sizes_px), seq_len=1024)


def c6_tiles(n_layers: int = 24, n_tiles: int = 8, out_dtype: str = "f32") -> Workload:
    """Eight 448x448 tiles (1024 patches + a class token each) through the class-token tower."""
    cfg = vit_cls_config(n_layers, out_dtype=out_dtype)
    return images_workload("c6_tiles", cfg, [(448, 448)] * n_tiles, seq_len=2048)


def small_cls(tile_patches=(6, 10), n_tiles: int = 3, n_layers: int = 2, dtype: str = "bf16") -> Workload:
    """A shallow class-token tower of the 0.3B shape on a few small tiles (61 tokens each for the
    default 6x10 grid: not a multiple of anything the kernels tile by)."""
    cfg = replace(vit_cls_config(n_layers), dtype=dtype, tile_patches=tuple(tile_patches))
    px = (tile_patches[0] * PATCH, tile_patches[1] * PATCH)
    return images_workload("small_cls", cfg, [px] * n_tiles, seq_len=256)
