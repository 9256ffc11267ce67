"""CPU checker ("oracle") for the encoder task and the embedding hand-off.

TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the GPU
library must compute, written with numpy in fp64, one operator at a time, in
raster token order, with dense boolean attention masks and no tiling, fusion or
reordering.  It shares no code with the GPU path and imports nothing from it;
only tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What the paper fixes (Sec. 2.1 "Data Plane"; Sec. 2.2 "Model Fission", Listing 1)
is the boundary: an encoder task turns each multimodal item of a request into
one embedding tensor, the tensors are appended in item order, and an LLM task
created to receive embeddings places them into its input instead of running an
encoder of its own.  The paper does not describe the inside of any encoder; the
operator definitions below are the standard ones for a Qwen2.5-VL-style vision
tower and a Whisper-style audio tower, with every reading that the paper leaves
open listed next to the function that takes it.

Pins: every function below is checked in tests/test_oracle_pins.py against
something other than itself (library routines of CPU PyTorch, closed forms,
invariants, brute-force loops, hand-computed indices).  The composition of a
whole tower has no printed reference activations anywhere; it is pinned by an
independent second composition built from PyTorch modules on small inputs.

Weights are ``[out_features, in_features]``; all inputs may be fp32 arrays (the
storage-rounded values); everything is widened to fp64 on entry.
"""
from __future__ import annotations

import math
from typing import Dict, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------
# elementwise and normalisation operators
# --------------------------------------------------------------------------
def linear(x: np.ndarray, W: np.ndarray, b=None) -> np.ndarray:
    """y = x W^T + b, W is [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(W, F64).T
    if b is not None:
        y = y + np.asarray(b, F64)
    return y


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i, per row."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def layernorm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    """y = (x - mean) / sqrt(var + eps) * g + b with the biased (1/n) variance, per row."""
    x = np.asarray(x, F64)
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(g, F64) + np.asarray(b, F64)


def silu(z: np.ndarray) -> np.ndarray:
    """z / (1 + exp(-z))."""
    z = np.asarray(z, F64)
    return z / (1.0 + np.exp(-z))


def gelu(z: np.ndarray) -> np.ndarray:
    """Exact GELU: z/2 * (1 + erf(z / sqrt 2))."""
    z = np.asarray(z, F64)
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


# --------------------------------------------------------------------------
# token geometry
# --------------------------------------------------------------------------
def token_coords(grid_thw: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """For a packed batch in raster order: item index ``[N]`` and position ``[N,3]`` =
    (t, row, col) in patch units, each item starting at (0,0,0)."""
    items, pos = [], []
    for i, (T, h, w) in enumerate(np.asarray(grid_thw).tolist()):
        t, r, c = np.meshgrid(np.arange(T), np.arange(h), np.arange(w), indexing="ij")
        pos.append(np.stack([t.ravel(), r.ravel(), c.ravel()], 1))
        items.append(np.full(T * h * w, i))
    return np.concatenate(items), np.concatenate(pos, 0)


def attention_allowed(item: np.ndarray, pos: np.ndarray, window: int) -> np.ndarray:
    """Boolean ``[N,N]``: may query p look at key p'?

    Full attention (window <= 0): same item.  Window attention: same item, same t,
    and the same window of ``window x window`` patches, windows tiling the frame from
    its top-left corner (the last window of a row or column is simply smaller when
    the grid is not a multiple of the window; no padding token takes part)."""
    same = item[:, None] == item[None, :]
    if window <= 0:
        return same
    t, r, c = pos[:, 0], pos[:, 1], pos[:, 2]
    wr, wc = r // window, c // window
    return same & (t[:, None] == t[None, :]) & (wr[:, None] == wr[None, :]) & (wc[:, None] == wc[None, :])


# --------------------------------------------------------------------------
# rotary position embedding
# --------------------------------------------------------------------------
def rotary_angles(pos: np.ndarray, sections: Sequence[int], theta: float) -> np.ndarray:
    """Angles ``[N, head_dim/2]``.  Rotary pair j belongs to the axis a whose section
    contains j (sections are laid out [t | row | col]); with i its offset inside that
    section of n_a pairs, angle_j = pos_a * theta^(-i / n_a)."""
    cols = []
    for a, n_a in enumerate(sections):
        for i in range(n_a):
            cols.append(np.asarray(pos[:, a], F64) * theta ** (-i / n_a))
    return np.stack(cols, 1) if cols else np.zeros((pos.shape[0], 0))


def apply_rotary(x: np.ndarray, ang: np.ndarray) -> np.ndarray:
    """x ``[N, heads, dh]``; pair j couples elements j and j + dh/2:
    (a, b) -> (a cos - b sin, b cos + a sin)."""
    x = np.asarray(x, F64)
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    cs, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    return np.concatenate([a * cs - b * sn, b * cs + a * sn], -1)


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, allowed: np.ndarray) -> np.ndarray:
    """softmax over the allowed keys of q k^T / sqrt(dh), times v; q,k,v ``[N, heads, dh]``."""
    N, nh, dh = q.shape
    out = np.empty((N, nh, dh), F64)
    for h in range(nh):
        s = (q[:, h, :] @ k[:, h, :].T) / math.sqrt(dh)
        s = np.where(allowed, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, h, :]
    return out


# --------------------------------------------------------------------------
# vision tower
# --------------------------------------------------------------------------
def merge_index(grid_thw: np.ndarray, merge: int) -> np.ndarray:
    """``[M, merge*merge]`` packed-batch patch indices feeding each merged token.  Merged
    token (t, R, C) of an item takes patches (t, 2R+dr, 2C+dc) in the order
    (dr,dc) = (0,0),(0,1),(1,0),(1,1); merged tokens are in raster order (t, R, C),
    items in input order."""
    rows, base = [], 0
    for (T, h, w) in np.asarray(grid_thw).tolist():
        for t in range(T):
            for R in range(h // merge):
                for C in range(w // merge):
                    rows.append([base + (t * h + merge * R + dr) * w + merge * C + dc
                                 for dr in range(merge) for dc in range(merge)])
        base += T * h * w
    return np.asarray(rows, np.int64)


def vit_block(x, W, p, cfg, ang, allowed):
    """Pre-norm transformer block with SwiGLU MLP (residual stream x ``[N, D]``)."""
    N = x.shape[0]
    nh, dh, D = cfg.n_heads, cfg.head_dim, cfg.hidden
    u = rmsnorm(x, W[p + "norm1.weight"], cfg.norm_eps)
    qkv = linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"])
    q = apply_rotary(qkv[:, 0 * D:1 * D].reshape(N, nh, dh), ang)
    k = apply_rotary(qkv[:, 1 * D:2 * D].reshape(N, nh, dh), ang)
    v = qkv[:, 2 * D:3 * D].reshape(N, nh, dh)
    a = attention(q, k, v, allowed).reshape(N, D)
    x = x + linear(a, W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
    u = rmsnorm(x, W[p + "norm2.weight"], cfg.norm_eps)
    m = silu(linear(u, W[p + "mlp.gate.weight"], W[p + "mlp.gate.bias"])) * \
        linear(u, W[p + "mlp.up.weight"], W[p + "mlp.up.bias"])
    return x + linear(m, W[p + "mlp.down.weight"], W[p + "mlp.down.bias"])


def vit_encode(cfg, W: Dict[str, np.ndarray], patches: np.ndarray, grid_thw: np.ndarray) -> np.ndarray:
    """The image / video encoder task: packed patches ``[N, patch_dim]`` (raster order per
    item) -> embedding rows ``[N / merge^2, out_hidden]``, item after item."""
    item, pos = token_coords(grid_thw)
    assert patches.shape[0] == item.shape[0]
    ang = rotary_angles(pos, cfg.rope_sections, cfg.rope_theta)
    full = attention_allowed(item, pos, 0)
    win = attention_allowed(item, pos, cfg.window) if cfg.window > 0 else full
    x = linear(patches, W["patch_embed.weight"])
    for l in range(cfg.n_layers):
        allowed = full if (cfg.window <= 0 or l in cfg.full_attn_layers) else win
        x = vit_block(x, W, f"blocks.{l}.", cfg, ang, allowed)
    z = rmsnorm(x, W["merger.norm.weight"], cfg.norm_eps)
    zc = z[merge_index(grid_thw, cfg.merge)].reshape(-1, cfg.merge * cfg.merge * cfg.hidden)
    y = gelu(linear(zc, W["merger.fc1.weight"], W["merger.fc1.bias"]))
    return linear(y, W["merger.fc2.weight"], W["merger.fc2.bias"])


# --------------------------------------------------------------------------
# audio tower
# --------------------------------------------------------------------------
def conv1d(x: np.ndarray, W: np.ndarray, b: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """x ``[Cin, T]``, W ``[Cout, Cin, k]``: y[o, t] = b[o] + sum_{c,d} W[o,c,d] x[c, t*stride + d - pad],
    zero outside [0, T)."""
    x = np.asarray(x, F64)
    W = np.asarray(W, F64)
    Cin, T = x.shape
    Cout, _, k = W.shape
    xp = np.zeros((Cin, T + 2 * pad), F64)
    xp[:, pad:pad + T] = x
    Tout = (T + 2 * pad - k) // stride + 1
    y = np.tile(np.asarray(b, F64)[:, None], (1, Tout))
    for d in range(k):
        y += W[:, :, d] @ xp[:, d:d + stride * (Tout - 1) + 1:stride]
    return y


def sinusoid_positions(length: int, channels: int) -> np.ndarray:
    """PE[pos, i] = sin(pos w_i) for i < C/2 and cos(pos w_{i-C/2}) after,
    w_i = exp(-i ln(10000) / (C/2 - 1))."""
    half = channels // 2
    w = np.exp(-np.arange(half, dtype=F64) * math.log(10000.0) / (half - 1))
    a = np.arange(length, dtype=F64)[:, None] * w[None, :]
    return np.concatenate([np.sin(a), np.cos(a)], 1)


def audio_attention_allowed(clip_tokens: Sequence[int], chunk: int) -> np.ndarray:
    """Boolean ``[N,N]`` for a batch of clips with the given token counts: a token sees the tokens
    of its own clip, and with chunk > 0 only those of its own chunk of `chunk` consecutive tokens
    of that clip (chunks counted from the clip's first token; the last may be shorter)."""
    item = np.concatenate([np.full(n, i) for i, n in enumerate(clip_tokens)])
    allowed = item[:, None] == item[None, :]
    if chunk > 0:
        local = np.concatenate([np.arange(n) for n in clip_tokens])
        allowed = allowed & ((local // chunk)[:, None] == (local // chunk)[None, :])
    return allowed


def audio_block(x, W, p, cfg, allowed):
    N = x.shape[0]
    nh, dh, D = cfg.n_heads, cfg.head_dim, cfg.hidden
    u = layernorm(x, W[p + "norm1.weight"], W[p + "norm1.bias"], cfg.norm_eps)
    qkv = linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"])
    q, k, v = (qkv[:, i * D:(i + 1) * D].reshape(N, nh, dh) for i in range(3))
    a = attention(q, k, v, allowed).reshape(N, D)
    x = x + linear(a, W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
    u = layernorm(x, W[p + "norm2.weight"], W[p + "norm2.bias"], cfg.norm_eps)
    return x + linear(gelu(linear(u, W[p + "mlp.fc1.weight"], W[p + "mlp.fc1.bias"])),
                      W[p + "mlp.fc2.weight"], W[p + "mlp.fc2.bias"])


def audio_encode(cfg, W: Dict[str, np.ndarray], frames: np.ndarray, cu_seqlens: np.ndarray) -> np.ndarray:
    """The audio encoder task: frame-major log-mel rows ``[sum T_i, n_mels]`` ->
    ``[sum T_i/4, out_hidden]``.  Two k=3 convolutions (stride 1 then 2, padding 1), each
    followed by GELU; sinusoidal positions; pre-LayerNorm blocks with full attention
    inside a clip (or, with cfg.attn_chunk > 0, inside each chunk of that many tokens of a clip:
    the block-diagonal attention long-audio encoders use; the convolutions and positions still
    run over the whole clip, which is the reading taken here); mean over frame pairs; LayerNorm;
    projection."""
    xs = []
    for i in range(len(cu_seqlens) - 1):
        mel = np.asarray(frames[cu_seqlens[i]:cu_seqlens[i + 1]], F64).T      # [n_mels, T]
        c1 = gelu(conv1d(mel, W["conv1.weight"], W["conv1.bias"], 1, 1))
        c2 = gelu(conv1d(c1, W["conv2.weight"], W["conv2.bias"], 2, 1))
        xi = c2.T + sinusoid_positions(c2.shape[1], cfg.hidden)
        xs.append(xi)
    x = np.concatenate(xs, 0)
    allowed = audio_attention_allowed([xi.shape[0] for xi in xs], getattr(cfg, "attn_chunk", 0))
    for l in range(cfg.n_layers):
        x = audio_block(x, W, f"blocks.{l}.", cfg, allowed)
    m = cfg.merge
    pooled = x.reshape(-1, m, cfg.hidden).mean(axis=1)      # clip lengths are multiples of m
    z = layernorm(pooled, W["post.norm.weight"], W["post.norm.bias"], cfg.norm_eps)
    return linear(z, W["post.proj.weight"], W["post.proj.bias"])


# --------------------------------------------------------------------------
# class-token vision tower (InternVL-style)
# --------------------------------------------------------------------------
def cls_block(x, W, p, cfg):
    """Pre-LayerNorm block over one image tile's tokens ``[1 + h*w, D]``: full attention, GELU
    MLP, and a learned per-channel scale on each branch before it joins the residual stream."""
    N, nh, dh, D = x.shape[0], cfg.n_heads, cfg.head_dim, cfg.hidden
    u = layernorm(x, W[p + "norm1.weight"], W[p + "norm1.bias"], cfg.norm_eps)
    qkv = linear(u, W[p + "attn.qkv.weight"], W[p + "attn.qkv.bias"])
    q, k, v = (qkv[:, i * D:(i + 1) * D].reshape(N, nh, dh) for i in range(3))
    a = attention(q, k, v, np.ones((N, N), bool)).reshape(N, D)
    x = x + W[p + "ls1"] * linear(a, W[p + "attn.proj.weight"], W[p + "attn.proj.bias"])
    u = layernorm(x, W[p + "norm2.weight"], W[p + "norm2.bias"], cfg.norm_eps)
    m = gelu(linear(u, W[p + "mlp.fc1.weight"], W[p + "mlp.fc1.bias"]))
    return x + W[p + "ls2"] * linear(m, W[p + "mlp.fc2.weight"], W[p + "mlp.fc2.bias"])


def cls_encode(cfg, W: Dict[str, np.ndarray], patches: np.ndarray, grid_thw: np.ndarray) -> np.ndarray:
    """The encoder task of a class-token vision tower, the kind InternVL-style models use (the paper
    names that family among the models it serves, Sec. 1 and Table 1, and says nothing of its inside): per tile
    (item, grid (1, h, w), raster patch rows) the tokens are [class token, patches], learned
    absolute positions are added (row 0 for the class token, row 1 + r*w + c for patch (r, c)),
    the blocks run with full attention inside the tile, the class token is dropped, every 2x2
    group of patches is concatenated in the order (r0c0, r0c1, r1c0, r1c1), and the projector
    LayerNorm(4D) -> Linear -> GELU -> Linear gives one embedding row per group, in raster order
    of the groups.  Returns ``[N / 4, out_hidden]``, tile after tile."""
    D, outs, base = cfg.hidden, [], 0
    g64 = np.asarray(grid_thw, np.int64)
    for T, h, w in g64.tolist():
        assert T == 1 and 1 + h * w == W["pos_embed"].shape[0]
        n = h * w
        x = linear(patches[base:base + n], W["patch_embed.weight"], W["patch_embed.bias"])
        x = np.concatenate([np.asarray(W["cls_token"], np.float64).reshape(1, D), x], 0) + W["pos_embed"]
        for l in range(cfg.n_layers):
            x = cls_block(x, W, f"blocks.{l}.", cfg)
        z = x[1:].reshape(h, w, D)
        zc = np.stack([np.concatenate([z[2 * R, 2 * C], z[2 * R, 2 * C + 1], z[2 * R + 1, 2 * C], z[2 * R + 1, 2 * C + 1]])
                       for R in range(h // 2) for C in range(w // 2)])
        zc = layernorm(zc, W["merger.norm.weight"], W["merger.norm.bias"], cfg.norm_eps)
        y = gelu(linear(zc, W["merger.fc1.weight"], W["merger.fc1.bias"]))
        outs.append(linear(y, W["merger.fc2.weight"], W["merger.fc2.bias"]))
        base += n
    return np.concatenate(outs, 0)


def encode(cfg, W, patches, cu_seqlens, grid_thw) -> np.ndarray:
    if cfg.arch == "vit":
        return vit_encode(cfg, W, patches, grid_thw)
    if cfg.arch == "vit_cls":
        return cls_encode(cfg, W, patches, grid_thw)
    return audio_encode(cfg, W, patches, cu_seqlens)


# --------------------------------------------------------------------------
# pixels -> patch rows (the step in front of the encoder task)
# --------------------------------------------------------------------------
def patchify(frames: np.ndarray, temporal_patch: int, patch: int = 14) -> Tuple[np.ndarray, Tuple[int, int, int]]:
    """frames [F, 3, H, W] of one item -> (patch rows [T*h*w, 3*tp*patch*patch], (T, h, w)).

    Patch (t, r, c) is row (t*h + r)*w + c; inside the row, element
    ((ch*tp + tt)*patch + py)*patch + px is pixel frames[t*tp + tt, ch, r*patch + py, c*patch + px].
    An item with a single frame shows that frame in every temporal slot.  Values are copied as they
    are (no arithmetic); the dtype of `frames` is kept.  Reading: the paper says nothing
    of preprocessing (in Listing 1 the encoder task is handed the request's multimodal data as it
    is); this is the layout such vision towers take."""
    F, C, H, W = frames.shape
    tp = temporal_patch
    assert C == 3 and H % patch == 0 and W % patch == 0 and (F == 1 or F % tp == 0)
    T, h, w = (1 if F == 1 else F // tp), H // patch, W // patch
    out = np.empty((T * h * w, C * tp * patch * patch), frames.dtype)
    for t in range(T):
        for r in range(h):
            for c in range(w):
                row = out[(t * h + r) * w + c].reshape(C, tp, patch, patch)
                for tt in range(tp):
                    f = 0 if F == 1 else t * tp + tt
                    row[:, tt] = frames[f, :, r * patch:(r + 1) * patch, c * patch:(c + 1) * patch]
    return out, (T, h, w)


def merge_major_order(grid_thw: np.ndarray, merge: int = 2) -> np.ndarray:
    """Row permutation between the two input orders of a packed batch: entry i is the raster row
    (t, row, col order inside each item) of the patch that sits at row i when every item is listed
    merge group by merge group, (t, row/merge, col/merge, row%merge, col%merge), which is how the
    stock preprocessors of such vision towers emit patches.  raster_patches[perm] is the
    merge-major batch."""
    perm = []
    base = 0
    for (T, h, w) in np.asarray(grid_thw).tolist():
        for t in range(T):
            for R in range(h // merge):
                for C in range(w // merge):
                    for dr in range(merge):
                        for dc in range(merge):
                            perm.append(base + (t * h + R * merge + dr) * w + C * merge + dc)
        base += T * h * w
    return np.asarray(perm, np.int64)


# --------------------------------------------------------------------------
# which pending items share the next packed call
# --------------------------------------------------------------------------
def pack_batch(rows: Sequence[int], row_budget: int, max_items: int) -> list:
    """First-fit in arrival order: `rows` lists the pending items' input-row counts oldest first.
    The oldest item is always taken; every later one is taken when the total stays within the
    budget and fewer than max_items are taken.  Returns the taken indices.  (The paper shares one
    encoder between apps, Sec. 2.2 "Component Sharing", and names no batching policy; first-fit is
    the policy chosen here.)"""
    taken, total = [], 0
    for i, r in enumerate(rows):
        if len(taken) >= max_items:
            break
        if not taken or total + r <= row_budget:
            taken.append(i)
            total += r
    return taken


# --------------------------------------------------------------------------
# embedding hand-off
# --------------------------------------------------------------------------
def forward_embeddings(src: np.ndarray, placeholder_index: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """dst[idx[i], :] = src[i, :] as a copy of storage words; index -1 skips the row; every
    other row of dst is left as it was.  Returns the updated copy of dst."""
    out = dst.copy()
    assert src.dtype == dst.dtype
    for i, j in enumerate(np.asarray(placeholder_index).tolist()):
        if j < 0:
            continue
        out[j, :] = src[i, :]
    return out


class ChannelModel:
    """The hand-off channel as a sequential program: a pool of equally sized slots, each FREE,
    WRITING or READY (Sec. 2.2 "Data Forwarding": a producer puts its tensor in a shared
    buffer, tells the consumer where it is, the consumer places it).  Every call happens at once
    and in call order; whatever overlap an implementation allows must give these results.
    Calls return a status word: "ok", "busy" (no free slot), "workspace" (tensor larger than a
    slot, or empty), "shape" (more rows published than reserved), "invalid" (slot in the wrong
    state or no such slot)."""

    FREE, WRITING, READY = 0, 1, 2

    def __init__(self, n_slots: int, slot_bytes: int):
        self.slot_bytes = slot_bytes
        self.state = [self.FREE] * n_slots
        self.reserved = [0] * n_slots
        self.rows = [None] * n_slots

    def acquire(self, nbytes: int):
        """-> (status, slot): the lowest-numbered free slot."""
        if nbytes <= 0 or nbytes > self.slot_bytes:
            return "workspace", -1
        for i, st in enumerate(self.state):
            if st == self.FREE:
                self.state[i], self.reserved[i] = self.WRITING, nbytes
                return "ok", i
        return "busy", -1

    def publish(self, slot: int, rows: np.ndarray) -> str:
        if not 0 <= slot < len(self.state) or self.state[slot] != self.WRITING:
            return "invalid"
        if rows.nbytes > self.reserved[slot]:
            return "shape"
        self.rows[slot], self.state[slot] = rows.copy(), self.READY
        return "ok"

    def forward(self, slot: int, placeholder_index: np.ndarray, dst: np.ndarray):
        """-> (status, dst after the placement)."""
        if not 0 <= slot < len(self.state) or self.state[slot] != self.READY:
            return "invalid", dst
        out = forward_embeddings(self.rows[slot], placeholder_index, dst) if len(self.rows[slot]) else dst.copy()
        self.state[slot], self.rows[slot] = self.FREE, None
        return "ok", out

    def release(self, slot: int) -> str:
        if not 0 <= slot < len(self.state) or self.state[slot] == self.FREE:
            return "invalid"
        self.state[slot], self.rows[slot] = self.FREE, None
        return "ok"
