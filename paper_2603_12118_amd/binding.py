"""ctypes binding of libcornenc.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/cornenc.h).  PyTorch
tensors are used as device memory and for the current HIP stream; no step of the encoder runs
in Python.  Importing this module needs the built library; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcornenc.so")

CS_F32, CS_BF16 = 0, 1
CS_ARCH_VIT, CS_ARCH_AUDIO, CS_ARCH_VIT_CLS = 0, 1, 2
CS_ORDER_RASTER, CS_ORDER_MERGE_MAJOR = 0, 1
CS_SLOT_FREE, CS_SLOT_WRITING, CS_SLOT_READY = 0, 1, 2
CS_ERR_INVALID_ARG, CS_ERR_SHAPE, CS_ERR_WORKSPACE, CS_ERR_UNSUPPORTED, CS_ERR_BUSY, CS_ERR_NO_MEMORY, CS_ERR_TIMEOUT = 1, 2, 3, 5, 8, 9, 10
CS_XSLOT_FREE, CS_XSLOT_WRITING, CS_XSLOT_PUBLISHING, CS_XSLOT_READY, CS_XSLOT_DRAINING = 0, 1, 2, 3, 4
STEPS = {"front": 1, "norm": 2, "qkv": 3, "attn_window": 4, "attn_full": 5, "proj": 6, "mlp_up": 7, "mlp_down": 8,
         "back": 9}


class CsError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"cornenc status {status}: {text}")
        self.status = status


class cs_encoder_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("arch", C.c_int32), ("dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("patch_dim", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n_layers", C.c_int32), ("mlp_dim", C.c_int32), ("merge", C.c_int32), ("merger_hidden", C.c_int32),
                ("out_hidden", C.c_int32), ("window", C.c_int32), ("full_attn_layer_mask", C.c_uint64),
                ("rope_sections", C.c_int32 * 3), ("rope_theta", C.c_float), ("norm_eps", C.c_float),
                ("conv_kernel", C.c_int32), ("input_order", C.c_int32), ("attn_chunk", C.c_int32)]


class cs_tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("data", C.c_void_p), ("numel", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run __graft_entry__.build() "
                               "(python -m paper_2603_12118_amd.build)")
        L = C.CDLL(LIB_PATH)
        vp, i32p, i64 = C.c_void_p, C.POINTER(C.c_int32), C.c_int64
        L.cs_encoder_create.argtypes = [C.POINTER(cs_encoder_config), C.POINTER(cs_tensor), C.c_int32, C.POINTER(vp)]
        L.cs_encoder_destroy.argtypes = [vp]
        L.cs_encoder_destroy.restype = None
        L.cs_encoder_query.argtypes = [vp, i32p, i32p, C.c_int32, C.POINTER(i64), C.POINTER(C.c_size_t)]
        L.cs_encode.argtypes = [vp, vp, i32p, i32p, C.c_int32, vp, vp, C.c_size_t, vp]
        L.cs_encode_static.argtypes = [vp, vp, i32p, i32p, C.c_int32, vp, vp]
        L.cs_encode_graph_create.argtypes = [vp, vp, i32p, i32p, C.c_int32, vp, vp, C.c_size_t, vp, C.POINTER(vp)]
        L.cs_encode_graph_launch.argtypes = [vp, vp]
        L.cs_encode_graph_destroy.argtypes = [vp]
        L.cs_encode_graph_destroy.restype = None
        L.cs_encoder_plan_cache_stats.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
        L.cs_forward_embeddings.argtypes = [vp, vp, vp, i64, i64, C.c_int32, C.c_int32, vp, vp]
        L.cs_plan_tokens.argtypes = [C.POINTER(cs_encoder_config), i32p, i32p, C.c_int32, i32p, i32p, i32p, C.c_int32, i32p]
        L.cs_linear_bf16.argtypes = [vp, i64, vp, vp, vp, C.c_int32, i64, C.c_int32, C.c_int32, vp]
        L.cs_attention_varlen.argtypes = [vp, vp, i64, vp, i32p, C.c_int32, C.c_int32, C.c_int32, vp]
        L.cs_pack_batch.argtypes = [i32p, C.c_int32, i64, C.c_int32, i32p, i32p, i32p, i32p]
        L.cs_patchify.argtypes = [vp, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_int32, vp, C.c_int32, i32p, i32p, vp]
        L.cs_channel_create.argtypes = [C.c_int32, C.c_size_t, C.POINTER(vp)]
        L.cs_channel_destroy.argtypes = [vp]
        L.cs_channel_destroy.restype = None
        L.cs_channel_acquire.argtypes = [vp, C.c_size_t, vp, i32p, C.POINTER(vp)]
        L.cs_channel_publish.argtypes = [vp, C.c_int32, i64, C.c_int32, C.c_int32, vp]
        L.cs_channel_forward.argtypes = [vp, C.c_int32, vp, vp, i64, vp, vp]
        L.cs_channel_release.argtypes = [vp, C.c_int32, vp]
        L.cs_channel_describe.argtypes = [vp, C.c_int32, i32p, C.POINTER(vp), C.POINTER(i64), i32p, i32p, i32p]
        L.cs_xchannel_create.argtypes = [C.c_char_p, C.c_int32, C.c_size_t, C.POINTER(vp)]
        L.cs_xchannel_open.argtypes = [C.c_char_p, C.POINTER(vp)]
        L.cs_xchannel_close.argtypes = [vp]
        L.cs_xchannel_close.restype = None
        L.cs_xchannel_acquire.argtypes = [vp, C.c_size_t, i32p, C.POINTER(vp)]
        L.cs_xchannel_publish.argtypes = [vp, C.c_int32, i64, C.c_int32, C.c_int32, vp]
        L.cs_xchannel_wait.argtypes = [vp, i64, i32p, C.POINTER(i64), i32p, i32p]
        L.cs_xchannel_forward.argtypes = [vp, C.c_int32, vp, vp, i64, vp, vp]
        L.cs_xchannel_release.argtypes = [vp, C.c_int32]
        L.cs_xchannel_describe.argtypes = [vp, C.c_int32, i32p, C.POINTER(vp), C.POINTER(i64), i32p, i32p,
                                           C.POINTER(i64), C.POINTER(i64)]
        L.cs_mfma_ceiling.argtypes = [vp, C.c_size_t, C.c_int32, C.c_int32, C.POINTER(C.c_double), vp]
        L.cs_encoder_step_kernel.argtypes = [vp, C.c_int32, i64, C.c_char_p, C.c_size_t]
        L.cs_encoder_time_step.argtypes = [vp, C.c_int32]
        L.cs_encoder_time_every.argtypes = [vp, C.c_int32]
        L.cs_encoder_read_timing.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
        L.cs_status_string.argtypes = [C.c_int]
        L.cs_status_string.restype = C.c_char_p
        L.cs_last_error.restype = C.c_char_p
        for f in ("cs_encoder_create", "cs_encoder_query", "cs_encode", "cs_encode_static", "cs_encoder_plan_cache_stats", "cs_encode_graph_create",
                  "cs_encode_graph_launch",
                  "cs_forward_embeddings", "cs_plan_tokens",
                  "cs_linear_bf16", "cs_attention_varlen", "cs_encoder_time_step", "cs_encoder_step_kernel", "cs_encoder_time_every",
                  "cs_encoder_read_timing", "cs_patchify", "cs_mfma_ceiling", "cs_pack_batch", "cs_channel_create",
                  "cs_channel_acquire", "cs_channel_publish", "cs_channel_forward", "cs_channel_release",
                  "cs_channel_describe", "cs_xchannel_create", "cs_xchannel_open", "cs_xchannel_acquire",
                  "cs_xchannel_publish", "cs_xchannel_wait", "cs_xchannel_forward", "cs_xchannel_release",
                  "cs_xchannel_describe"):
            getattr(L, f).restype = C.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        L = lib()
        raise CsError(status, f"{L.cs_status_string(status).decode()}: {L.cs_last_error().decode()}")


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _i32p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def make_config(cfg) -> cs_encoder_config:
    """workloads.EncoderConfig -> C struct."""
    c = cs_encoder_config()
    c.struct_size = C.sizeof(cs_encoder_config)
    c.arch = {"vit": CS_ARCH_VIT, "audio": CS_ARCH_AUDIO, "vit_cls": CS_ARCH_VIT_CLS}[cfg.arch]
    c.dtype = CS_BF16 if cfg.dtype == "bf16" else CS_F32
    c.out_dtype = CS_BF16 if cfg.out_dtype == "bf16" else CS_F32
    for k in ("patch_dim", "hidden", "n_heads", "head_dim", "n_layers", "mlp_dim", "merge", "merger_hidden",
              "out_hidden", "window", "conv_kernel"):
        setattr(c, k, int(getattr(cfg, k)))
    mask = 0
    for l in cfg.full_attn_layers:
        mask |= 1 << int(l)
    c.full_attn_layer_mask = mask
    c.rope_sections = (C.c_int32 * 3)(*[int(s) for s in cfg.rope_sections])
    c.rope_theta = float(cfg.rope_theta)
    c.norm_eps = float(cfg.norm_eps)
    c.input_order = {"raster": CS_ORDER_RASTER, "merge_major": CS_ORDER_MERGE_MAJOR}[getattr(cfg, "input_order", "raster")]
    c.attn_chunk = int(getattr(cfg, "attn_chunk", 0))
    return c


class Encoder:
    """Owns a cs_encoder handle."""

    def __init__(self, cfg, weights: Dict[str, np.ndarray]):
        self.cfg = cfg
        self._h = C.c_void_p()
        cc = make_config(cfg)
        keep, arr = [], (cs_tensor * len(weights))()
        for i, (name, w) in enumerate(weights.items()):
            w32 = np.ascontiguousarray(w, dtype=np.float32)
            if cfg.dtype == "bf16":      # values are bf16-representable: hand over the 16-bit words
                buf = np.ascontiguousarray((w32.view(np.uint32) >> np.uint32(16)).astype(np.uint16))
            else:
                buf = w32
            keep.append(buf)
            arr[i].name = name.encode()
            arr[i].data = buf.ctypes.data
            arr[i].numel = buf.size
        _check(lib().cs_encoder_create(C.byref(cc), arr, len(weights), C.byref(self._h)))

    def close(self) -> None:
        if self._h:
            lib().cs_encoder_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def cs_encoder_query(self, cu_seqlens, grid_thw):
        cu, g = _i32(cu_seqlens), _i32(grid_thw)
        n_out, ws = C.c_int64(), C.c_size_t()
        _check(lib().cs_encoder_query(self._h, _i32p(cu), _i32p(g), g.shape[0], C.byref(n_out), C.byref(ws)))
        return n_out.value, ws.value

    def cs_encoder_time_step(self, step: int) -> None:
        _check(lib().cs_encoder_time_step(self._h, step))

    def cs_encoder_step_kernel(self, step: int, n_tokens: int) -> str:
        buf = C.create_string_buffer(128)
        _check(lib().cs_encoder_step_kernel(self._h, step, n_tokens, buf, 128))
        return buf.value.decode()

    def cs_encoder_time_every(self, every: int) -> None:
        _check(lib().cs_encoder_time_every(self._h, every))

    def cs_encoder_read_timing(self):
        ms, n = C.c_double(), C.c_int64()
        _check(lib().cs_encoder_read_timing(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def cs_encode(self, patches, cu_seqlens, grid_thw, out=None, workspace=None, stream=None):
        """patches: device tensor [N, patch_dim] of the config dtype.  Returns (out, workspace).
        `out` may also be a device tensor view of a channel slot (Channel.slot_tensor)."""
        import torch
        cu, g = _i32(cu_seqlens), _i32(grid_thw)
        n_out, ws_bytes = self.cs_encoder_query(cu, g)
        if out is None:
            dt = torch.bfloat16 if self.cfg.out_dtype == "bf16" else torch.float32
            out = torch.empty((n_out, self.cfg.out_hidden), dtype=dt, device=patches.device)
        if workspace is None or workspace.numel() < ws_bytes:
            workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=patches.device)
        assert patches.is_contiguous() and out.is_contiguous()
        _check(lib().cs_encode(self._h, patches.data_ptr(), _i32p(cu), _i32p(g), g.shape[0], out.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream(stream)))
        return out, workspace


    def cs_encode_static(self, patches, cu_seqlens, grid_thw, out=None, stream=None):
        """cs_encode with the library's static scratch as workspace (no allocation inside the call when
        `out` is given).  Returns out."""
        import torch
        cu, g = _i32(cu_seqlens), _i32(grid_thw)
        if out is None:
            n_out, _ = self.cs_encoder_query(cu, g)
            dt = torch.bfloat16 if self.cfg.out_dtype == "bf16" else torch.float32
            out = torch.empty((n_out, self.cfg.out_hidden), dtype=dt, device=patches.device)
        assert patches.is_contiguous() and out.is_contiguous()
        _check(lib().cs_encode_static(self._h, patches.data_ptr(), _i32p(cu), _i32p(g), g.shape[0], out.data_ptr(),
                                      _stream(stream)))
        return out

    def cs_encode_graph_create(self, patches, cu_seqlens, grid_thw, out, workspace, stream):
        """-> EncodeGraph replaying cs_encode(patches, ...) into `out` (all buffers stay bound to it)."""
        cu, g = _i32(cu_seqlens), _i32(grid_thw)
        h = C.c_void_p()
        _check(lib().cs_encode_graph_create(self._h, patches.data_ptr(), _i32p(cu), _i32p(g), g.shape[0], out.data_ptr(),
                                            workspace.data_ptr(), workspace.numel(), int(stream.cuda_stream), C.byref(h)))
        return EncodeGraph(h, (patches, out, workspace))

    def cs_encoder_plan_cache_stats(self):
        hits, misses = C.c_int64(), C.c_int64()
        _check(lib().cs_encoder_plan_cache_stats(self._h, C.byref(hits), C.byref(misses)))
        return hits.value, misses.value


class EncodeGraph:
    """Owns a cs_encode_graph handle and keeps the tensors it is bound to alive."""

    def __init__(self, handle, bound):
        self._h, self._bound = handle, bound

    def cs_encode_graph_launch(self, stream=None) -> None:
        _check(lib().cs_encode_graph_launch(self._h, _stream(stream)))

    def close(self) -> None:
        if self._h:
            lib().cs_encode_graph_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cs_plan_tokens(cfg, cu_seqlens, grid_thw):
    """Host-only: (src_row, out_row, win_cu) of the internal token order for a vit batch."""
    cu, g = _i32(cu_seqlens), _i32(grid_thw)
    cc = make_config(cfg)
    n = max(int(cu[-1]), 0) if len(cu) else 0
    n_items = g.shape[0] if g.ndim == 2 else 0
    n_tok = n + 4 * n_items if cfg.arch == "vit_cls" else n          # class token + padding per tile
    src_row, out_row = np.empty(max(n_tok, 1), np.int32), np.empty(max(n_tok // 4, 1), np.int32)
    win_cu, nw = np.empty(n + 2, np.int32), C.c_int32()
    _check(lib().cs_plan_tokens(C.byref(cc), _i32p(cu), _i32p(g), n_items, _i32p(src_row),
                                _i32p(out_row), _i32p(win_cu), n + 2, C.byref(nw)))
    return src_row[:n_tok], out_row[:n_tok // 4], win_cu[:nw.value + 1].copy()


def cs_forward_embeddings(src, placeholder_index, dst_seq, err_flag=None, stream=None) -> None:
    """dst_seq[placeholder_index[i], :] = src[i, :] on the GPU (device tensors)."""
    import torch
    assert src.is_contiguous() and dst_seq.is_contiguous() and placeholder_index.dtype == torch.int64
    assert src.dtype == dst_seq.dtype and src.dim() == 2 and dst_seq.dim() == 2
    if src.dtype == torch.bfloat16:
        dt = CS_BF16
    elif src.dtype == torch.float32:
        dt = CS_F32
    else:
        raise TypeError("rows must be bf16 or fp32")
    _check(lib().cs_forward_embeddings(src.data_ptr(), placeholder_index.data_ptr(), dst_seq.data_ptr(),
                                       src.shape[0], dst_seq.shape[0], src.shape[1], dt,
                                       err_flag.data_ptr() if err_flag is not None else None, _stream(stream)))


class _DevView:
    """Device memory at a raw address as an object torch.as_tensor accepts."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


class Channel:
    """Owns a cs_channel handle; methods carry the names of the C calls and return the status
    where a test wants to see it (`check=False`)."""

    def __init__(self, n_slots: int, slot_bytes: int):
        self._h = C.c_void_p()
        _check(lib().cs_channel_create(n_slots, slot_bytes, C.byref(self._h)))

    def close(self) -> None:
        if self._h:
            lib().cs_channel_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def cs_channel_acquire(self, nbytes: int, producer_stream=None, check: bool = True):
        """-> (status, slot, device address)"""
        slot, ptr = C.c_int32(-1), C.c_void_p()
        st = lib().cs_channel_acquire(self._h, nbytes, _stream(producer_stream), C.byref(slot), C.byref(ptr))
        if check:
            _check(st)
        return st, slot.value, ptr.value

    def slot_tensor(self, ptr: int, rows: int, hidden: int, dtype):
        """A torch view [rows, hidden] of slot memory (no copy, no ownership)."""
        import torch
        nbytes = rows * hidden * torch.empty((), dtype=dtype).element_size()
        raw = torch.as_tensor(_DevView(ptr, nbytes), device="cuda")
        return raw.view(dtype).view(rows, hidden)

    def cs_channel_publish(self, slot: int, n_rows: int, hidden: int, dtype: int, producer_stream=None, check: bool = True) -> int:
        st = lib().cs_channel_publish(self._h, slot, n_rows, hidden, dtype, _stream(producer_stream))
        if check:
            _check(st)
        return st

    def cs_channel_forward(self, slot: int, placeholder_index, dst_seq, err_flag=None, consumer_stream=None,
                           check: bool = True) -> int:
        st = lib().cs_channel_forward(self._h, slot, placeholder_index.data_ptr(), dst_seq.data_ptr(), dst_seq.shape[0],
                                      err_flag.data_ptr() if err_flag is not None else None, _stream(consumer_stream))
        if check:
            _check(st)
        return st

    def cs_channel_release(self, slot: int, stream=None, check: bool = True) -> int:
        st = lib().cs_channel_release(self._h, slot, _stream(stream))
        if check:
            _check(st)
        return st

    def cs_channel_describe(self, slot: int):
        """-> dict(state, ptr, n_rows, hidden, dtype, arrived)"""
        state, ptr, rows = C.c_int32(), C.c_void_p(), C.c_int64()
        hidden, dtype, arrived = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().cs_channel_describe(self._h, slot, C.byref(state), C.byref(ptr), C.byref(rows), C.byref(hidden),
                                         C.byref(dtype), C.byref(arrived)))
        return {"state": state.value, "ptr": ptr.value, "n_rows": rows.value, "hidden": hidden.value,
                "dtype": dtype.value, "arrived": arrived.value}


class XChannel:
    """Owns a cs_xchannel handle (the hand-off between two processes): `create=True` in the producer
    process, `create=False` (open by name) in the consumer process."""

    def __init__(self, name: str, n_slots: int = 0, slot_bytes: int = 0, create: bool = True):
        self._h = C.c_void_p()
        if create:
            _check(lib().cs_xchannel_create(name.encode(), n_slots, slot_bytes, C.byref(self._h)))
        else:
            _check(lib().cs_xchannel_open(name.encode(), C.byref(self._h)))

    def close(self) -> None:
        if self._h:
            lib().cs_xchannel_close(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    slot_tensor = Channel.slot_tensor

    def cs_xchannel_acquire(self, nbytes: int):
        """-> (status, slot, device address)"""
        slot, ptr = C.c_int32(-1), C.c_void_p()
        st = lib().cs_xchannel_acquire(self._h, nbytes, C.byref(slot), C.byref(ptr))
        return st, slot.value, ptr.value

    def cs_xchannel_publish(self, slot: int, n_rows: int, hidden: int, dtype: int, producer_stream=None) -> int:
        return lib().cs_xchannel_publish(self._h, slot, n_rows, hidden, dtype, _stream(producer_stream))

    def cs_xchannel_wait(self, timeout_us: int):
        """-> (status, slot, n_rows, hidden, dtype)"""
        slot, rows, hidden, dtype = C.c_int32(-1), C.c_int64(), C.c_int32(), C.c_int32()
        st = lib().cs_xchannel_wait(self._h, timeout_us, C.byref(slot), C.byref(rows), C.byref(hidden), C.byref(dtype))
        return st, slot.value, rows.value, hidden.value, dtype.value

    def cs_xchannel_forward(self, slot: int, placeholder_index, dst_seq, err_flag=None, consumer_stream=None) -> int:
        return lib().cs_xchannel_forward(self._h, slot, placeholder_index.data_ptr(), dst_seq.data_ptr(), dst_seq.shape[0],
                                         err_flag.data_ptr() if err_flag is not None else None, _stream(consumer_stream))

    def cs_xchannel_release(self, slot: int) -> int:
        return lib().cs_xchannel_release(self._h, slot)

    def cs_xchannel_describe(self, slot: int):
        state, ptr, rows = C.c_int32(), C.c_void_p(), C.c_int64()
        hidden, dtype, t_ready, t_placed = C.c_int32(), C.c_int32(), C.c_int64(), C.c_int64()
        _check(lib().cs_xchannel_describe(self._h, slot, C.byref(state), C.byref(ptr), C.byref(rows), C.byref(hidden),
                                          C.byref(dtype), C.byref(t_ready), C.byref(t_placed)))
        return {"state": state.value, "ptr": ptr.value, "n_rows": rows.value, "hidden": hidden.value,
                "dtype": dtype.value, "t_ready_ns": t_ready.value, "t_placed_ns": t_placed.value}


def cs_forward_embeddings_raw(src_ptr, idx_ptr, dst_ptr, n_rows, dst_rows, hidden, dtype, err_ptr=None, stream=0) -> int:
    """The C call with plain integers, returning the status (for argument-validation tests)."""
    return lib().cs_forward_embeddings(src_ptr, idx_ptr, dst_ptr, n_rows, dst_rows, hidden, dtype, err_ptr, stream)


def cs_linear_bf16(A, W, bias, out, stream=None) -> None:
    import torch
    M, K = A.shape
    N = W.shape[0]
    assert A.dtype == torch.bfloat16 and W.dtype == torch.bfloat16 and W.shape[1] == K
    assert out.shape == (M, N) and out.is_contiguous() and W.is_contiguous() and A.stride(1) == 1
    _check(lib().cs_linear_bf16(A.data_ptr(), A.stride(0), W.data_ptr(), bias.data_ptr() if bias is not None else None,
                                out.data_ptr(), CS_BF16 if out.dtype == torch.bfloat16 else CS_F32, M, N, K,
                                _stream(stream)))


def cs_attention_varlen(qk, vt, out, seg_cu: Sequence[int], n_heads: int, head_dim: int, stream=None) -> None:
    seg = _i32(seg_cu)
    _check(lib().cs_attention_varlen(qk.data_ptr(), vt.data_ptr(), vt.stride(0), out.data_ptr(), _i32p(seg),
                                     len(seg) - 1, n_heads, head_dim, _stream(stream)))


def cs_pack_batch(grid_thw, row_budget: int, max_items: int = 1 << 30):
    """First-fit choice of pending items (oldest first) for the next packed call.
    Returns (selected indices, cu_seqlens, packed grid_thw)."""
    g = np.ascontiguousarray(np.asarray(grid_thw, np.int32).reshape(-1, 3))
    n = g.shape[0]
    sel = np.zeros(max(n, 1), np.int32)
    cu = np.zeros(n + 1, np.int32)
    pg = np.zeros((max(n, 1), 3), np.int32)
    k = C.c_int32(0)
    _check(lib().cs_pack_batch(_i32p(g), n, int(row_budget), int(min(max_items, 1 << 30)), _i32p(sel), C.byref(k),
                               _i32p(cu), _i32p(pg)))
    return sel[:k.value].copy(), cu[:k.value + 1].copy(), pg[:k.value].copy()


def cs_patchify(frames, frame_dims, temporal_patch: int, patch: int = 14, out_dtype=None, stream=None):
    """frames: device tensor holding the items' [F,3,H,W] pixels back to back (fp32 or bf16);
    frame_dims: [n_items,3] = (F,H,W).  Returns (patches device tensor, cu_seqlens, grid_thw)."""
    import torch
    fd = np.ascontiguousarray(np.asarray(frame_dims, np.int32).reshape(-1, 3))
    n = fd.shape[0]
    T = np.where(fd[:, 0] == 1, 1, fd[:, 0] // temporal_patch)
    rows = int((T * (fd[:, 1] // patch) * (fd[:, 2] // patch)).sum())
    out_dtype = out_dtype or torch.bfloat16
    out = torch.empty(rows, 3 * temporal_patch * patch * patch, dtype=out_dtype, device=frames.device)
    grid = np.zeros((n, 3), np.int32)
    cu = np.zeros(n + 1, np.int32)
    dt = {torch.float32: CS_F32, torch.bfloat16: CS_BF16}
    _check(lib().cs_patchify(frames.data_ptr(), dt[frames.dtype], _i32p(fd), n, temporal_patch, patch, out.data_ptr(),
                             dt[out_dtype], _i32p(grid), _i32p(cu), _stream(stream)))
    return out, cu, grid


def cs_mfma_ceiling(random_operands: bool, iters: int = 8000, stream=None) -> float:
    """TFLOP/s of a bare MFMA loop on the current device (see cornenc.h)."""
    import torch
    scratch = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    out = C.c_double(0.0)
    _check(lib().cs_mfma_ceiling(scratch.data_ptr(), scratch.numel() * 4, int(bool(random_operands)), int(iters),
                                 C.byref(out), _stream(stream)))
    return out.value


def last_error() -> str:
    return lib().cs_last_error().decode()
