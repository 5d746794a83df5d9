"""ctypes binding of liblosa.so: the same entry points as include/losa.h, taking torch
tensors.  Argument marshalling only: every step of the path runs in the HIP kernels.
torch is used for device memory and the current stream, nothing else.

The library must have been built (python -m paper_2604_12056_amd.build, or
__graft_entry__.build()); there is no fallback path if it is missing."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

from .build import LIB_PATH

LOSA_OK, LOSA_ERR_INVALID_ARG, LOSA_ERR_UNSUPPORTED, LOSA_ERR_WORKSPACE, LOSA_ERR_HIP = range(5)
LOSA_BF16, LOSA_F32 = 0, 1
LOSA_SEL_TOPK, LOSA_SEL_FRACTION, LOSA_SEL_THRESHOLD, LOSA_SEL_MASS = 0, 1, 2, 3

EXPORTS = ["losa_workspace_bytes", "losa_create", "losa_destroy", "losa_last_error", "losa_select_active",
           "losa_page_bounds", "losa_score_pages", "losa_sparse_attn", "losa_step", "losa_profile_enable",
           "losa_profile_read", "losa_calibration_copy", "losa_block_merge", "losa_score_pages_shared",
           "losa_select_active_static", "losa_set_tuning", "losa_calibration_read"]
(LOSA_TUNE_ATTN_WORKGROUPS, LOSA_TUNE_SELECT_ROUND, LOSA_TUNE_SCORE_ROUND, LOSA_TUNE_RANK_IN_SCORES,
 LOSA_TUNE_UNION_IN_ATTENTION, LOSA_TUNE_SHARED_TILES, LOSA_TUNE_HALF_PRECISION_VALUES) = range(7)
STAGES = ["locality", "score", "topk", "attn", "merge", "bounds", "block"]


class LosaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"losa status {status}: {text}")
        self.status = status
        self.text = text


class losa_config(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("hidden_size", C.c_int32), ("page_size", C.c_int32),
                ("block_size", C.c_int32), ("max_pages_per_seq", C.c_int32), ("max_topk_pages", C.c_int32),
                ("dtype", C.c_int32), ("sm_scale", C.c_float)]


class losa_kv(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("meta", C.c_void_p),
                ("page_indptr", C.c_void_p), ("page_indices", C.c_void_p), ("seq_lens", C.c_void_p),
                ("batch", C.c_int32), ("num_pages", C.c_int32), ("max_seq_pages", C.c_int32)]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree liblosa.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_12056_amd.build`")
    lib = C.CDLL(LIB_PATH)
    p, i32, f32, vp = C.c_void_p, C.c_int32, C.c_float, C.c_void_p
    lib.losa_workspace_bytes.restype = C.c_size_t
    lib.losa_workspace_bytes.argtypes = [C.POINTER(losa_config)]
    lib.losa_create.restype = C.c_int
    lib.losa_create.argtypes = [C.POINTER(losa_config), vp, C.c_size_t, C.POINTER(vp)]
    lib.losa_destroy.restype = C.c_int
    lib.losa_destroy.argtypes = [vp]
    lib.losa_last_error.restype = C.c_char_p
    lib.losa_last_error.argtypes = [vp]
    lib.losa_select_active.restype = C.c_int
    lib.losa_select_active.argtypes = [vp, vp, i32, p, p, C.c_int, f32, p, p, p, p]
    lib.losa_select_active_static.restype = C.c_int
    lib.losa_select_active_static.argtypes = [vp, i32, i32, i32, i32, p, p, C.c_int, f32, p, p, p, p]
    lib.losa_page_bounds.restype = C.c_int
    lib.losa_page_bounds.argtypes = [vp, vp, C.POINTER(losa_kv), i32, i32]
    lib.losa_score_pages.restype = C.c_int
    lib.losa_score_pages.argtypes = [vp, vp, C.POINTER(losa_kv), p, p, p, i32, p, p, p, i32]
    lib.losa_score_pages_shared.restype = C.c_int
    lib.losa_score_pages_shared.argtypes = [vp, vp, C.POINTER(losa_kv), p, p, p, i32, p, p, i32]
    lib.losa_sparse_attn.restype = C.c_int
    lib.losa_sparse_attn.argtypes = [vp, vp, C.POINTER(losa_kv), p, p, p, p, p, i32, p, p]
    lib.losa_step.restype = C.c_int
    lib.losa_step.argtypes = [vp, vp, C.POINTER(losa_kv), i32, p, p, p, C.c_int, f32, i32, p, p, p, p]
    lib.losa_set_tuning.restype = C.c_int
    lib.losa_set_tuning.argtypes = [vp, C.c_int, C.c_int64]
    lib.losa_profile_enable.restype = C.c_int
    lib.losa_profile_enable.argtypes = [vp, i32]
    lib.losa_profile_read.restype = C.c_int
    lib.losa_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.losa_block_merge.restype = C.c_int
    lib.losa_block_merge.argtypes = [vp, vp, i32, p, p, p, p, p, p, p, p]
    lib.losa_calibration_copy.restype = C.c_int
    lib.losa_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.losa_calibration_read.restype = C.c_int
    lib.losa_calibration_read.argtypes = [vp, C.c_size_t, vp, i32, vp, vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return int(stream) or None
    import torch
    return torch.cuda.current_stream().cuda_stream or None


class PagedKV:
    """Device tensors of one layer's paged prefix cache plus the host-side counts."""

    def __init__(self, k_pages, v_pages, meta, page_indptr, page_indices, seq_lens, max_seq_pages: int = 0):
        self.k_pages, self.v_pages, self.meta = k_pages, v_pages, meta
        self.page_indptr, self.page_indices, self.seq_lens = page_indptr, page_indices, seq_lens
        self.batch = int(seq_lens.numel())
        self.num_pages = int(k_pages.shape[0])
        self.max_seq_pages = int(max_seq_pages)

    def as_struct(self) -> losa_kv:
        return losa_kv(_ptr(self.k_pages), _ptr(self.v_pages), _ptr(self.meta), _ptr(self.page_indptr),
                       _ptr(self.page_indices), _ptr(self.seq_lens), self.batch, self.num_pages, self.max_seq_pages)


class Context:
    """Owns the losa_ctx handle and the torch tensor that backs its workspace."""

    def __init__(self, handle: int, workspace, cfg: losa_config):
        self.handle, self.workspace, self.cfg = handle, workspace, cfg

    def close(self):
        if self.handle:
            load_library().losa_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _check(ctx: Optional[Context], status: int):
    if status != LOSA_OK:
        text = load_library().losa_last_error(ctx.handle if ctx else None)
        raise LosaError(status, text.decode() if text else "")


def make_config(*, max_batch, num_q_heads, num_kv_heads, head_dim, hidden_size, page_size, block_size,
                max_pages_per_seq, max_topk_pages, dtype=LOSA_BF16, sm_scale=0.0) -> losa_config:
    return losa_config(max_batch, num_q_heads, num_kv_heads, head_dim, hidden_size, page_size, block_size,
                       max_pages_per_seq, max_topk_pages, dtype, sm_scale)


def losa_workspace_bytes(cfg: losa_config) -> int:
    return int(load_library().losa_workspace_bytes(C.byref(cfg)))


def losa_create(cfg: losa_config, device="cuda:0") -> Context:
    """Allocates the workspace with torch on `device` and creates the context."""
    import torch
    lib = load_library()
    nbytes = lib.losa_workspace_bytes(C.byref(cfg))
    if nbytes == 0:
        # let the library say what is wrong with the configuration
        out = C.c_void_p()
        _check(None, lib.losa_create(C.byref(cfg), None, 0, C.byref(out)))
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    out = C.c_void_p()
    _check(None, lib.losa_create(C.byref(cfg), ws.data_ptr() + off, nbytes, C.byref(out)))
    return Context(out.value, ws, cfg)


def losa_destroy(ctx: Context):
    ctx.close()


def losa_select_active(ctx: Context, h_cur, h_prev, mode: int, param: float, delta, mask, active_idx, active_count,
                       batch: Optional[int] = None, stream=None):
    batch = int(active_count.numel()) if batch is None else batch
    _check(ctx, load_library().losa_select_active(ctx.handle, _stream(stream), batch, _ptr(h_cur), _ptr(h_prev),
                                                 mode, param, _ptr(delta), _ptr(mask), _ptr(active_idx),
                                                 _ptr(active_count)))


def losa_select_active_static(dtype: int, batch: int, block_size: int, hidden_size: int, h_cur, h_prev, mode: int,
                              param: float, delta, mask, active_idx, active_count, stream=None):
    """The allocation-free variant: no context, no workspace (ticket counters live in the library)."""
    _check(None, load_library().losa_select_active_static(_stream(stream), dtype, batch, block_size, hidden_size,
                                                         _ptr(h_cur), _ptr(h_prev), mode, param, _ptr(delta),
                                                         _ptr(mask), _ptr(active_idx), _ptr(active_count)))


def losa_page_bounds(ctx: Context, kv: PagedKV, first_logical_page: int = 0, num_logical_pages: int = -1, stream=None):
    s = kv.as_struct()
    _check(ctx, load_library().losa_page_bounds(ctx.handle, _stream(stream), C.byref(s), first_logical_page,
                                               num_logical_pages))


def losa_score_pages(ctx: Context, kv: PagedKV, q, active_idx, active_count, topk_pages: int, topk_out, sel_pages,
                     sel_count, cap: int, stream=None):
    s = kv.as_struct()
    _check(ctx, load_library().losa_score_pages(ctx.handle, _stream(stream), C.byref(s), _ptr(q), _ptr(active_idx),
                                               _ptr(active_count), topk_pages, _ptr(topk_out), _ptr(sel_pages),
                                               _ptr(sel_count), cap))


def losa_score_pages_shared(ctx: Context, kv: PagedKV, q, active_idx, active_count, topk_pages: int, sel_pages,
                            sel_count, cap: int, stream=None):
    s = kv.as_struct()
    _check(ctx, load_library().losa_score_pages_shared(ctx.handle, _stream(stream), C.byref(s), _ptr(q),
                                                      _ptr(active_idx), _ptr(active_count), topk_pages,
                                                      _ptr(sel_pages), _ptr(sel_count), cap))


def losa_sparse_attn(ctx: Context, kv: PagedKV, q, active_idx, active_count, sel_pages, sel_count, cap: int, o_p,
                     lse_p, stream=None):
    s = kv.as_struct()
    _check(ctx, load_library().losa_sparse_attn(ctx.handle, _stream(stream), C.byref(s), _ptr(q), _ptr(active_idx),
                                               _ptr(active_count), _ptr(sel_pages), _ptr(sel_count), cap, _ptr(o_p),
                                               _ptr(lse_p)))


def losa_step(ctx: Context, kv: PagedKV, step_index: int, h_cur, h_prev, q, mode: int, param: float,
              topk_pages: int, o_p, lse_p, mask=None, sel_count=None, stream=None):
    s = kv.as_struct()
    _check(ctx, load_library().losa_step(ctx.handle, _stream(stream), C.byref(s), step_index, _ptr(h_cur),
                                        _ptr(h_prev), _ptr(q), mode, param, topk_pages, _ptr(o_p), _ptr(lse_p),
                                        _ptr(mask), _ptr(sel_count)))


def losa_set_tuning(ctx: Context, knob: int, value: int):
    _check(ctx, load_library().losa_set_tuning(ctx.handle, knob, int(value)))


def losa_profile_enable(ctx: Context, enable: bool):
    _check(ctx, load_library().losa_profile_enable(ctx.handle, 1 if enable else 0))


def losa_profile_read(ctx: Context):
    """-> ({stage: milliseconds}, {stage: launches}) since the last read."""
    ms = (C.c_double * len(STAGES))()
    cnt = (C.c_int64 * len(STAGES))()
    _check(ctx, load_library().losa_profile_read(ctx.handle, ms, cnt))
    return dict(zip(STAGES, list(ms))), dict(zip(STAGES, list(cnt)))


def losa_calibration_copy(dst, src, stream=None):
    """Plain copy of src into dst (same byte size): the known-size reference for byte counters."""
    nbytes = src.numel() * src.element_size()
    _check(None, load_library().losa_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def losa_calibration_read(pool, tile_bytes: int, tile_ids, sink, stream=None):
    """Read-only stream over the tiles of `pool` listed in tile_ids (int32 tensor); nothing is written."""
    _check(None, load_library().losa_calibration_read(_ptr(pool), tile_bytes, _ptr(tile_ids), int(tile_ids.numel()),
                                                     _ptr(sink), _stream(stream)))


def losa_block_merge(ctx: Context, q, k_b, v_b, o_p, lse_p, out, o_b=None, lse_b=None, batch: Optional[int] = None,
                     stream=None):
    batch = int(lse_p.shape[0] // ctx.cfg.block_size) if batch is None else batch
    _check(ctx, load_library().losa_block_merge(ctx.handle, _stream(stream), batch, _ptr(q), _ptr(k_b), _ptr(v_b),
                                               _ptr(o_p), _ptr(lse_p), _ptr(out), _ptr(o_b), _ptr(lse_b)))
