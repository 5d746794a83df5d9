"""Moves a synthetic workload (synth.Inputs) into device memory in the layout liblosa.so
reads, and builds the matching configuration.  Plumbing for tests, smoke and the
benchmark; no arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding, synth


def to_device(arr: np.ndarray, device) -> torch.Tensor:
    """numpy storage array -> torch tensor on `device` (uint16 arrays become bfloat16)."""
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """torch tensor -> numpy (bfloat16 tensors come back as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def config_of(w: synth.Workload, max_topk_pages: int | None = None) -> binding.losa_config:
    return binding.make_config(
        max_batch=w.batch, num_q_heads=w.Hq, num_kv_heads=w.Hkv, head_dim=w.d, hidden_size=w.H,
        page_size=w.g, block_size=w.B, max_pages_per_seq=w.max_pages,
        max_topk_pages=max(w.topk_pages, max_topk_pages or 1),
        dtype=binding.LOSA_BF16 if w.dtype == "bf16" else binding.LOSA_F32)


class DeviceLayer:
    """One layer's paged KV cache on the device."""

    def __init__(self, inp: synth.Inputs, device="cuda:0", poison: bool = True):
        w = inp.w
        k_pages, v_pages = synth.pack_pages(inp, poison=poison)
        self.k_pages = to_device(k_pages, device)
        self.v_pages = to_device(v_pages, device)
        self.meta = torch.zeros((inp.num_pages, w.Hkv, 2, w.d), dtype=self.k_pages.dtype, device=device)
        self.page_indptr = torch.from_numpy(inp.page_indptr).to(device)
        self.page_indices = torch.from_numpy(inp.page_indices).to(device)
        self.seq_lens = torch.from_numpy(inp.seq_lens).to(device)
        self.kv = binding.PagedKV(self.k_pages, self.v_pages, self.meta, self.page_indptr, self.page_indices,
                                  self.seq_lens, max_seq_pages=w.max_pages)


class DeviceBlock:
    """Per-step hidden states and queries of the block being denoised, plus the cached
    prefix statistics (o_p, lse_p) and the selection outputs."""

    def __init__(self, inp: synth.Inputs, device="cuda:0"):
        w = inp.w
        rows = w.batch * w.B
        self.h = to_device(inp.h, device)            # [T, rows, H]
        self.q = to_device(inp.q, device)            # [T, rows, Hq, d]
        self.o_p = torch.zeros((rows, w.Hq, w.d), dtype=torch.float32, device=device)
        self.lse_p = torch.zeros((rows, w.Hq), dtype=torch.float32, device=device)
        self.delta = torch.zeros(rows, dtype=torch.float32, device=device)
        self.mask = torch.zeros(rows, dtype=torch.uint8, device=device)
        self.active_idx = torch.full((rows,), -1, dtype=torch.int32, device=device)
        self.active_count = torch.zeros(w.batch, dtype=torch.int32, device=device)
        self.cap = w.max_pages
        self.sel_pages = torch.full((w.batch, w.Hkv, self.cap), -1, dtype=torch.int32, device=device)
        self.sel_count = torch.zeros((w.batch, w.Hkv), dtype=torch.int32, device=device)
