"""Seeded synthetic inputs shaped like the paper's latency workloads.

This module only *makes data*: random draws, storage-format conversion
(float32 <-> bfloat16 bit patterns) and the paged memory layout.  It holds
none of the method's arithmetic (no locality score, no page bounds, no
scoring, no attention), so the CPU oracle and the HIP path can both be fed
from it without sharing any computation.

The paper measures latency on Trado-8B-Instruct activations over TriviaQA
(Latency Analysis section); neither the weights nor the dataset are
available here, so these generators stand in for them with the shapes of
the five benchmark configurations (block size, head counts, prefix length,
page size, active fraction, page budget).

Logical data handed to the oracle:  K[b], V[b] : [L_b, Hkv, d]  (the paper's
K_p, V_p per head), h[t] : [batch*B, H], q[t] : [batch*B, Hq, d].
Physical data handed to the HIP path: the same values scattered into pages,
see `pack_pages`.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

BF16_NAN_BITS = 0x7FC0


# --------------------------------------------------------------------------
# storage format helpers
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32, exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> storage array of the workload's element type."""
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def load(x: np.ndarray) -> np.ndarray:
    """storage array -> float32 values (uint16 is read as bfloat16 bits)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x)
    return np.asarray(x, dtype=np.float32)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    Hq: int            # query heads
    Hkv: int           # KV heads
    d: int             # head dim
    g: int             # page size (tokens)
    B: int             # block size (query tokens per denoising step)
    T: int             # denoising steps per block (step 0 is the dense initialisation)
    n_active: int      # |A| per sequence and step
    topk_pages: int    # K = k / g pages per (active token, query head)
    seq_lens: Tuple[int, ...]   # prefix length L_b of every sequence
    outliers: str      # "fixed4x8" or "lognormal"
    seed: int
    dtype: str = "bf16"

    @property
    def H(self) -> int:          # hidden size of the tensor the detector compares
        return self.Hq * self.d

    @property
    def G(self) -> int:          # GQA group size
        return self.Hq // self.Hkv

    @property
    def pages_per_seq(self) -> Tuple[int, ...]:
        return tuple((L + self.g - 1) // self.g for L in self.seq_lens)

    @property
    def max_pages(self) -> int:
        return max(self.pages_per_seq)

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def active_count(fraction: float, B: int) -> int:
    """Number of active tokens for an 'active fraction' f of a block of B tokens."""
    return max(1, int(np.floor(fraction * B + 0.5)))


def _c2_seq_lens(seed: int, batch: int = 16) -> Tuple[int, ...]:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 77])))
    return tuple(int(v) for v in rng.integers(8192, 32768 + 1, size=batch))


def config(idx: int, *, active_fraction: Optional[float] = None,
           budget_tokens: Optional[int] = None, dtype: str = "bf16") -> Workload:
    """The five benchmark configurations (C0..C4).  C4 is a sweep: pass
    active_fraction in {0.05, 0.10, 0.25, 0.50, 1.00} and budget_tokens in
    {1024, 2048, 4096}."""
    if idx == 0:
        w = Workload("C0-tiny", 1, 4, 1, 64, 16, 32, 8, active_count(0.25, 32), 512 // 16,
                     (2048,), "fixed4x8", 1000)
    elif idx == 1:
        w = Workload("C1-qwen2.5-7b-32k", 1, 28, 4, 128, 16, 32, 16, active_count(0.20, 32),
                     2048 // 16, (32768,), "lognormal", 1001)
    elif idx == 2:
        w = Workload("C2-batched-ragged", 16, 28, 4, 128, 16, 32, 8, active_count(0.15, 32),
                     1024 // 16, _c2_seq_lens(1002), "lognormal", 1002)
    elif idx == 3:
        w = Workload("C3-long-128k", 1, 28, 4, 128, 16, 32, 16, active_count(0.10, 32),
                     4096 // 16, (131072,), "lognormal", 1003)
    elif idx == 4:
        f = 0.10 if active_fraction is None else active_fraction
        k = 2048 if budget_tokens is None else budget_tokens
        w = Workload("C4-llama3-8b-64k", 4, 32, 8, 128, 32, 64, 8, active_count(f, 64),
                     k // 32, (65536,) * 4, "lognormal", 1004)
    else:
        raise ValueError(idx)
    return w.replace(dtype=dtype)


# --------------------------------------------------------------------------
# generated inputs
# --------------------------------------------------------------------------
@dataclass
class Inputs:
    w: Workload
    K: List[np.ndarray]          # per sequence [L_b, Hkv, d]   storage dtype
    V: List[np.ndarray]          # per sequence [L_b, Hkv, d]
    h: np.ndarray                # [T, batch*B, H]
    q: np.ndarray                # [T, batch*B, Hq, d]
    picked: np.ndarray           # [T, batch, n_active] tokens perturbed going into step t (row 0 unused)
    seq_lens: np.ndarray         # int32 [batch]
    page_indptr: np.ndarray      # int32 [batch+1]
    page_indices: np.ndarray     # int32 [sum P_b]  logical page -> physical page id
    num_pages: int


def _rng(seed: int, *tag: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *tag])))


def channel_scales(w: Workload, which: int, heads: int) -> np.ndarray:
    """Per-(head, channel) multipliers.  which: 0=K, 1=V, 2=Q."""
    if w.outliers == "fixed4x8":
        ch = _rng(w.seed, 10).permutation(w.d)[:4]      # same 4 channels for K, V and Q
        s = np.ones((heads, w.d), dtype=np.float32)
        s[:, ch] = 8.0
        return s
    if w.outliers == "lognormal":
        return _rng(w.seed, 11, which).lognormal(0.0, 1.0, size=(heads, w.d)).astype(np.float32)
    raise ValueError(w.outliers)


def make_kv(w: Workload) -> Tuple[List[np.ndarray], List[np.ndarray]]:
    sK = channel_scales(w, 0, w.Hkv)
    sV = channel_scales(w, 1, w.Hkv)
    K, V = [], []
    for b, L in enumerate(w.seq_lens):
        rk = _rng(w.seed, 20, b)
        rv = _rng(w.seed, 21, b)
        K.append(store(rk.standard_normal((L, w.Hkv, w.d), dtype=np.float32) * sK[None], w.dtype))
        V.append(store(rv.standard_normal((L, w.Hkv, w.d), dtype=np.float32) * sV[None], w.dtype))
    return K, V


def make_block_states(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Hidden states h_t, queries q_t and the perturbed-token lists for t = 0..T-1.

    h_0 ~ N(0,1).  Going into step t >= 1, n_active tokens per sequence
    (uniform without replacement) receive a N(0, 0.5) increment, the others a
    N(0, 1e-3) increment (0.5 and 1e-3 are standard deviations); the running
    state is kept in float32 and each h_t is that state rounded to the
    storage type.  q_t[i, h, c] = h_t[i, h*d + c] * s_Q[h, c], rounded."""
    rows = w.batch * w.B
    sQ = channel_scales(w, 2, w.Hq).reshape(1, w.H)
    r = _rng(w.seed, 30)
    state = r.standard_normal((rows, w.H), dtype=np.float32)
    h = np.empty((w.T, rows, w.H), dtype=np.uint16 if w.dtype == "bf16" else np.float32)
    q = np.empty((w.T, rows, w.Hq, w.d), dtype=h.dtype)
    picked = np.full((w.T, w.batch, w.n_active), -1, dtype=np.int32)
    for t in range(w.T):
        if t > 0:
            sigma = np.full((rows, 1), 1e-3, dtype=np.float32)
            for b in range(w.batch):
                p = np.sort(r.permutation(w.B)[: w.n_active])
                picked[t, b] = p
                sigma[b * w.B + p] = 0.5
            state = state + sigma * r.standard_normal((rows, w.H), dtype=np.float32)
        h[t] = store(state, w.dtype)
        q[t] = store(load(h[t]) * sQ, w.dtype).reshape(rows, w.Hq, w.d)
    return h, q, picked


def make_block_kv(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Keys / values of the block's own tokens per step, [T, batch*B, Hkv, d]: N(0,1) times the
    same per-channel scales as the prefix keys / values, redrawn every step (the block's K_b,
    V_b change at each denoising step)."""
    rows = w.batch * w.B
    sK = channel_scales(w, 0, w.Hkv)
    sV = channel_scales(w, 1, w.Hkv)
    r = _rng(w.seed, 50)
    kb = np.empty((w.T, rows, w.Hkv, w.d), dtype=np.uint16 if w.dtype == "bf16" else np.float32)
    vb = np.empty_like(kb)
    for t in range(w.T):
        kb[t] = store(r.standard_normal((rows, w.Hkv, w.d), dtype=np.float32) * sK[None], w.dtype)
        vb[t] = store(r.standard_normal((rows, w.Hkv, w.d), dtype=np.float32) * sV[None], w.dtype)
    return kb, vb


def make_page_table(w: Workload) -> Tuple[np.ndarray, np.ndarray, int]:
    """Logical -> physical page map: one seeded permutation over all pages of the batch,
    so a sequence's pages are scattered through the pool."""
    counts = np.array(w.pages_per_seq, dtype=np.int64)
    indptr = np.zeros(w.batch + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(counts)
    total = int(indptr[-1])
    indices = _rng(w.seed, 40).permutation(total).astype(np.int32)
    return indptr, indices, total


def make_inputs(w: Workload) -> Inputs:
    K, V = make_kv(w)
    h, q, picked = make_block_states(w)
    indptr, indices, total = make_page_table(w)
    return Inputs(w, K, V, h, q, picked, np.array(w.seq_lens, dtype=np.int32), indptr, indices, total)


def pack_pages(inp: Inputs, poison: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    """Scatter the logical K, V into the paged layout the HIP path reads:

        k_pages [num_pages, Hkv, g, d]   (token-major tile)
        v_pages [num_pages, Hkv, d, g]   (channel-major tile: V transposed inside a page)

    Slots past the end of a sequence in its last page hold NaN (or zeros with
    poison=False); no consumer may let them influence a result."""
    w = inp.w
    kd = inp.K[0].dtype
    fill = (BF16_NAN_BITS if kd == np.uint16 else np.float32(np.nan)) if poison else 0
    k_pages = np.full((inp.num_pages, w.Hkv, w.g, w.d), fill, dtype=kd)
    v_pages = np.full((inp.num_pages, w.Hkv, w.d, w.g), fill, dtype=kd)
    for b, L in enumerate(w.seq_lens):
        P = w.pages_per_seq[b]
        phys = inp.page_indices[inp.page_indptr[b]: inp.page_indptr[b + 1]]
        kb = np.full((P * w.g, w.Hkv, w.d), fill, dtype=kd)
        vb = np.full((P * w.g, w.Hkv, w.d), fill, dtype=kd)
        kb[:L] = inp.K[b]
        vb[:L] = inp.V[b]
        k_pages[phys] = kb.reshape(P, w.g, w.Hkv, w.d).transpose(0, 2, 1, 3)
        v_pages[phys] = vb.reshape(P, w.g, w.Hkv, w.d).transpose(0, 2, 3, 1)
    return k_pages, v_pages
