"""CPU oracle for the LoSA prefix-attention hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy restatement of what the paper defines, written
from the paper alone.  It shares no code with the HIP library and never
imports it.  Only tests, the smoke check and the benchmark's cpu_baseline
leg may call it; the product path never does.

Notation is the paper's (Preliminaries; Methodology): B block size, L prefix
length, d head dim, g page size, K_p/V_p prefix keys/values, A the active
set, I_i the pages picked for query i, I their union, (o_p, L_p) the prefix
attention output and its log-normaliser.  The paper is written for a single
attention head; the multi-head / grouped-query reading used here is: keys,
values and page bounds belong to a KV head; every query head of an active
token picks its own top pages (the paper's per-query budget); the union is
taken per KV head over the queries of its group; all of those queries then
attend over that shared union (Methodology, "Sparse attention with smaller
union size").

Arithmetic is float64 on inputs widened exactly from their storage type
(the statement of the problem asks for a plain float32 reference; float64
is the same definitions evaluated more exactly, so that the reference's own
rounding stays far below the tolerances it is used to check).  Where a
floating value decides an integer result (which tokens are active, which
pages are picked) the float64 value is first rounded to float32, the
precision that statement gives the reference and in which "equal" scores
are defined; ties go to the smaller index.

Parity pins (tests/test_oracle_pins.py): every function below is pinned to a
closed form, an invariant, a library routine or brute force.  End-to-end
task accuracy (the paper's LongBench / commonsense tables) is *parity
unpinned*: it needs model weights and datasets that are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SEL_TOPK, SEL_FRACTION, SEL_THRESHOLD, SEL_MASS = 0, 1, 2, 3


def widen(x: np.ndarray) -> np.ndarray:
    """Storage -> float64, exactly.  uint16 arrays are bfloat16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


# --------------------------------------------------------------------------
# Locality score and locality pruning  (Motivation, eq. mse_locality; Methodology, Locality Pruning)
# --------------------------------------------------------------------------
def locality_score(x_cur: np.ndarray, x_prev: np.ndarray) -> np.ndarray:
    """Delta in R^B: per token, the mean over all of its features of the squared
    change between two consecutive denoising steps."""
    diff = widen(x_cur) - widen(x_prev)
    return (diff * diff).sum(axis=-1) / diff.shape[-1]


def num_active(mode: int, param: float, B: int) -> int:
    if mode == SEL_TOPK:
        return max(0, min(B, int(param)))
    if mode == SEL_FRACTION:
        return max(1, min(B, int(np.floor(np.float32(param) * np.float32(B) + np.float32(0.5)))))
    raise ValueError(mode)


def active_set(delta: np.ndarray, mode: int, param: float) -> np.ndarray:
    """A: the tokens ranked highest by Delta (top-n), those with Delta > tau, or the shortest
    run of top tokens carrying a fraction tau of the total.  Returned ascending by token index."""
    d32 = np.asarray(delta, dtype=np.float64).astype(np.float32)
    B = d32.shape[0]
    if mode == SEL_THRESHOLD:
        return np.nonzero(d32 > np.float32(param))[0].astype(np.int32)
    order = sorted(range(B), key=lambda i: (-float(d32[i]), i))
    if mode == SEL_MASS:
        # Locality figures (threshold line): tokens in descending score order until their
        # running sum reaches the fraction `param` of the block total; float32 sums in that order.
        total = np.float32(0.0)
        for i in order:
            total = np.float32(total + d32[i])
        n = 0
        if total > 0 and np.float32(param) > 0:
            target = np.float32(np.float32(param) * total)
            run, n = np.float32(0.0), B
            for k, i in enumerate(order):
                run = np.float32(run + d32[i])
                if run >= target:
                    n = k + 1
                    break
        return np.array(sorted(order[:n]), dtype=np.int32)
    n = num_active(mode, param, B)
    return np.array(sorted(order[:n]), dtype=np.int32)


# --------------------------------------------------------------------------
# QUEST page selector  (Preliminaries, Sparse Attention Algorithms for LLMs)
# --------------------------------------------------------------------------
def page_min_max(K_p: np.ndarray, g: int) -> Tuple[np.ndarray, np.ndarray]:
    """K_p [L, ...] -> elementwise min and max key of every page of g tokens
    ([P, ...] each); the last page covers only the tokens that exist."""
    Kf = widen(K_p)
    L = Kf.shape[0]
    P = (L + g - 1) // g
    kmin = np.empty((P,) + Kf.shape[1:], dtype=np.float64)
    kmax = np.empty_like(kmin)
    for p in range(P):
        page = Kf[p * g: min(L, (p + 1) * g)]
        kmin[p] = page.min(axis=0)
        kmax[p] = page.max(axis=0)
    return kmin, kmax


def page_upper_bound(q: np.ndarray, kmin: np.ndarray, kmax: np.ndarray) -> np.ndarray:
    """Query-dependent upper bound on q.k over each page: per channel the larger
    of q_c*min_c and q_c*max_c, summed over channels.  q [d]; kmin,kmax [P, d] -> [P]."""
    return np.maximum(q[None, :] * kmin, q[None, :] * kmax).sum(axis=-1)


def top_pages(score: np.ndarray, K: int) -> np.ndarray:
    """The min(K, P) pages with the largest bound (float32 decision, ties to the
    smaller page index), ascending by page index."""
    s32 = np.asarray(score, dtype=np.float64).astype(np.float32)
    P = s32.shape[0]
    order = np.lexsort((np.arange(P), -s32.astype(np.float64)))
    return np.sort(order[: min(K, P)]).astype(np.int32)


def shared_top_pages(scores: np.ndarray, K: int) -> np.ndarray:
    """NOT in the paper: the other reading of "a page budget per KV head".  One page set per
    (sequence, KV head) for all of its active queries: every page is scored by the largest
    bound any of those queries gives it (scores [M, P], float32 values), and the min(K, P)
    best pages are kept - exactly min(K, P) pages are then read, where the per-query budget
    of the paper reads between K and M*K.  Ties to the smaller page, ascending output."""
    s32 = np.asarray(scores, dtype=np.float64).astype(np.float32)
    if s32.shape[0] == 0:
        return np.zeros(0, dtype=np.int32)
    return top_pages(s32.max(axis=0), K)


def union_pages(sets: Sequence[np.ndarray]) -> np.ndarray:
    """I = union of the I_i, ascending."""
    if len(sets) == 0:
        return np.zeros(0, dtype=np.int32)
    return np.unique(np.concatenate(list(sets))).astype(np.int32)


# --------------------------------------------------------------------------
# Prefix attention with its log-normaliser  (Preliminaries, Attention Decomposition With Online Softmax)
# --------------------------------------------------------------------------
def prefix_attention(Q: np.ndarray, K_sel: np.ndarray, V_sel: np.ndarray, scale: float
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Q [M, d], K_sel/V_sel [N, d] (float64) -> o_p [M, d], L_p [M].
    s = scale * Q K^T ; L_p = log sum exp(s) ; o_p = exp(s - L_p) V."""
    s = scale * (Q @ K_sel.T)
    m = s.max(axis=-1, keepdims=True)
    w = np.exp(s - m)
    l = w.sum(axis=-1, keepdims=True)
    return (w @ V_sel) / l, (m + np.log(l))[:, 0]


def merge_partials(o1: np.ndarray, L1: np.ndarray, o2: np.ndarray, L2: np.ndarray
                   ) -> Tuple[np.ndarray, np.ndarray]:
    """Online-softmax merge of two (output, log-normaliser) pairs over disjoint key sets."""
    Lm = np.maximum(L1, L2)
    w1, w2 = np.exp(L1 - Lm), np.exp(L2 - Lm)
    return (o1 * w1[:, None] + o2 * w2[:, None]) / (w1 + w2)[:, None], Lm + np.log(w1 + w2)


def tokens_of_pages(pages: np.ndarray, g: int, L: int) -> np.ndarray:
    """Prefix positions covered by a list of pages (the last page may be partial)."""
    if len(pages) == 0:
        return np.zeros(0, dtype=np.int64)
    t = (np.asarray(pages, dtype=np.int64)[:, None] * g + np.arange(g)[None, :]).reshape(-1)
    return t[t < L]


# --------------------------------------------------------------------------
# One denoising step of one layer  (Methodology; Fig. MethodOverview steps i-iii)
# --------------------------------------------------------------------------
@dataclass
class StepTrace:
    """Everything a step decided, for stage-by-stage comparison."""
    delta: Optional[np.ndarray] = None                    # [batch*B] float64
    active: List[np.ndarray] = field(default_factory=list)            # per sequence, ascending token ids
    scores: Dict[Tuple[int, int, int], np.ndarray] = field(default_factory=dict)   # (b, token, head) -> [P_b] float64
    picks: Dict[Tuple[int, int, int], np.ndarray] = field(default_factory=dict)    # (b, token, head) -> pages
    union: Dict[Tuple[int, int], np.ndarray] = field(default_factory=dict)         # (b, kv head) -> pages


class PrefixCache:
    """Per-sequence prefix keys/values widened once, with their page bounds."""

    def __init__(self, K: Sequence[np.ndarray], V: Sequence[np.ndarray], g: int):
        self.g = g
        self.K = [widen(k) for k in K]         # [L_b, Hkv, d]
        self.V = [widen(v) for v in V]
        self.L = [k.shape[0] for k in self.K]
        self.bounds = [page_min_max(k, g) for k in self.K]      # ([P_b, Hkv, d], [P_b, Hkv, d])

    def num_pages(self, b: int) -> int:
        return (self.L[b] + self.g - 1) // self.g


def losa_step(cache: PrefixCache, step_index: int,
              x_cur: Optional[np.ndarray], x_prev: Optional[np.ndarray], q: np.ndarray,
              mode: int, param: float, topk_pages: int, B: int, Hq: int,
              o_p: np.ndarray, L_p: np.ndarray, scale: Optional[float] = None,
              forced_active: Optional[List[np.ndarray]] = None,
              forced_union: Optional[Dict[Tuple[int, int], np.ndarray]] = None,
              keep_scores: bool = False) -> StepTrace:
    """Updates o_p [batch*B, Hq, d] and L_p [batch*B, Hq] (float64) in place.

    step_index 0 is the dense initialisation: every token is active and every
    page is used.  Otherwise: Delta -> A -> per-query top pages -> union per KV
    head -> attention of the active queries over the union; rows of stable
    tokens are left exactly as they were (the reuse rule).
    forced_active / forced_union replace the corresponding decisions (used to
    compare one stage at a time)."""
    batch = len(cache.K)
    Hkv, d = cache.K[0].shape[1], cache.K[0].shape[2]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    qf = widen(q)
    tr = StepTrace()
    dense = step_index == 0
    if not dense and forced_active is None:
        tr.delta = locality_score(x_cur, x_prev)
    for b in range(batch):
        P = cache.num_pages(b)
        if dense:
            A = np.arange(B, dtype=np.int32)
        elif forced_active is not None:
            A = np.asarray(forced_active[b], dtype=np.int32)
        else:
            A = active_set(tr.delta[b * B:(b + 1) * B], mode, param)
        tr.active.append(A)
        kmin, kmax = cache.bounds[b]
        for j in range(Hkv):
            heads = range(j * G, (j + 1) * G)
            if dense:
                I = np.arange(P, dtype=np.int32)
            elif forced_union is not None:
                I = np.asarray(forced_union[(b, j)], dtype=np.int32)
            else:
                picks = []
                for i in A:
                    for h in heads:
                        s = page_upper_bound(qf[b * B + i, h], kmin[:, j], kmax[:, j])
                        I_ih = top_pages(s, topk_pages)
                        if keep_scores:
                            tr.scores[(b, int(i), h)] = s
                        tr.picks[(b, int(i), h)] = I_ih
                        picks.append(I_ih)
                I = union_pages(picks)
            tr.union[(b, j)] = I
            if len(A) == 0:
                continue
            tok = tokens_of_pages(I, cache.g, cache.L[b])
            if len(tok) == 0:
                # attention over an empty key set: the neutral element of the online-softmax merge
                for h in heads:
                    o_p[b * B + A, h] = 0.0
                    L_p[b * B + A, h] = -np.inf
                continue
            K_sel, V_sel = cache.K[b][tok, j], cache.V[b][tok, j]
            for h in heads:
                o, lse = prefix_attention(qf[b * B + A, h], K_sel, V_sel, scale)
                o_p[b * B + A, h] = o
                L_p[b * B + A, h] = lse
    return tr


def block_attention_and_merge(q: np.ndarray, k_b: np.ndarray, v_b: np.ndarray, o_p: np.ndarray, L_p: np.ndarray,
                              B: int, scale: Optional[float] = None
                              ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Dense attention inside the block and the final merge with the prefix statistics
    (Methodology, Computation of the Suffix Tokens and Final Output).
    q [batch*B, Hq, d], k_b / v_b [batch*B, Hkv, d] (storage types), o_p [batch*B, Hq, d],
    L_p [batch*B, Hq] (float64).  Returns (O, o_b, L_b)."""
    qf, kf, vf = widen(q), widen(k_b), widen(v_b)
    rows, Hq, d = qf.shape
    Hkv = kf.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    O = np.empty_like(qf)
    o_b = np.empty_like(qf)
    L_b = np.empty((rows, Hq))
    for b in range(rows // B):
        sl = slice(b * B, (b + 1) * B)
        for h in range(Hq):
            ob, Lb = prefix_attention(qf[sl, h], kf[sl, h // G], vf[sl, h // G], scale)
            o_b[sl, h], L_b[sl, h] = ob, Lb
            O[sl, h], _ = merge_partials(np.asarray(o_p[sl, h], dtype=np.float64), np.asarray(L_p[sl, h], dtype=np.float64), ob, Lb)
    return O, o_b, L_b


def dense_block_attention(Q_b: np.ndarray, K_all: np.ndarray, V_all: np.ndarray) -> np.ndarray:
    """Full attention of one head, O = softmax(Q_b [K_p,K_b]^T / sqrt(d)) [V_p,V_b]
    (Preliminaries, eq. full_attn), as a direct row-by-row softmax."""
    d = Q_b.shape[-1]
    out = np.empty((Q_b.shape[0], V_all.shape[-1]), dtype=np.float64)
    for i in range(Q_b.shape[0]):
        s = (K_all @ Q_b[i]) / np.sqrt(d)
        e = np.exp(s - s.max())
        out[i] = (e / e.sum()) @ V_all
    return out
