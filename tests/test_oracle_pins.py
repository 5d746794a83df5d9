"""Pins for the CPU oracle: closed forms, hand-worked values, library routines
(scipy softmax / logsumexp), invariants the paper states, and brute force on
tiny inputs.  None of these re-use the oracle's own formulas."""
import itertools
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import losa_oracle as orc
from paper_2604_12056_amd import synth


def _read_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        rows = [[float(v) for v in r.split()] for r in rest.split(";")]
        out[key] = np.array(rows if len(rows) > 1 else rows[0], dtype=np.float64)
    return out


# ---------------------------------------------------------------- attention
def test_hand_worked_attention_and_merge(golden_dir):
    gold = _read_golden(os.path.join(golden_dir, "hand_worked_attention.txt"))
    q = gold["q"][None, :]
    scale = float(gold["scale"][0])
    o1, L1 = orc.prefix_attention(q, gold["K1"], gold["V1"], scale)
    np.testing.assert_allclose(o1[0], gold["o1"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(L1[0], gold["L1"][0], rtol=0, atol=1e-14)
    o2, L2 = orc.prefix_attention(q, gold["K2"][None, :], gold["V2"][None, :], scale)
    np.testing.assert_allclose(o2[0], gold["o2"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(L2[0], gold["L2"][0], rtol=0, atol=1e-14)
    o12, L12 = orc.merge_partials(o1, L1, o2, L2)
    np.testing.assert_allclose(o12[0], gold["o12"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(L12[0], gold["L12"][0], rtol=0, atol=1e-14)


def test_attention_matches_scipy_softmax_and_logsumexp():
    rng = np.random.default_rng(1)
    Q = rng.standard_normal((5, 16))
    K = rng.standard_normal((37, 16)) * 3
    V = rng.standard_normal((37, 16))
    scale = 0.25
    o, L = orc.prefix_attention(Q, K, V, scale)
    s = scale * np.einsum("md,nd->mn", Q, K)
    np.testing.assert_allclose(o, softmax(s, axis=-1) @ V, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(L, logsumexp(s, axis=-1), rtol=1e-13, atol=1e-13)
    # a transposed operand or a dropped scale changes these
    assert not np.allclose(o, softmax(s / scale, axis=-1) @ V)


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    Q = rng.standard_normal((3, 8))
    K = rng.standard_normal((20, 8))
    # constant V -> output is that constant
    V = np.tile(np.array([[1.5, -2.0, 0.25, 7.0]]), (20, 1))
    o, L = orc.prefix_attention(Q, K, V, 0.3)
    np.testing.assert_allclose(o, V[:3], atol=1e-13)
    # all keys equal -> uniform weights: o = mean(V), L = s + ln N
    K1 = np.tile(K[:1], (20, 1))
    V2 = rng.standard_normal((20, 4))
    o, L = orc.prefix_attention(Q, K1, V2, 0.3)
    np.testing.assert_allclose(o, np.tile(V2.mean(0), (3, 1)), atol=1e-13)
    np.testing.assert_allclose(L, 0.3 * Q @ K[0] + np.log(20), atol=1e-13)
    # log-normaliser bounds: max s <= L <= max s + ln N
    o, L = orc.prefix_attention(Q, K, V2, 0.3)
    smax = (0.3 * Q @ K.T).max(-1)
    assert np.all(L >= smax) and np.all(L <= smax + np.log(20) + 1e-12)
    # adding a constant vector c to every key shifts every score of row m by scale*q_m.c:
    # o unchanged, L shifted by exactly that
    c = rng.standard_normal(8)
    o3, L3 = orc.prefix_attention(Q, K + c, V2, 0.3)
    np.testing.assert_allclose(o3, o, atol=1e-12)
    np.testing.assert_allclose(L3, L + 0.3 * Q @ c, atol=1e-12)
    # huge scores must not overflow
    o4, L4 = orc.prefix_attention(Q * 1e3, K, V2, 1.0)
    assert np.all(np.isfinite(o4)) and np.all(np.isfinite(L4))


def test_merge_over_any_partition_equals_one_shot():
    rng = np.random.default_rng(3)
    Q = rng.standard_normal((4, 8))
    K = rng.standard_normal((50, 8)) * 2
    V = rng.standard_normal((50, 8))
    o_all, L_all = orc.prefix_attention(Q, K, V, 0.35)
    for cut in (1, 17, 49):
        oa, La = orc.prefix_attention(Q, K[:cut], V[:cut], 0.35)
        ob, Lb = orc.prefix_attention(Q, K[cut:], V[cut:], 0.35)
        o, L = orc.merge_partials(oa, La, ob, Lb)
        np.testing.assert_allclose(o, o_all, atol=1e-13)
        np.testing.assert_allclose(L, L_all, atol=1e-13)


def test_prefix_plus_block_merge_equals_full_attention():
    # eq. full_attn: softmax(Q_b [K_p,K_b]^T / sqrt(d)) [V_p,V_b], here via scipy
    rng = np.random.default_rng(4)
    d = 16
    Qb, Kb, Vb = (rng.standard_normal((6, d)) for _ in range(3))
    Kp, Vp = rng.standard_normal((40, d)), rng.standard_normal((40, d))
    full = softmax(Qb @ np.concatenate([Kp, Kb]).T / np.sqrt(d), axis=-1) @ np.concatenate([Vp, Vb])
    op, Lp = orc.prefix_attention(Qb, Kp, Vp, 1 / np.sqrt(d))
    ob, Lb = orc.prefix_attention(Qb, Kb, Vb, 1 / np.sqrt(d))
    o, _ = orc.merge_partials(op, Lp, ob, Lb)
    np.testing.assert_allclose(o, full, atol=1e-13)
    np.testing.assert_allclose(orc.dense_block_attention(Qb, np.concatenate([Kp, Kb]),
                                                         np.concatenate([Vp, Vb])), full, atol=1e-13)


# ---------------------------------------------------------------- locality
def test_locality_score_hand_values():
    x_prev = np.array([[1, 2], [3, 4], [5, 6]], dtype=np.float32)
    x_cur = np.array([[1, 4], [0, 4], [5, 6]], dtype=np.float32)
    # by hand: (0+4)/2, (9+0)/2, 0
    np.testing.assert_array_equal(orc.locality_score(x_cur, x_prev), [2.0, 4.5, 0.0])
    # shifting every feature of a token by c gives exactly c^2
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 64)).astype(np.float32)
    y = x.astype(np.float64) + np.array([[0.5], [0.0], [-2.0], [0.25]])
    np.testing.assert_allclose(orc.locality_score(y, x), [0.25, 0.0, 4.0, 0.0625], rtol=1e-12)
    # numpy's own mean of squares
    a, b = rng.standard_normal((2, 7, 33)).astype(np.float32)
    np.testing.assert_allclose(orc.locality_score(a, b),
                               ((a.astype(np.float64) - b.astype(np.float64)) ** 2).mean(-1), rtol=1e-13)


def test_locality_score_reads_bf16_bits():
    # 0x3F80 = 1.0, 0x4000 = 2.0, 0xC040 = -3.0 in bfloat16
    cur = np.array([[0x3F80, 0x4000]], dtype=np.uint16)
    prev = np.array([[0xC040, 0x4000]], dtype=np.uint16)
    np.testing.assert_array_equal(orc.locality_score(cur, prev), [8.0])


def test_active_set_rules(golden_dir):
    delta = np.array([0.1, 0.9, 0.3, 0.9, 0.0, 0.5])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_TOPK, 1), [1])          # tie -> smaller index
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_TOPK, 3), [1, 3, 5])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_TOPK, 6), [0, 1, 2, 3, 4, 5])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_THRESHOLD, 0.3), [1, 3, 5])  # strict >
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_THRESHOLD, 5.0), [])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_FRACTION, 1.0), np.arange(6))
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_FRACTION, 0.0), [1])     # at least one
    # the paper's setting: top-5 of a block of 16
    consts = dict(l.split() for l in open(os.path.join(golden_dir, "paper_constants.txt"))
                  if l.strip() and not l.startswith("#"))
    rng = np.random.default_rng(6)
    d16 = rng.random(int(consts["default_block"]))
    A = orc.active_set(d16, orc.SEL_TOPK, int(consts["top_tokens"]))
    assert len(A) == 5 and set(A) == set(np.argsort(-d16)[:5])
    # active counts of the benchmark configurations
    assert [orc.num_active(orc.SEL_FRACTION, f, B) for f, B in
            [(0.25, 32), (0.20, 32), (0.15, 32), (0.10, 32)]] == [8, 6, 5, 3]
    assert [orc.num_active(orc.SEL_FRACTION, f, 64) for f in (0.05, 0.10, 0.25, 0.50, 1.0)] == [3, 6, 16, 32, 64]
    assert [synth.active_count(f, 64) for f in (0.05, 0.10, 0.25, 0.50, 1.0)] == [3, 6, 16, 32, 64]


def test_active_set_cumulative_mass_rule():
    # hand values: sorted 8, 4, 2, 1, 1 (total 16); half the mass is reached by the first token alone,
    # 0.75 needs two (12 >= 12), 0.76 needs three, all of it needs all five
    delta = np.array([1.0, 8.0, 2.0, 4.0, 1.0])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_MASS, 0.5), [1])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_MASS, 0.75), [1, 3])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_MASS, 0.76), [1, 2, 3])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_MASS, 1.0), [0, 1, 2, 3, 4])
    np.testing.assert_array_equal(orc.active_set(delta, orc.SEL_MASS, 0.0), [])
    np.testing.assert_array_equal(orc.active_set(np.zeros(4), orc.SEL_MASS, 0.5), [])
    # brute force: the chosen set is a prefix of the descending order, reaches the mass, and is minimal
    rng = np.random.default_rng(12)
    for _ in range(50):
        d = rng.random(int(rng.integers(1, 20))) ** 4
        tau = float(rng.random())
        A = orc.active_set(d, orc.SEL_MASS, tau)
        srt = np.sort(d)[::-1]
        assert sorted(d[A], reverse=True) == list(srt[:len(A)])
        assert d[A].sum() >= tau * d.sum() * (1 - 1e-6)
        if len(A) > 1:
            assert srt[:len(A) - 1].sum() < tau * d.sum() * (1 + 1e-6)


def test_active_set_brute_force():
    rng = np.random.default_rng(7)
    for _ in range(50):
        B = int(rng.integers(1, 12))
        delta = rng.integers(0, 4, size=B).astype(np.float64)      # many exact ties
        n = int(rng.integers(0, B + 1))
        A = orc.active_set(delta, orc.SEL_TOPK, n)
        assert len(A) == n and list(A) == sorted(A)
        # every chosen token beats every other token under (value desc, index asc)
        rest = [i for i in range(B) if i not in set(A)]
        for i, j in itertools.product(A, rest):
            assert delta[i] > delta[j] or (delta[i] == delta[j] and i < j)


# ---------------------------------------------------------------- QUEST selector
def test_page_min_max_hand_values_and_partial_page():
    K = np.array([[1, -1], [3, -5], [2, 0], [-4, 9], [7, 7]], dtype=np.float32)   # L=5, g=2 -> 3 pages
    kmin, kmax = orc.page_min_max(K, 2)
    np.testing.assert_array_equal(kmin, [[1, -5], [-4, 0], [7, 7]])
    np.testing.assert_array_equal(kmax, [[3, -1], [2, 9], [7, 7]])
    rng = np.random.default_rng(8)
    Kb = synth.f32_to_bf16_bits(rng.standard_normal((70, 3, 8)).astype(np.float32))
    kmin, kmax = orc.page_min_max(Kb, 16)
    Kf = synth.bf16_bits_to_f32(Kb).astype(np.float64)
    assert kmin.shape == (5, 3, 8)
    for t in range(70):
        assert np.all(kmin[t // 16] <= Kf[t]) and np.all(Kf[t] <= kmax[t // 16])
    # bounds are attained, and are values of the page (no rounding)
    for p in range(5):
        page = Kf[p * 16: min(70, p * 16 + 16)]
        assert np.all((page == kmin[p][None]).any(0)) and np.all((page == kmax[p][None]).any(0))


def test_page_bound_is_upper_bound_tight_and_exact_for_single_token():
    rng = np.random.default_rng(9)
    d, g, L = 32, 4, 64
    K = rng.standard_normal((L, d)) * np.exp(rng.standard_normal(d))
    kmin, kmax = orc.page_min_max(K, g)
    for _ in range(20):
        q = rng.standard_normal(d) * 3
        s = orc.page_upper_bound(q, kmin, kmax)
        true_max = (K @ q).reshape(L // g, g).max(-1)
        assert np.all(s >= true_max - 1e-12)
        # same thing split by sign of q: q+ . max + q- . min
        alt = np.maximum(q, 0) @ kmax.T + np.minimum(q, 0) @ kmin.T
        np.testing.assert_allclose(s, alt, rtol=1e-13, atol=1e-12)
    # page of a single token: the bound is q.k itself
    kmin1, kmax1 = orc.page_min_max(K, 1)
    q = rng.standard_normal(d)
    np.testing.assert_allclose(orc.page_upper_bound(q, kmin1, kmax1), K @ q, rtol=1e-13, atol=1e-13)
    # the bound is attained when the page holds the corner key
    lo, hi = -np.abs(rng.standard_normal(d)), np.abs(rng.standard_normal(d))
    corner = np.where(q > 0, hi, lo)
    page = np.stack([corner, np.where(q > 0, lo, hi)])
    pm, pM = orc.page_min_max(page, 2)
    np.testing.assert_allclose(orc.page_upper_bound(q, pm, pM)[0], q @ corner, rtol=1e-13)
    # hand value: q=[2,-1], min=[-1,-3], max=[4,5] -> max(-2,8) + max(3,-5) = 11
    np.testing.assert_array_equal(
        orc.page_upper_bound(np.array([2.0, -1.0]), np.array([[-1.0, -3.0]]), np.array([[4.0, 5.0]])), [11.0])


def test_top_pages_brute_force_with_ties():
    rng = np.random.default_rng(10)
    for _ in range(100):
        P = int(rng.integers(1, 33))
        K = int(rng.integers(1, 40))
        s = rng.integers(-3, 4, size=P).astype(np.float64) * 0.5
        got = orc.top_pages(s, K)
        pairs = sorted(((-s[p], p) for p in range(P)))               # full sort: value desc, index asc
        want = sorted(p for _, p in pairs[: min(K, P)])
        assert list(got) == want
    np.testing.assert_array_equal(orc.top_pages(np.array([1.0, 5.0, 5.0, 2.0]), 2), [1, 2])
    np.testing.assert_array_equal(orc.top_pages(np.array([5.0, 1.0, 5.0, 5.0]), 2), [0, 2])
    # decision is taken on the float32 value: these two differ only below float32 resolution -> tie -> smaller index
    np.testing.assert_array_equal(orc.top_pages(np.array([1.0, 1.0 + 1e-12]), 1), [0])


def test_union_pages():
    np.testing.assert_array_equal(orc.union_pages([np.array([3, 1]), np.array([1, 7]), np.array([], dtype=np.int32)]),
                                  [1, 3, 7])
    np.testing.assert_array_equal(orc.union_pages([]), [])


def test_tokens_of_pages_partial_last_page():
    np.testing.assert_array_equal(orc.tokens_of_pages(np.array([0, 2]), 4, 10), [0, 1, 2, 3, 8, 9])


# ---------------------------------------------------------------- whole step
def _small_inputs(dtype="bf16", seq_lens=(200,), n_active=3, topk=3, T=4, batch=None, Hq=4, Hkv=2, seed=5):
    w = synth.config(0, dtype=dtype).replace(seq_lens=tuple(seq_lens), batch=len(seq_lens), n_active=n_active,
                                             topk_pages=topk, T=T, B=8, Hq=Hq, Hkv=Hkv, d=16, seed=seed)
    return synth.make_inputs(w)


def _dense_reference(inp, t):
    """Prefix-only dense attention for every row, through scipy."""
    w = inp.w
    o = np.empty((w.batch * w.B, w.Hq, w.d))
    L = np.empty((w.batch * w.B, w.Hq))
    qf = synth.load(inp.q[t]).astype(np.float64)
    for b in range(w.batch):
        Kf, Vf = synth.load(inp.K[b]).astype(np.float64), synth.load(inp.V[b]).astype(np.float64)
        for h in range(w.Hq):
            s = qf[b * w.B:(b + 1) * w.B, h] @ Kf[:, h // w.G].T / np.sqrt(w.d)
            o[b * w.B:(b + 1) * w.B, h] = softmax(s, -1) @ Vf[:, h // w.G]
            L[b * w.B:(b + 1) * w.B, h] = logsumexp(s, -1)
    return o, L


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dense_init_and_budget_covering_all_pages_equal_dense(dtype):
    inp = _small_inputs(dtype, seq_lens=(200, 37))
    w = inp.w
    cache = orc.PrefixCache(inp.K, inp.V, w.g)
    o = np.zeros((w.batch * w.B, w.Hq, w.d)); L = np.zeros((w.batch * w.B, w.Hq))
    tr = orc.losa_step(cache, 0, None, None, inp.q[0], orc.SEL_TOPK, w.n_active, w.topk_pages, w.B, w.Hq, o, L)
    ro, rL = _dense_reference(inp, 0)
    np.testing.assert_allclose(o, ro, atol=1e-12)
    np.testing.assert_allclose(L, rL, atol=1e-12)
    assert all(len(a) == w.B for a in tr.active)
    # sparse step with every token active and a budget of at least P pages is dense attention too
    o2 = np.full_like(o, np.nan); L2 = np.full_like(L, np.nan)
    orc.losa_step(cache, 1, inp.h[1], inp.h[0], inp.q[1], orc.SEL_FRACTION, 1.0, 10 ** 6, w.B, w.Hq, o2, L2)
    ro, rL = _dense_reference(inp, 1)
    np.testing.assert_allclose(o2, ro, atol=1e-12)
    np.testing.assert_allclose(L2, rL, atol=1e-12)


def test_sparse_step_reuse_union_and_attention_over_union():
    inp = _small_inputs(seq_lens=(200, 150), n_active=3, topk=3)
    w = inp.w
    cache = orc.PrefixCache(inp.K, inp.V, w.g)
    o = np.zeros((w.batch * w.B, w.Hq, w.d)); L = np.zeros((w.batch * w.B, w.Hq))
    orc.losa_step(cache, 0, None, None, inp.q[0], orc.SEL_TOPK, w.n_active, w.topk_pages, w.B, w.Hq, o, L)
    o_before, L_before = o.copy(), L.copy()
    tr = orc.losa_step(cache, 1, inp.h[1], inp.h[0], inp.q[1], orc.SEL_TOPK, w.n_active, w.topk_pages,
                       w.B, w.Hq, o, L, keep_scores=True)
    qf = synth.load(inp.q[1]).astype(np.float64)
    for b in range(w.batch):
        A = tr.active[b]
        # the generator perturbed exactly these tokens
        np.testing.assert_array_equal(A, inp.picked[1, b])
        stable = np.setdiff1d(np.arange(w.B), A) + b * w.B
        # reuse rule: stable rows are bit-identical
        assert np.array_equal(o[stable], o_before[stable]) and np.array_equal(L[stable], L_before[stable])
        P = w.pages_per_seq[b]
        Kf, Vf = synth.load(inp.K[b]).astype(np.float64), synth.load(inp.V[b]).astype(np.float64)
        for j in range(w.Hkv):
            I = tr.union[(b, j)]
            M = len(A) * w.G
            # union size bounds (Union Size section)
            assert w.topk_pages <= len(I) <= min(P, M * w.topk_pages)
            members = set()
            for i in A:
                for h in range(j * w.G, (j + 1) * w.G):
                    pk = tr.picks[(b, int(i), h)]
                    assert len(pk) == min(w.topk_pages, P)
                    s = tr.scores[(b, int(i), h)]
                    # brute force: no unpicked page has a larger float32 bound than a picked one
                    s32 = s.astype(np.float32)
                    outside = np.setdiff1d(np.arange(P), pk)
                    assert s32[pk].min() >= s32[outside].max()
                    members |= set(int(p) for p in pk)
            assert sorted(members) == list(I)
            # active rows: attention over exactly the union's tokens (scipy)
            tok = np.concatenate([np.arange(p * w.g, min(w.seq_lens[b], (p + 1) * w.g)) for p in I])
            for i in A:
                for h in range(j * w.G, (j + 1) * w.G):
                    s = qf[b * w.B + i, h] @ Kf[tok, j].T / np.sqrt(w.d)
                    np.testing.assert_allclose(o[b * w.B + i, h], softmax(s) @ Vf[tok, j], atol=1e-12)
                    np.testing.assert_allclose(L[b * w.B + i, h], logsumexp(s), atol=1e-12)


def test_union_never_grows_when_fewer_tokens_are_active():
    inp = _small_inputs(seq_lens=(400,), n_active=2, topk=4)
    w = inp.w
    cache = orc.PrefixCache(inp.K, inp.V, w.g)
    o = np.zeros((w.B, w.Hq, w.d)); L = np.zeros((w.B, w.Hq))
    sizes = []
    for n in (1, 2, 4, 8):
        tr = orc.losa_step(cache, 1, inp.h[1], inp.h[0], inp.q[1], orc.SEL_TOPK, n, w.topk_pages, w.B, w.Hq, o, L)
        sizes.append([len(tr.union[(0, j)]) for j in range(w.Hkv)])
        for j in range(w.Hkv):
            assert len(tr.union[(0, j)]) <= min(w.pages_per_seq[0], n * w.G * w.topk_pages)
    sizes = np.array(sizes)
    assert np.all(np.diff(sizes, axis=0) >= 0)          # |U(A)| <= |U(A')| for A subset A' (top-n sets are nested)


def test_dense_prefix_plus_block_merge_equals_full_attention_over_prefix_and_block():
    # eq. full_attn through scipy, for every token and head, GQA included
    inp = _small_inputs(seq_lens=(100, 37))
    w = inp.w
    kb, vb = synth.make_block_kv(w)
    cache = orc.PrefixCache(inp.K, inp.V, w.g)
    o = np.zeros((w.batch * w.B, w.Hq, w.d)); L = np.zeros((w.batch * w.B, w.Hq))
    orc.losa_step(cache, 0, None, None, inp.q[0], 0, 0, 0, w.B, w.Hq, o, L)
    O, o_b, L_b = orc.block_attention_and_merge(inp.q[0], kb[0], vb[0], o, L, w.B)
    qf = synth.load(inp.q[0]).astype(np.float64)
    kbf, vbf = synth.load(kb[0]).astype(np.float64), synth.load(vb[0]).astype(np.float64)
    for b in range(w.batch):
        Kp, Vp = synth.load(inp.K[b]).astype(np.float64), synth.load(inp.V[b]).astype(np.float64)
        sl = slice(b * w.B, (b + 1) * w.B)
        for h in range(w.Hq):
            j = h // w.G
            K_all = np.concatenate([Kp[:, j], kbf[sl, j]]); V_all = np.concatenate([Vp[:, j], vbf[sl, j]])
            full = softmax(qf[sl, h] @ K_all.T / np.sqrt(w.d), axis=-1) @ V_all
            np.testing.assert_allclose(O[sl, h], full, atol=1e-12)
            np.testing.assert_allclose(L_b[sl, h], logsumexp(qf[sl, h] @ kbf[sl, j].T / np.sqrt(w.d), axis=-1), atol=1e-12)
    # an empty prefix (L_p = -inf) leaves the block attention alone
    O2, o_b2, _ = orc.block_attention_and_merge(inp.q[0], kb[0], vb[0], np.zeros_like(o), np.full_like(L, -np.inf), w.B)
    np.testing.assert_allclose(O2, o_b2, atol=1e-14)


def test_empty_active_set_is_a_no_op():
    inp = _small_inputs()
    w = inp.w
    cache = orc.PrefixCache(inp.K, inp.V, w.g)
    o = np.full((w.B, w.Hq, w.d), 3.0); L = np.full((w.B, w.Hq), -1.0)
    tr = orc.losa_step(cache, 1, inp.h[1], inp.h[0], inp.q[1], orc.SEL_THRESHOLD, 1e9, w.topk_pages, w.B, w.Hq, o, L)
    assert len(tr.active[0]) == 0 and np.all(o == 3.0) and np.all(L == -1.0)


def test_cache_state_size_matches_paper(golden_dir):
    consts = dict(l.split() for l in open(os.path.join(golden_dir, "paper_constants.txt"))
                  if l.strip() and not l.startswith("#"))
    B, d = 16, 128
    o = np.zeros((B, 1, d)); L = np.zeros((B, 1))
    assert o.size + L.size == int(consts["cache_scalars_B16_d128"]) == B * (d + 1)


# ---------------------------------------------------------------- input generators
def test_bf16_conversion_matches_torch():
    import torch
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(20000) * np.exp(rng.standard_normal(20000) * 4)).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]          # includes exact ties (round to even)
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())
    np.testing.assert_array_equal(orc.widen(bits), ref.to(torch.float64).numpy())


def test_generators_are_seeded_and_shaped():
    w = synth.config(0)
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    assert np.array_equal(a.h, b.h) and np.array_equal(a.K[0], b.K[0]) and np.array_equal(a.page_indices, b.page_indices)
    assert a.K[0].shape == (2048, 1, 64) and a.h.shape == (8, 32, 256) and a.q.shape == (8, 32, 4, 64)
    assert sorted(a.page_indices) == list(range(128))
    kp, vp = synth.pack_pages(a)
    p, tok = 5, 3
    phys = a.page_indices[p]
    assert np.array_equal(kp[phys, 0, tok], a.K[0][p * 16 + tok, 0])
    assert np.array_equal(vp[phys, 0, :, tok], a.V[0][p * 16 + tok, 0])
    c2 = synth.config(2)
    assert len(c2.seq_lens) == 16 and min(c2.seq_lens) >= 8192 and max(c2.seq_lens) <= 32768
    assert [synth.config(i).n_active for i in range(4)] == [8, 6, 5, 3]
    assert [synth.config(i).topk_pages for i in range(4)] == [32, 128, 64, 256]


# --------------------------------------------------------------------------
# Shared page budget per KV head (not in the paper; the alternative reading of the budget)
# --------------------------------------------------------------------------
def test_shared_budget_reads_exactly_k_pages_and_reduces_to_the_per_query_rule_for_one_query():
    rng = np.random.default_rng(77)
    P, M, K = 40, 6, 7
    s = rng.normal(size=(M, P)).astype(np.float32)
    got = orc.shared_top_pages(s, K)
    assert len(got) == K and np.all(np.diff(got) > 0)
    assert len(orc.shared_top_pages(s, P + 5)) == P                      # budget above the page count
    assert np.array_equal(orc.shared_top_pages(s[:1], K), orc.top_pages(s[0], K))   # one query: same rule
    # brute force: a page is kept iff fewer than K pages beat its best score (ties: smaller page wins)
    best = s.max(axis=0)
    want = [p for p in range(P)
            if sum((best[r] > best[p]) or (best[r] == best[p] and r < p) for r in range(P)) < K]
    assert list(got) == want
    # no dropped page has a better best-score than a kept one; the overall best page is always kept
    kept = np.zeros(P, dtype=bool)
    kept[got] = True
    assert best[kept].min() >= best[~kept].max()
    assert int(np.argmax(best)) in set(orc.shared_top_pages(s, 1))
    # growing the budget only adds pages
    assert set(orc.shared_top_pages(s, 5)) <= set(orc.shared_top_pages(s, 9))


def test_shared_budget_ties_go_to_the_smaller_page():
    s = np.zeros((3, 10), dtype=np.float32)
    s[1, 7] = 1.0
    assert list(orc.shared_top_pages(s, 4)) == [0, 1, 2, 7]
