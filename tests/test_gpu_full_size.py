"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times (losa_step, top-n selection).  The numpy oracle is fast enough to check every
output of these steps, so nothing is sampled: dense initialisation, then sparse steps, active
masks / union sizes / (o_p, lse_p) against the oracle after each."""
import numpy as np
import pytest

from oracle import losa_oracle as orc
from paper_2604_12056_amd import synth

from parity_util import Rig, check_page_bounds, run_steps_end_to_end

pytestmark = pytest.mark.gpu


def _run(w, steps):
    rig = Rig(w)
    try:
        check_page_bounds(rig)
        run_steps_end_to_end(rig, steps, orc.SEL_TOPK, float(w.n_active), w.topk_pages)
        assert rig.near_ties <= 4, f"{rig.near_ties} near-tie decisions differed"
    finally:
        rig.close()


def test_c1_full_32k():
    _run(synth.config(1).replace(T=4), range(4))


def test_c3_full_128k():
    _run(synth.config(3).replace(T=3), range(3))


def test_c2_ragged_batch_full():
    w = synth.config(2)
    _run(w.replace(T=3), range(3))


@pytest.mark.parametrize("fraction,budget", [(0.05, 1024), (0.25, 2048), (0.5, 2048), (1.0, 1024)])
def test_c4_sweep_points(fraction, budget):
    # batch 2 of the 4 sequences keeps the oracle's host memory and time modest; shapes are C4's
    w = synth.config(4, active_fraction=fraction, budget_tokens=budget)
    _run(w.replace(batch=2, seq_lens=w.seq_lens[:2], T=3), range(3))


def test_c1_full_float_mode():
    _run(synth.config(1, dtype="f32").replace(T=2, seq_lens=(8192 + 40,)), range(2))


@pytest.mark.parametrize("pages,tail", [(3001, 5), (9001, 5), (9004, 11), (16384, 0)])
def test_long_sequences_up_to_the_page_limit(pages, tail):
    """Above 2048 / 8192 pages the selection kernel holds 32 / 64 keys per thread (16384 pages is
    the limit of the interface); page counts that are not a multiple of four take its scalar
    score loads.  A single-KV-head shape keeps the oracle quick."""
    L = 16 * (pages - 1) + (tail if tail else 16)
    w = synth.config(0).replace(seq_lens=(L,), topk_pages=96, T=3, name=f"C0-{pages}-pages")
    assert w.max_pages == pages
    _run(w, range(3))


@pytest.mark.parametrize("pages", [3001, 9004])
def test_shared_budget_on_long_sequences(pages):
    """The shared page budget per KV head (one workgroup per head) in its 1024-thread forms."""
    from parity_util import check_score_pages_shared, check_sparse_attn
    w = synth.config(0).replace(seq_lens=(16 * (pages - 1) + 9,), topk_pages=96, T=2, name=f"C0-{pages}-pages-shared")
    rig = Rig(w)
    try:
        check_page_bounds(rig)
        check_sparse_attn(rig, 0, None, None, dense=True)
        delta = orc.locality_score(rig.inp.h[1], rig.inp.h[0])
        active = [orc.active_set(delta[:w.B], orc.SEL_TOPK, float(w.n_active))]
        sets = check_score_pages_shared(rig, 1, active, w.topk_pages)
        check_sparse_attn(rig, 1, active, sets)
        assert rig.near_ties <= 2
    finally:
        rig.close()


def _random_large_workload(seed: int):
    rng = np.random.Generator(np.random.Philox(5000 + seed))
    B = int(rng.choice([16, 32, 64]))
    Hkv = int(rng.choice([1, 2]))
    G = int(rng.choice([1, 4, 7, 8]))
    d = int(rng.choice([64, 128]))
    g = int(rng.choice([16, 32]))
    batch = int(rng.integers(1, 3))
    lens = tuple(int(rng.integers(1, 60000)) for _ in range(batch))
    dtype = "f32" if rng.integers(0, 6) == 0 else "bf16"
    if dtype == "f32":
        lens = tuple(min(x, 6000) for x in lens)
    return synth.config(0, dtype=dtype).replace(B=B, Hq=Hkv * G, Hkv=Hkv, d=d, g=g, batch=batch, seq_lens=lens,
                                                n_active=int(rng.integers(1, B + 1)), topk_pages=int(rng.integers(1, 40)),
                                                T=3, outliers=str(rng.choice(["fixed4x8", "lognormal"])),
                                                seed=9000 + seed, name=f"random-large-{seed}")


@pytest.mark.parametrize("seed", range(10))
def test_random_large_shapes(seed):
    """Seeded random shapes with prefixes up to 60k tokens (the 1024-thread selection forms), up to
    512 query rows per KV head in sparse steps (the many-row attention shape) and, now and then,
    the float mode; a randomly chosen selection mode."""
    w = _random_large_workload(seed)
    rng = np.random.Generator(np.random.Philox(300 + seed))
    mode, param = [(orc.SEL_TOPK, float(w.n_active)), (orc.SEL_FRACTION, w.n_active / w.B),
                   (orc.SEL_THRESHOLD, 0.01), (orc.SEL_MASS, 0.5)][int(rng.integers(0, 4))]
    rig = Rig(w)
    try:
        check_page_bounds(rig)
        run_steps_end_to_end(rig, range(w.T), mode, param, w.topk_pages)
        assert rig.near_ties <= 6
    finally:
        rig.close()
