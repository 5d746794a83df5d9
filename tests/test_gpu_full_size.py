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


def test_c1_every_denoising_step_of_a_block():
    """All 16 steps of a C1 block in a row (dense initialisation, then 15 sparse steps on the state the
    previous ones left): rows that are never active keep their initial values bit for bit, active rows
    follow the oracle step by step."""
    _run(synth.config(1), range(16))


def test_c3_full_128k():
    _run(synth.config(3).replace(T=3), range(3))


def test_c2_ragged_batch_full():
    w = synth.config(2)
    _run(w.replace(T=3), range(3))


@pytest.fixture(scope="module")
def c4_rig():
    """C4 at its stated size (batch 4, 64k-token prefixes, pages of 32, block 64): keys, values and
    page bounds are shared by every sweep point, and so is the dense initialisation (step 0 sees
    the same h_0 / q_0 whatever the number of active tokens), which is checked once here."""
    import torch
    rig = Rig(synth.config(4).replace(T=2))
    check_page_bounds(rig)
    run_steps_end_to_end(rig, [0], orc.SEL_TOPK, float(rig.w.n_active), rig.w.topk_pages)
    torch.cuda.synchronize()
    rig.dense = (rig.blk.o_p.clone(), rig.blk.lse_p.clone(), rig.o_ref.copy(), rig.L_ref.copy(), rig.inp.q[0].copy())
    yield rig
    rig.close()


@pytest.mark.parametrize("budget", [1024, 2048, 4096])
@pytest.mark.parametrize("fraction", [0.05, 0.10, 0.25, 0.50, 1.00])
def test_c4_sweep_points_at_batch_4(c4_rig, fraction, budget):
    """Every point of the C4 sweep (active fraction x page budget, 100 % active being the
    QUEST-style setting without locality pruning) at the full batch of 4: sparse steps on top of
    the shared dense initialisation, every decision and every output against the oracle.  The two
    points the reports quote (10 % / 2048 tokens and 5 % / 4096 tokens) run two sparse steps."""
    from paper_2604_12056_amd.device_inputs import DeviceBlock
    rig = c4_rig
    quoted = (fraction, budget) in ((0.10, 2048), (0.05, 4096))
    w = synth.config(4, active_fraction=fraction, budget_tokens=budget).replace(T=3 if quoted else 2)
    h, q, picked = synth.make_block_states(w)
    o_p0, lse_p0, o_ref0, L_ref0, q0 = rig.dense
    assert np.array_equal(q[0], q0), "step 0 of every sweep point must see the same queries"
    rig.w = w
    rig.inp.w, rig.inp.h, rig.inp.q, rig.inp.picked = w, h, q, picked
    rig.blk = DeviceBlock(rig.inp)
    rig.blk.o_p.copy_(o_p0); rig.blk.lse_p.copy_(lse_p0)
    rig.o_ref[:], rig.L_ref[:] = o_ref0, L_ref0
    rig.near_ties = 0
    run_steps_end_to_end(rig, range(1, w.T), orc.SEL_TOPK, float(w.n_active), w.topk_pages)
    assert rig.near_ties <= 4, f"{rig.near_ties} near-tie decisions differed"


def test_c1_full_float_mode():
    _run(synth.config(1, dtype="f32").replace(T=2, seq_lens=(8192 + 40,)), range(2))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_float_mode_at_the_stated_sizes(cfg):
    """The float validation mode at each benchmark configuration's own size (C1 32k, C2 sixteen
    ragged sequences, C3 128k, C4 four sequences of 64k with 64-token blocks and 32-token pages):
    dense initialisation and a sparse step, every decision and output against the oracle at 1e-4."""
    _run(synth.config(cfg, dtype="f32").replace(T=2), range(2))


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
