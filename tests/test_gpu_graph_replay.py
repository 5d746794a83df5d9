"""GPU parity of the launch path the benchmark times: a block's whole sequence of calls (dense
initialisation, the sparse denoising steps, the in-block attention and final merge) captured
once into a HIP graph and replayed.  Every replay is checked against the oracle: the cached
prefix statistics after the last step (rows keep the values of the step that last recomputed
them, so every step shows in the final state), the per-step active masks and union sizes the
steps reported, and the merged attention output.  Between the replays the program does eager
work of its own on the same context and synchronises."""
import numpy as np
import pytest
import torch

from oracle import losa_oracle as orc
from paper_2604_12056_amd import binding as L
from paper_2604_12056_amd import synth
from paper_2604_12056_amd.device_inputs import to_device

from parity_util import Rig, check_page_bounds, compare_state, follow_step, tol

pytestmark = pytest.mark.gpu


def _graph_of_a_block(rig, mode, param, topk, masks, counts, dkb, dvb, out):
    w, blk = rig.w, rig.blk

    def calls():
        for t in range(w.T):
            L.losa_step(rig.ctx, rig.layer.kv, t, blk.h[t] if t else None, blk.h[t - 1] if t else None, blk.q[t],
                        mode, param, topk, blk.o_p, blk.lse_p, masks[t], counts[t])
        L.losa_block_merge(rig.ctx, blk.q[w.T - 1], dkb, dvb, blk.o_p, blk.lse_p, out)

    calls()                       # eager once: one-time set-up of the library happens outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    return g


def _replay_and_compare(w, mode, param, replays=2):
    rig = Rig(w)
    try:
        blk = rig.blk
        dev = blk.q.device
        check_page_bounds(rig)
        rows = w.batch * w.B
        masks = torch.zeros((w.T, rows), dtype=torch.uint8, device=dev)
        counts = torch.zeros((w.T, w.batch, w.Hkv), dtype=torch.int32, device=dev)
        kb, vb = synth.make_block_kv(w)
        dkb, dvb = to_device(kb[w.T - 1], dev), to_device(vb[w.T - 1], dev)
        out = torch.empty_like(blk.o_p)
        g = _graph_of_a_block(rig, mode, param, w.topk_pages, masks, counts, dkb, dvb, out)
        for rep in range(replays):
            # eager work and state the replay must overwrite: garbage in the cached statistics and the
            # diagnostics, one eager step of another kind on the same context
            blk.o_p.fill_(float("nan")); blk.lse_p.fill_(7.0); out.fill_(float("nan"))
            masks.fill_(3); counts.fill_(-5)
            L.losa_step(rig.ctx, rig.layer.kv, 1, blk.h[1], blk.h[0], blk.q[1], orc.SEL_THRESHOLD, 0.01, w.topk_pages,
                        blk.o_p, blk.lse_p)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            # oracle over the same block, following the decisions each step reported
            rig.o_ref[:] = 0.0; rig.L_ref[:] = 0.0
            o_gpu, l_gpu = blk.o_p.clone(), blk.lse_p.clone()      # follow_step runs losa_score_pages: keep the state apart
            out_gpu = out.cpu().numpy()
            mk, ct = masks.cpu().numpy(), counts.cpu().numpy()
            orc.losa_step(rig.cache, 0, None, None, rig.inp.q[0], mode, param, w.topk_pages, w.B, w.Hq, rig.o_ref, rig.L_ref)
            for t in range(1, w.T):
                follow_step(rig, t, mode, param, w.topk_pages, mk[t], ct[t])
            assert torch.equal(blk.o_p, o_gpu) and torch.equal(blk.lse_p, l_gpu)
            compare_state(rig, [np.arange(w.B)] * w.batch)
            O_ref, _, _ = orc.block_attention_and_merge(rig.inp.q[w.T - 1], kb[w.T - 1], vb[w.T - 1], rig.o_ref, rig.L_ref, w.B)
            err = np.abs(out_gpu - O_ref).max()
            assert err <= tol(w), f"replay {rep}: merged attention output off by {err}"
        assert rig.near_ties <= 4
    finally:
        rig.close()


SMALL = synth.config(2).replace(batch=3, seq_lens=(1000, 517, 2049), topk_pages=8, T=4, name="C2-small")


@pytest.mark.parametrize("mode,param", [(orc.SEL_TOPK, float(SMALL.n_active)), (orc.SEL_FRACTION, SMALL.n_active / SMALL.B),
                                        (orc.SEL_THRESHOLD, 0.01), (orc.SEL_MASS, 0.5)])
def test_graph_replay_small_every_selection_mode(mode, param):
    _replay_and_compare(SMALL, mode, param)


def test_graph_replay_tiny_config():
    w = synth.config(0).replace(T=4)
    _replay_and_compare(w, orc.SEL_TOPK, float(w.n_active))


def test_graph_replay_c1_full_size():
    """The benchmark's configuration and launch path: C1 at its full size, top-n selection."""
    w = synth.config(1).replace(T=4)
    _replay_and_compare(w, orc.SEL_TOPK, float(w.n_active))


def test_graph_replay_float_mode():
    w = synth.config(0, dtype="f32").replace(T=3, name="C0-f32")
    _replay_and_compare(w, orc.SEL_TOPK, float(w.n_active))
