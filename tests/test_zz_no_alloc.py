"""The allocation-free entry point (losa_select_active_static: ticket counters in a device array
of the library instead of the caller's workspace) against the entry point it is a variant of,
through the C ABI: same locality scores bit for bit, same masks, lists and counts, in every
selection mode, on two calls in a row of which the second has a smaller input."""
import numpy as np
import pytest
import torch

from oracle import losa_oracle as orc
from paper_2604_12056_amd import binding as L
from paper_2604_12056_amd import synth
from paper_2604_12056_amd.device_inputs import DeviceBlock, config_of

pytestmark = pytest.mark.gpu


def _outputs(rows, batch, dev):
    return (torch.full((rows,), -3.0, dtype=torch.float32, device=dev), torch.full((rows,), 9, dtype=torch.uint8, device=dev),
            torch.full((rows,), -9, dtype=torch.int32, device=dev), torch.full((batch,), -9, dtype=torch.int32, device=dev))


def _compare(w, mode, param, dev="cuda:0"):
    inp = synth.make_inputs(w)
    blk = DeviceBlock(inp, dev)
    ctx = L.losa_create(config_of(w), dev)
    try:
        rows = w.batch * w.B
        dtype = L.LOSA_BF16 if w.dtype == "bf16" else L.LOSA_F32
        for t in range(1, w.T):
            ref = _outputs(rows, w.batch, dev)
            got = _outputs(rows, w.batch, dev)
            L.losa_select_active(ctx, blk.h[t], blk.h[t - 1], mode, param, *ref)
            L.losa_select_active_static(dtype, w.batch, w.B, w.H, blk.h[t], blk.h[t - 1], mode, param, *got)
            torch.cuda.synchronize()
            for a, b, what in zip(got, ref, ("delta", "mask", "active_idx", "active_count")):
                assert torch.equal(a, b), f"{w.name} step {t} mode {mode}: {what} differs from losa_select_active"
            # and the oracle's active sets, so that the pair is not only self-consistent
            delta = orc.locality_score(inp.h[t], inp.h[t - 1])
            cnt = got[3].cpu().numpy()
            idx = got[2].cpu().numpy().reshape(w.batch, w.B)
            for b in range(w.batch):
                A = orc.active_set(delta[b * w.B:(b + 1) * w.B], mode, param)
                assert np.array_equal(idx[b, :cnt[b]], A)
    finally:
        ctx.close()


def test_static_scratch_variant_matches_on_two_calls_in_a_row():
    big = synth.config(2).replace(batch=16, seq_lens=(64,) * 16, T=3, name="static-big")                 # 16 sequences of 32 tokens
    small = synth.config(0).replace(B=16, Hq=4, Hkv=1, d=64, batch=3, seq_lens=(64,) * 3, n_active=5, T=3,
                                    name="static-small")                                                   # then 3 sequences of 16
    for mode_of in (lambda w: (orc.SEL_TOPK, float(w.n_active)), lambda w: (orc.SEL_FRACTION, 0.25),
                    lambda w: (orc.SEL_THRESHOLD, 0.01), lambda w: (orc.SEL_MASS, 0.5)):
        _compare(big, *mode_of(big))
        _compare(small, *mode_of(small))
    f32 = synth.config(0, dtype="f32").replace(batch=2, seq_lens=(64, 64), T=3, name="static-f32")
    _compare(f32, orc.SEL_TOPK, float(f32.n_active))


def test_static_scratch_variant_rejects_sizes_beyond_its_array():
    lib = L.load_library()
    fake = 1 << 20
    uns, inv = L.LOSA_ERR_UNSUPPORTED, L.LOSA_ERR_INVALID_ARG
    assert lib.losa_select_active_static(None, 0, 4097, 32, 256, fake, fake, 0, 5.0, fake, fake, fake, fake) == uns
    assert b"4096" in lib.losa_last_error(None)
    assert lib.losa_select_active_static(None, 0, 4, 1025, 256, fake, fake, 0, 5.0, fake, fake, fake, fake) == uns
    assert lib.losa_select_active_static(None, 0, 4, 32, 252, fake, fake, 0, 5.0, fake, fake, fake, fake) == uns
    assert lib.losa_select_active_static(None, 0, 0, 32, 256, fake, fake, 0, 5.0, fake, fake, fake, fake) == inv
    assert lib.losa_select_active_static(None, 0, 4, 32, 256, None, fake, 0, 5.0, fake, fake, fake, fake) == inv
    assert lib.losa_select_active_static(None, 0, 4, 32, 256, fake, fake, 9, 5.0, fake, fake, fake, fake) == inv
    assert lib.losa_select_active_static(None, 7, 4, 32, 256, fake, fake, 0, 5.0, fake, fake, fake, fake) == inv
