"""The C-ABI library loads, exports every symbol the header declares, and its host-side
validation reports errors without touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2604_12056_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_12056_amd.build import build_library
        build_library(verbose=False)
    return binding.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "losa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(losa_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def _cfg(**kw):
    base = dict(max_batch=2, num_q_heads=8, num_kv_heads=2, head_dim=128, hidden_size=1024, page_size=16,
                block_size=32, max_pages_per_seq=64, max_topk_pages=16)
    base.update(kw)
    return binding.make_config(**base)


@pytest.mark.parametrize("kw", [dict(num_q_heads=7), dict(block_size=0), dict(max_batch=0), dict(dtype=5),
                                dict(max_pages_per_seq=0), dict(max_topk_pages=0), dict(sm_scale=-1.0), dict(head_dim=0)])
def test_invalid_config_is_rejected(lib, kw):
    cfg = _cfg(**kw)
    assert binding.losa_workspace_bytes(cfg) == 0
    out = C.c_void_p()
    st = lib.losa_create(C.byref(cfg), 4096, 1 << 40, C.byref(out))
    assert st == binding.LOSA_ERR_INVALID_ARG and not out.value
    assert len(lib.losa_last_error(None)) > 0


@pytest.mark.parametrize("kw", [dict(head_dim=96), dict(head_dim=256), dict(page_size=8), dict(page_size=64),
                                dict(block_size=257), dict(hidden_size=1001), dict(max_pages_per_seq=16385),
                                dict(block_size=256, num_q_heads=34, num_kv_heads=2)])
def test_configuration_outside_what_the_kernels_are_built_for_is_unsupported(lib, kw):
    """Sensible values the kernels have no instantiation for are reported as LOSA_ERR_UNSUPPORTED,
    apart from values that make no sense at all (LOSA_ERR_INVALID_ARG)."""
    cfg = _cfg(**kw)
    assert binding.losa_workspace_bytes(cfg) == 0
    out = C.c_void_p()
    st = lib.losa_create(C.byref(cfg), 4096, 1 << 40, C.byref(out))
    assert st == binding.LOSA_ERR_UNSUPPORTED and not out.value
    assert len(lib.losa_last_error(None)) > 0


def test_workspace_checks_and_argument_validation(lib):
    cfg = _cfg()
    need = binding.losa_workspace_bytes(cfg)
    assert need > 0
    out = C.c_void_p()
    assert lib.losa_create(C.byref(cfg), None, need, C.byref(out)) == binding.LOSA_ERR_WORKSPACE
    assert lib.losa_create(C.byref(cfg), 4096 + 8, need, C.byref(out)) == binding.LOSA_ERR_WORKSPACE   # misaligned
    assert lib.losa_create(C.byref(cfg), 4096, need - 1, C.byref(out)) == binding.LOSA_ERR_WORKSPACE
    assert b"needed" in lib.losa_last_error(None)
    # a context over a fake (never dereferenced) workspace address: host-side validation only
    assert lib.losa_create(C.byref(cfg), 4096, need, C.byref(out)) == binding.LOSA_OK and out.value
    ctx = out.value
    try:
        fake = 1 << 20
        kv = binding.losa_kv(fake, fake, fake, fake, fake, fake, 2, 100, 0)
        inv = binding.LOSA_ERR_INVALID_ARG
        assert lib.losa_select_active(ctx, None, 3, fake, fake, 0, 5.0, fake, fake, fake, fake) == inv   # batch > max
        assert lib.losa_select_active(ctx, None, 1, None, fake, 0, 5.0, fake, fake, fake, fake) == inv   # NULL input
        assert lib.losa_select_active(ctx, None, 1, fake, fake, 7, 5.0, fake, fake, fake, fake) == inv   # bad mode
        assert lib.losa_select_active(ctx, None, 1, fake, fake, 1, 1.5, fake, fake, fake, fake) == inv   # fraction > 1
        assert lib.losa_select_active(ctx, None, 1, fake, fake, 3, 1.5, fake, fake, fake, fake) == inv   # mass > 1
        assert lib.losa_block_merge(ctx, None, 1, fake, None, fake, fake, fake, fake, None, None) == inv  # NULL k_b
        assert lib.losa_block_merge(ctx, None, 9, fake, fake, fake, fake, fake, fake, None, None) == inv  # batch > max
        assert lib.losa_page_bounds(ctx, None, None, 0, -1) == inv
        assert lib.losa_page_bounds(ctx, None, C.byref(kv), -1, -1) == inv
        bad = binding.losa_kv(fake, fake, None, fake, fake, fake, 2, 100, 0)
        assert lib.losa_page_bounds(ctx, None, C.byref(bad), 0, -1) == inv                     # no metadata buffer
        bad = binding.losa_kv(fake, fake, fake, fake, fake, fake, 3, 100, 0)
        assert lib.losa_page_bounds(ctx, None, C.byref(bad), 0, -1) == inv                     # batch > max
        bad = binding.losa_kv(fake, fake, fake, fake, fake, fake, 2, 100, 65)
        assert lib.losa_page_bounds(ctx, None, C.byref(bad), 0, -1) == inv                     # max_seq_pages > config
        assert lib.losa_score_pages(ctx, None, C.byref(kv), fake, fake, fake, 17, None, fake, fake, 64) == inv  # K > max
        assert lib.losa_score_pages(ctx, None, C.byref(kv), fake, fake, fake, 4, None, fake, fake, 8) == inv    # cap small
        assert b"worst case" in lib.losa_last_error(ctx)
        assert lib.losa_score_pages_shared(ctx, None, C.byref(kv), fake, fake, fake, 17, fake, fake, 64) == inv  # K > max
        assert lib.losa_score_pages_shared(ctx, None, C.byref(kv), fake, fake, fake, 4, fake, fake, 3) == inv    # cap small
        assert lib.losa_score_pages_shared(ctx, None, C.byref(kv), fake, None, fake, 4, fake, fake, 64) == inv   # NULL list
        assert lib.losa_sparse_attn(ctx, None, C.byref(kv), fake, fake, None, None, None, 0, fake, fake) == inv  # half a pair
        assert lib.losa_sparse_attn(ctx, None, C.byref(kv), fake, None, None, fake, None, 0, fake, fake) == inv
        assert lib.losa_sparse_attn(ctx, None, C.byref(kv), None, None, None, None, None, 0, fake, fake) == inv
        assert lib.losa_step(ctx, None, C.byref(kv), 1, None, None, fake, 0, 5.0, 4, fake, fake, None, None) == inv
        assert lib.losa_step(ctx, None, C.byref(kv), -1, fake, fake, fake, 0, 5.0, 4, fake, fake, None, None) == inv
        assert lib.losa_step(ctx, None, C.byref(kv), 1, fake, fake, fake, 0, 5.0, 99, fake, fake, None, None) == inv
        assert lib.losa_set_tuning(ctx, binding.LOSA_TUNE_ATTN_WORKGROUPS, 0) == inv
        assert lib.losa_set_tuning(ctx, binding.LOSA_TUNE_ATTN_WORKGROUPS, 5000) == inv
        assert lib.losa_set_tuning(ctx, binding.LOSA_TUNE_SCORE_ROUND, 0) == inv
        assert lib.losa_set_tuning(ctx, 99, 1) == inv
        assert lib.losa_set_tuning(ctx, binding.LOSA_TUNE_SHARED_TILES, 0) == binding.LOSA_OK
        assert lib.losa_set_tuning(ctx, binding.LOSA_TUNE_HALF_PRECISION_VALUES, 0) == binding.LOSA_OK
        assert lib.losa_set_tuning(None, binding.LOSA_TUNE_SHARED_TILES, 0) == inv
    finally:
        assert lib.losa_destroy(ctx) == binding.LOSA_OK


def test_workspace_size_is_sane():
    # C1 shape: tens of MiB (split-K partials for 1024 work items of 64 rows, the score matrix)
    cfg = binding.make_config(max_batch=1, num_q_heads=28, num_kv_heads=4, head_dim=128, hidden_size=3584,
                              page_size=16, block_size=32, max_pages_per_seq=2048, max_topk_pages=128)
    n = binding.losa_workspace_bytes(cfg)
    assert 1 << 20 < n < 64 << 20


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more must end with a message, not a silent run."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
