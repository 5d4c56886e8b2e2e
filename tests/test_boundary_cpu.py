"""Host-side tests of the C-ABI library that need no GPU: the library loads, exports every
symbol the header declares, rejects bad arguments before touching HIP, and its integer window
schedule equals the oracle's."""
import ctypes
import os
import re

import pytest

from oracle import fc_oracle as orc
from paper_2505_21467_amd import binding as fc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # 16-byte aligned non-NULL "device pointer"; never dereferenced on the host


def _cfg(**kw):
    base = dict(n_layers=2, batch=2, hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=128, max_seq=300,
                dtype="bf16")
    base.update(kw)
    return fc.make_config(**base)


@pytest.fixture()
def cache():
    h = fc.fc_cache_alloc(_cfg(), FAKE, FAKE)
    yield h
    fc.fc_cache_free(h)


def test_library_exports_every_declared_symbol():
    text = ""
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        if name.endswith(".h"):
            text += open(os.path.join(inc, name)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fc_[a-z_0-9]+)\s*\(", text))
    assert {"fc_cache_alloc", "fc_qkv_project_scatter", "fc_active_attention", "fc_refresh"} <= declared
    L = fc.lib()
    for sym in declared:
        assert hasattr(L, sym), "libfreecache.so does not export " + sym
    assert declared == set(fc.EXPORTS)


def test_storage_bytes_and_layout_padding():
    c = _cfg()
    spad = 320  # 300 rounded up to a multiple of 64
    assert fc.fc_cache_storage_bytes(c) == 2 * 2 * 2 * spad * 128 * 2
    assert fc.fc_cache_storage_bytes(_cfg(dtype="f32", max_seq=64)) == 2 * 2 * 2 * 64 * 128 * 4
    assert fc.fc_cache_storage_bytes(_cfg(head_dim=96)) == 0


def _raises(status, fn, *a, **k):
    with pytest.raises(fc.FreeCacheError) as e:
        fn(*a, **k)
    assert e.value.status == status, (e.value.status, str(e.value))
    assert fc.fc_last_error() != ""


def test_config_validation():
    for bad, st in [
        (dict(n_q_heads=7), fc.FC_ERR_UNSUPPORTED), (dict(head_dim=96), fc.FC_ERR_UNSUPPORTED),
        (dict(hidden=100), fc.FC_ERR_UNSUPPORTED), (dict(max_seq=0), fc.FC_ERR_INVALID_ARG),
        (dict(batch=0), fc.FC_ERR_INVALID_ARG), (dict(n_layers=-1), fc.FC_ERR_INVALID_ARG),
        (dict(rope_base=0.5), fc.FC_ERR_INVALID_ARG), (dict(softmax_scale=-1.0), fc.FC_ERR_INVALID_ARG),
        (dict(max_seq=(1 << 24) + 1), fc.FC_ERR_UNSUPPORTED),
    ]:
        _raises(st, fc.fc_cache_alloc, _cfg(**bad), FAKE, FAKE)
    c = _cfg()
    c.dtype = 7
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_cache_alloc, c, FAKE, FAKE)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_cache_alloc, _cfg(), FAKE, None)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_cache_alloc, _cfg(), FAKE + 4, FAKE)
    assert fc.lib().fc_cache_alloc(ctypes.byref(_cfg()), FAKE, FAKE, None) == fc.FC_ERR_INVALID_ARG
    assert fc.lib().fc_cache_alloc(None, FAKE, FAKE, ctypes.byref(ctypes.c_void_p())) == fc.FC_ERR_INVALID_ARG
    fc.fc_cache_free(None)  # accepted


def test_cache_ptrs_are_layer_offsets(cache):
    k0, v0 = fc.fc_cache_ptrs(cache, 0)
    k1, v1 = fc.fc_cache_ptrs(cache, 1)
    per_layer = fc.fc_cache_storage_bytes(_cfg()) // 2
    assert (k0, v0) == (FAKE, FAKE) and k1 - k0 == per_layer and v1 - v0 == per_layer
    _raises(fc.FC_ERR_BOUNDS, fc.fc_cache_ptrs, cache, 2)
    _raises(fc.FC_ERR_BOUNDS, fc.fc_cache_ptrs, cache, -1)


def test_compute_entry_points_reject_bad_arguments_before_any_launch(cache):
    S = 0  # stream
    P = fc.fc_qkv_project_scatter
    _raises(fc.FC_ERR_INVALID_ARG, P, None, 0, FAKE, FAKE, None, 0, 32, None, FAKE, S)
    _raises(fc.FC_ERR_BOUNDS, P, cache, 2, FAKE, FAKE, None, 0, 32, None, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, P, cache, 0, None, FAKE, None, 0, 32, None, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, P, cache, 0, FAKE, None, None, 0, 32, None, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, P, cache, 0, FAKE, FAKE, None, 0, 32, None, None, S)
    _raises(fc.FC_ERR_INVALID_ARG, P, cache, 0, FAKE, FAKE, None, 0, 0, None, FAKE, S)
    _raises(fc.FC_ERR_BOUNDS, P, cache, 0, FAKE, FAKE, None, -1, 32, None, FAKE, S)
    _raises(fc.FC_ERR_BOUNDS, P, cache, 0, FAKE, FAKE, None, 300 - 31, 32, None, FAKE, S)

    At = fc.fc_active_attention
    _raises(fc.FC_ERR_INVALID_ARG, At, None, 0, FAKE, 32, 100, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, At, cache, 5, FAKE, 32, 100, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_INVALID_ARG, At, cache, 0, None, 32, 100, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_INVALID_ARG, At, cache, 0, FAKE, 32, 100, None, None, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_INVALID_ARG, At, cache, 0, FAKE, 0, 100, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, At, cache, 0, FAKE, 32, 0, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, At, cache, 0, FAKE, 32, 301, None, FAKE, FAKE, 1 << 30, S)

    R = fc.fc_refresh
    _raises(fc.FC_ERR_INVALID_ARG, R, cache, 0, None, FAKE, None, 0, 64, 64, FAKE, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_INVALID_ARG, R, cache, 0, FAKE, FAKE, None, 0, 64, 64, None, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_INVALID_ARG, R, cache, 0, FAKE, FAKE, None, 0, 0, 64, FAKE, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, R, cache, 0, FAKE, FAKE, None, 280, 64, 300, FAKE, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, R, cache, 0, FAKE, FAKE, None, 0, 64, 63, FAKE, FAKE, FAKE, 1 << 30, S)
    _raises(fc.FC_ERR_BOUNDS, R, cache, 0, FAKE, FAKE, None, 0, 64, 301, FAKE, FAKE, FAKE, 1 << 30, S)

    for fn in (fc.fc_cache_write_rows, fc.fc_cache_read_rows):
        _raises(fc.FC_ERR_INVALID_ARG, fn, cache, 0, None, FAKE, 0, 4, S)
        _raises(fc.FC_ERR_INVALID_ARG, fn, cache, 0, FAKE, FAKE, 0, 0, S)
        _raises(fc.FC_ERR_BOUNDS, fn, cache, 0, FAKE, FAKE, 298, 4, S)
        _raises(fc.FC_ERR_BOUNDS, fn, cache, 0, FAKE, FAKE, -1, 4, S)
        _raises(fc.FC_ERR_BOUNDS, fn, cache, 3, FAKE, FAKE, 0, 4, S)


def test_workspace_is_demanded_when_the_plan_splits_keys():
    # the long-context shape must split the key range, hence need a workspace
    c = fc.make_config(1, 1, 3584, 28, 4, 128, 16800, "bf16")
    need = fc.fc_workspace_bytes(c, 32)
    assert need > 0 and need % 4 == 0
    assert fc.fc_workspace_bytes(c, 0) == 0
    h = fc.fc_cache_alloc(c, FAKE, FAKE)
    try:
        _raises(fc.FC_ERR_WORKSPACE, fc.fc_active_attention, h, 0, FAKE, 32, 16800, None, FAKE, None, 0, 0)
        # `need` covers every window of up to 32 rows; any window's own requirement is far above 4 KB
        _raises(fc.FC_ERR_WORKSPACE, fc.fc_active_attention, h, 0, FAKE, 32, 16800, None, FAKE, FAKE, 4096, 0)
        _raises(fc.FC_ERR_WORKSPACE, fc.fc_active_attention, h, 0, FAKE, 7, 16800, None, FAKE, FAKE, 4096, 0)
        _raises(fc.FC_ERR_WORKSPACE, fc.fc_refresh, h, 0, FAKE, FAKE, None, 0, 32, 16800, FAKE, FAKE, FAKE, 8, 0)
    finally:
        fc.fc_cache_free(h)


def test_tuning_knobs_change_the_attention_plan_and_are_restored():
    c = fc.make_config(1, 1, 3584, 28, 4, 128, 16800, "bf16")
    base = fc.fc_attention_plan(c, 32, 16800)
    assert base["kind"] == 1 and base["row_tiles"] == 7 and base["splits"] * base["keys_per_split"] >= 16800
    assert base["keys_per_split"] % 64 == 0 and (base["splits"] - 1) * base["keys_per_split"] < 16800
    try:
        fc.fc_tuning_set("FC_ATTN_TILES", "8,8")
        fc.fc_tuning_set("FC_ATTN_WGS", 64)
        forced = fc.fc_attention_plan(c, 32, 16800)
        assert forced["tiles_per_wg"] == 8 and forced["waves"] == 8 and forced["splits"] < base["splits"]
        _raises(fc.FC_ERR_INVALID_ARG, fc.fc_tuning_set, "FC_NO_SUCH_KNOB", 1)
    finally:
        fc.fc_tuning_set("FC_ATTN_TILES", None)
        fc.fc_tuning_set("FC_ATTN_WGS", None)
    assert fc.fc_attention_plan(c, 32, 16800) == base
    assert fc.fc_attention_plan(fc.make_config(1, 1, 256, 4, 4, 64, 288, "f32"), 32, 288)["kind"] == 0
    with pytest.raises(fc.FreeCacheError):
        fc.fc_attention_plan(c, 32, 16801)


def test_static_scratch_attention_validates_on_the_host():
    """The entry point that allocates nothing checks its arguments like fc_active_attention and
    refuses, before any HIP call, a shape whose partial results exceed its static array."""
    St = fc.fc_active_attention_static
    cap = fc.fc_active_attention_static_max_bytes()
    assert cap == 16 * 1024 * 1024
    c = fc.make_config(1, 1, 256, 32, 4, 128, 8192, "bf16")
    assert fc.fc_workspace_bytes(c, 64) > cap
    assert fc.fc_workspace_bytes(fc.make_config(1, 1, 3584, 28, 4, 128, 16800, "bf16"), 32) <= cap
    h = fc.fc_cache_alloc(c, FAKE, FAKE)
    try:
        _raises(fc.FC_ERR_WORKSPACE, St, h, 0, FAKE, 64, 8192, None, FAKE, 0)
        _raises(fc.FC_ERR_INVALID_ARG, St, None, 0, FAKE, 64, 8192, None, FAKE, 0)
        _raises(fc.FC_ERR_INVALID_ARG, St, h, 0, None, 64, 8192, None, FAKE, 0)
        _raises(fc.FC_ERR_INVALID_ARG, St, h, 0, FAKE, 64, 8192, None, None, 0)
        _raises(fc.FC_ERR_INVALID_ARG, St, h, 0, FAKE, 0, 8192, None, FAKE, 0)
        _raises(fc.FC_ERR_BOUNDS, St, h, 1, FAKE, 64, 8192, None, FAKE, 0)
        _raises(fc.FC_ERR_BOUNDS, St, h, 0, FAKE, 64, 8193, None, FAKE, 0)
    finally:
        fc.fc_cache_free(h)


@pytest.mark.parametrize("mode", [0, 1])
def test_window_schedule_equals_oracle(mode):
    cases = [(16384, 416, 32, 8, 0), (2048, 256, 32, 8, 8), (0, 70, 32, 1, 3), (5, 64, 64, 4, 2), (9, 1, 1, 1, 1)]
    for P, G, Bk, spb, every in cases:
        n_blocks = -(-G // Bk)
        for s in range(n_blocks * spb):
            assert fc.fc_window(s, P, G, Bk, spb, every, mode) == orc.window(s, P, G, Bk, spb, every, mode)
        _raises(fc.FC_ERR_BOUNDS, fc.fc_window, n_blocks * spb, P, G, Bk, spb, every, mode)
        with pytest.raises(IndexError):
            orc.window(n_blocks * spb, P, G, Bk, spb, every, mode)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_window, -1, 0, 32, 32, 1)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_window, 0, 0, 0, 32, 1)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_window, 0, 0, 32, 0, 1)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_window, 0, 0, 32, 32, 0)
    _raises(fc.FC_ERR_INVALID_ARG, fc.fc_window, 0, 0, 32, 32, 1, 0, 2)
    assert fc.lib().fc_window(0, 0, 32, 32, 1, 0, 0, None, None, None) == fc.FC_ERR_INVALID_ARG


def test_rest_of_layer_entry_points_reject_bad_arguments_before_any_launch(cache):
    S, BF = 0, "bf16"
    N = fc.fc_rmsnorm
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, None, FAKE, 1e-6, 4, 64, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, FAKE, None, 1e-6, 4, 64, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, FAKE, FAKE, 1e-6, 4, 64, None, S)
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, FAKE, FAKE, -1.0, 4, 64, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, FAKE, FAKE, 1e-6, 0, 64, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, N, BF, FAKE, FAKE, 1e-6, 4, 0, FAKE, S)
    assert fc.lib().fc_rmsnorm(9, FAKE, FAKE, 1e-6, 4, 64, FAKE, None) == fc.FC_ERR_INVALID_ARG

    Lr = fc.fc_linear_residual
    big = 1 << 30
    _raises(fc.FC_ERR_INVALID_ARG, Lr, BF, None, FAKE, None, 32, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, Lr, BF, FAKE, None, None, 32, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, Lr, BF, FAKE, FAKE, None, 32, 512, 128, None, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, Lr, BF, FAKE, FAKE, None, 0, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_UNSUPPORTED, Lr, BF, FAKE, FAKE, None, 32, 100, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, Lr, BF, FAKE + 2, FAKE, None, 32, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_WORKSPACE, Lr, BF, FAKE, FAKE, None, 32, 1024, 128, FAKE, None, 0, S)
    _raises(fc.FC_ERR_WORKSPACE, Lr, BF, FAKE, FAKE, None, 32, 1024, 128, FAKE, FAKE, 64, S)
    Gu = fc.fc_ffn_gate_up
    _raises(fc.FC_ERR_INVALID_ARG, Gu, BF, FAKE, FAKE, None, 32, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, Gu, BF, FAKE, None, FAKE, 32, 512, 128, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_WORKSPACE, Gu, BF, FAKE, FAKE, FAKE, 32, 1024, 128, FAKE, FAKE, 64, S)

    # workspace sizes: the slice-wise streaming kernels need one (partial tiles), the whole-row kernel
    # (hidden 3584 with at least one item per compute unit) and other shapes do not; the gated query is N = 2 F
    assert fc.fc_linear_workspace_bytes(BF, 32, 3584, 3584) > 0
    assert fc.fc_linear_workspace_bytes(BF, 32, 18944, 3584) > 0
    assert fc.fc_linear_workspace_bytes(BF, 32, 3584, 2 * 18944) == 0
    assert fc.fc_linear_workspace_bytes(BF, 32, 520, 3584) == 0      # K not a multiple of 512
    assert fc.fc_linear_workspace_bytes("f32", 32, 3584, 3584) == 0
    assert fc.fc_linear_workspace_bytes(BF, 0, 3584, 3584) == 0
    assert fc.fc_linear_workspace_bytes(BF, 64, 3584, 3584) >= fc.fc_linear_workspace_bytes(BF, 32, 3584, 3584)

    c = _cfg()
    need = fc.fc_full_layer_workspace_bytes(c, 512, 32)
    assert need > 0 and need % 256 == 0
    assert fc.fc_full_layer_workspace_bytes(c, 0, 32) == 0 and fc.fc_full_layer_workspace_bytes(c, 512, 0) == 0
    assert fc.fc_full_layer_workspace_bytes(c, 512, 64) > need
    wt = fc.make_layer_weights(FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 1e-6)
    Fl = fc.fc_full_layer_step
    _raises(fc.FC_ERR_INVALID_ARG, Fl, None, 0, wt, FAKE, 0, 32, None, 100, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_BOUNDS, Fl, cache, 2, wt, FAKE, 0, 32, None, 100, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_INVALID_ARG, Fl, cache, 0, wt, None, 0, 32, None, 100, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_INVALID_ARG, Fl, cache, 0, wt, FAKE, 0, 32, None, 100, None, FAKE, need, S)
    _raises(fc.FC_ERR_INVALID_ARG, Fl, cache, 0, wt, FAKE, 0, 0, None, 100, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_BOUNDS, Fl, cache, 0, wt, FAKE, 280, 32, None, 300, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_BOUNDS, Fl, cache, 0, wt, FAKE, 0, 32, None, 301, FAKE, FAKE, need, S)
    _raises(fc.FC_ERR_WORKSPACE, Fl, cache, 0, wt, FAKE, 0, 32, None, 100, FAKE, FAKE, need - 1, S)
    _raises(fc.FC_ERR_WORKSPACE, Fl, cache, 0, wt, FAKE, 0, 32, None, 100, FAKE, None, 0, S)
    for missing in ("norm1", "w_qkv", "w_out", "norm2", "w_gate", "w_up", "w_down"):
        bad = fc.make_layer_weights(FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 1e-6)
        setattr(bad, missing, None)
        _raises(fc.FC_ERR_INVALID_ARG, Fl, cache, 0, bad, FAKE, 0, 32, None, 100, FAKE, FAKE, need, S)
    bad = fc.make_layer_weights(FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 1e-6)
    _raises(fc.FC_ERR_INVALID_ARG, Fl, cache, 0, bad, FAKE, 0, 32, None, 100, FAKE, FAKE, need, S)


def test_unmasking_entry_points_reject_bad_arguments_before_any_launch():
    S, BF, big = 0, "bf16", 1 << 30
    H = fc.fc_lm_head_argmax
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, None, FAKE, 32, 512, 1024, FAKE, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, FAKE, None, 32, 512, 1024, FAKE, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, FAKE, FAKE, 32, 512, 1024, None, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, FAKE, FAKE, 32, 512, 1024, FAKE, None, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, FAKE, FAKE, 0, 512, 1024, FAKE, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_INVALID_ARG, H, BF, FAKE, FAKE, 32, 512, 0, FAKE, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_UNSUPPORTED, H, BF, FAKE, FAKE, 32, 100, 1024, FAKE, FAKE, FAKE, big, S)
    _raises(fc.FC_ERR_WORKSPACE, H, BF, FAKE, FAKE, 32, 512, 1024, FAKE, FAKE, None, 0, S)
    need = fc.fc_lm_head_workspace_bytes(BF, 32, 512, 1024)
    assert need > 0 and need % 256 == 0
    _raises(fc.FC_ERR_WORKSPACE, H, BF, FAKE, FAKE, 32, 512, 1024, FAKE, FAKE, FAKE, need - 1, S)
    assert fc.fc_lm_head_workspace_bytes(BF, 0, 512, 1024) == 0
    assert fc.fc_lm_head_workspace_bytes("f32", 4, 40, 300) > 0          # the plain kernel keeps per-part state too
    assert fc.fc_lm_head_workspace_bytes(BF, 32, 1024, 152064) > fc.fc_lm_head_workspace_bytes(BF, 32, 1024, 1024)
    # hidden 3584: the whole-row kernel keeps one (largest, index, sum) per workgroup and row, nothing else
    assert fc.fc_lm_head_workspace_bytes(BF, 32, 3584, 152064) == 3 * 256 * 32 * 4

    U = fc.fc_unmask_select
    _raises(fc.FC_ERR_INVALID_ARG, U, None, FAKE, FAKE, 0, 2, 32, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, None, FAKE, 0, 2, 32, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 32, 4, 9, None, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 32, 4, 9, FAKE, 100, None, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 32, 4, 9, FAKE, 100, FAKE + 256, None, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 0, 32, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 0, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 32, -1, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_INVALID_ARG, U, FAKE, FAKE, FAKE, 0, 2, 32, 4, 9, FAKE, 100, FAKE, FAKE, S)      # pos_next == pos
    _raises(fc.FC_ERR_UNSUPPORTED, U, FAKE, FAKE, FAKE, 0, 2, 9000, 4, 9, FAKE, 10000, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_BOUNDS, U, FAKE, FAKE, None, 80, 2, 32, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)
    _raises(fc.FC_ERR_BOUNDS, U, FAKE, FAKE, None, -1, 2, 32, 4, 9, FAKE, 100, FAKE + 256, FAKE, S)


def test_gather_rows_rejects_bad_arguments_before_any_launch():
    G = fc.fc_gather_rows
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", None, 10, 64, FAKE, 4, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", FAKE, 10, 64, None, 4, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", FAKE, 10, 64, FAKE, 4, None, 0)
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", FAKE, 0, 64, FAKE, 4, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", FAKE, 10, 64, FAKE, 0, FAKE, 0)
    _raises(fc.FC_ERR_UNSUPPORTED, G, "bf16", FAKE, 10, 12, FAKE, 4, FAKE, 0)   # 24-byte rows
    _raises(fc.FC_ERR_INVALID_ARG, G, "bf16", FAKE + 8, 10, 64, FAKE, 4, FAKE, 0)


def test_guided_accept_rejects_bad_arguments_before_any_launch():
    Gd = fc.fc_guided_accept
    ok = dict(dlm=FAKE, ar=FAKE, pos=FAKE, win_start=0, B=2, A=32, V=1000, topk=2, tau=0.5, mask_id=9, tokens=FAKE, L=100,
              n_accept=FAKE, pos_next=FAKE + 256, count_next=FAKE, workspace=FAKE, workspace_bytes=1 << 20, stream=0)
    need = fc.fc_guided_accept_workspace_bytes(2, 32, 1000)
    assert need >= 2 * 2 * 32 * 4 and fc.fc_guided_accept_workspace_bytes(0, 32, 1000) == 0
    assert fc.fc_guided_accept_workspace_bytes(1, 32, 152064) > fc.fc_guided_accept_workspace_bytes(1, 32, 1000)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return lambda: Gd(**a)
    for kw, st in [
        (dict(dlm=None), fc.FC_ERR_INVALID_ARG), (dict(ar=None), fc.FC_ERR_INVALID_ARG),
        (dict(tokens=None), fc.FC_ERR_INVALID_ARG), (dict(n_accept=None), fc.FC_ERR_INVALID_ARG),
        (dict(pos_next=None), fc.FC_ERR_INVALID_ARG), (dict(count_next=None), fc.FC_ERR_INVALID_ARG),
        (dict(B=0), fc.FC_ERR_INVALID_ARG), (dict(V=0), fc.FC_ERR_INVALID_ARG), (dict(topk=0), fc.FC_ERR_INVALID_ARG),
        (dict(topk=9), fc.FC_ERR_UNSUPPORTED), (dict(V=1, topk=2), fc.FC_ERR_INVALID_ARG),
        (dict(tau=float("nan")), fc.FC_ERR_INVALID_ARG), (dict(pos_next=FAKE), fc.FC_ERR_INVALID_ARG),
        (dict(pos=None, win_start=80), fc.FC_ERR_BOUNDS), (dict(workspace=None), fc.FC_ERR_WORKSPACE),
        (dict(workspace_bytes=need - 1), fc.FC_ERR_WORKSPACE),
    ]:
        _raises(st, call(**kw))


def test_kv_similarity_rejects_bad_arguments_before_any_launch(cache):
    Sm = fc.fc_kv_similarity
    _raises(fc.FC_ERR_INVALID_ARG, Sm, None, 0, FAKE, FAKE, 0, 4, FAKE, FAKE, 0)
    _raises(fc.FC_ERR_BOUNDS, Sm, cache, 2, FAKE, FAKE, 0, 4, FAKE, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, Sm, cache, 0, None, FAKE, 0, 4, FAKE, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, Sm, cache, 0, FAKE, FAKE, 0, 4, None, FAKE, 0)
    _raises(fc.FC_ERR_INVALID_ARG, Sm, cache, 0, FAKE, FAKE, 0, 0, FAKE, FAKE, 0)
    _raises(fc.FC_ERR_BOUNDS, Sm, cache, 0, FAKE, FAKE, 298, 4, FAKE, FAKE, 0)
    _raises(fc.FC_ERR_BOUNDS, Sm, cache, 0, FAKE, FAKE, -1, 4, FAKE, FAKE, 0)
