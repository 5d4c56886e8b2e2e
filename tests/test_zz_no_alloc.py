"""The attention entry point that allocates nothing (static device scratch) against the ordinary
entry point with a caller-provided workspace, through the C ABI: same kernels and launch plan, so
the outputs must be bit-identical.  Two calls in a row share the one static array, the second with
a smaller input, so stale partial results of the first call lie behind the ones the second uses.
The ordinary entry point itself is checked against the oracle on one of the cases."""
import numpy as np
import pytest
import torch

from paper_2505_21467_amd import binding as fc
from paper_2505_21467_amd import inputs
from tests.harness import GpuLayerCache, OracleLayerCache, assert_close

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def _attend_both(g, Qd, A, kv_len, posd=None):
    """(workspace entry point, static entry point) outputs as raw bit patterns."""
    shape = (g.B, A, g.Hq * g.Dh)
    O_ws = torch.full(shape, float("nan"), dtype=g.tdt, device=g.dev)
    O_st = torch.full(shape, float("nan"), dtype=g.tdt, device=g.dev)
    fc.fc_active_attention(g.handle, 0, Qd, A, kv_len, posd, O_ws, g.workspace, g.ws_bytes)
    fc.fc_active_attention_static(g.handle, 0, Qd, A, kv_len, posd, O_st)
    torch.cuda.synchronize()
    return O_ws, O_st


def _bits(t):
    return t.view(torch.int16).cpu().numpy()


def test_static_scratch_attention_matches_workspace_attention_two_calls():
    dtype, B, d, Hq, Hkv, Dh = "bf16", 2, 256, 28, 4, 128
    S1, A1 = 2500, 32      # several splits, ragged last stage
    S2, A2 = 700, 20       # smaller second call: fewer splits, ragged row tile
    w = inputs.C2.scaled(batch=B, hidden=d)
    g = GpuLayerCache(dtype, B, d, Hq, Hkv, Dh, S1, max_rows=64)
    o = OracleLayerCache(dtype, B, d, Hq, Hkv, Dh, S1)
    K, V = inputs.kv_fill(w, 11, S1)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    assert fc.fc_workspace_bytes(g.cfg, 64) <= fc.fc_active_attention_static_max_bytes()

    _say("static-scratch attention, first call: B%d Hq%d/%d A%d kv_len %d" % (B, Hq, Hkv, A1, S1))
    Q1 = inputs.normal(3, "q_static_1", (B, Hq, A1, Dh), 1.0, dtype)
    Q1d = g.dev_t(Q1)
    O_ws, O_st = _attend_both(g, Q1d, A1, S1)
    assert np.array_equal(_bits(O_ws), _bits(O_st)), "first call: static and workspace outputs differ"
    from oracle import fc_oracle as orc
    Oo = orc.attend(o.cfg, inputs.as_oracle(Q1), o.Kc, o.Vc, S1, None)
    assert_close(inputs.as_oracle(O_st), Oo, dtype, "static-scratch attention vs oracle")

    _say("static-scratch attention, second call, smaller: A%d kv_len %d, padded rows" % (A2, S2))
    Q2 = inputs.normal(4, "q_static_2", (B, Hq, A2, Dh), 1.0, dtype)
    pos = inputs.window_positions(B, S2 - A2, A2).clone()
    pos[0, 3] = -1
    pos[1, A2 - 1] = -1
    Q2d, posd = g.dev_t(Q2), g.dev_t(pos)
    O_ws2, O_st2 = _attend_both(g, Q2d, A2, S2, posd)
    assert np.array_equal(_bits(O_ws2), _bits(O_st2)), "second call: static and workspace outputs differ"
    Oo2 = orc.attend(o.cfg, inputs.as_oracle(Q2), o.Kc, o.Vc, S2, inputs.as_oracle(pos))
    assert_close(inputs.as_oracle(O_st2), Oo2, dtype, "static-scratch attention (second call) vs oracle")
    assert np.all(inputs.as_oracle(O_st2)[0, 3] == 0) and np.all(inputs.as_oracle(O_st2)[1, A2 - 1] == 0)

    _say("static-scratch attention, first shape again after the smaller call")
    O_ws3, O_st3 = _attend_both(g, Q1d, A1, S1)
    assert np.array_equal(_bits(O_st3), _bits(O_st)) and np.array_equal(_bits(O_ws3), _bits(O_st3))
    g.close()


def test_static_scratch_rejects_shapes_beyond_its_size():
    _say("static-scratch attention: a shape whose partial results exceed 16 MiB is refused on the host")
    # 32/4 heads x 64 rows = 16 row tiles per KV head, 32 key ranges: 2048 (tile, range) slots of 8.5 KB
    B, Hq, Hkv, Dh, A, S = 1, 32, 4, 128, 64, 8192
    cfg = fc.make_config(1, B, 256, Hq, Hkv, Dh, S, "bf16")
    need = fc.fc_workspace_bytes(cfg, A)
    assert need > fc.fc_active_attention_static_max_bytes(), need
    k = torch.zeros(fc.fc_cache_storage_bytes(cfg) // 2, dtype=torch.bfloat16, device="cuda:0")
    v = torch.zeros_like(k)
    h = fc.fc_cache_alloc(cfg, k, v)
    q = torch.zeros((B, Hq, A, Dh), dtype=torch.bfloat16, device="cuda:0")
    out = torch.full((B, A, Hq * Dh), 3.0, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(fc.FreeCacheError) as ei:
        fc.fc_active_attention_static(h, 0, q, A, S, None, out)
    assert ei.value.status == fc.FC_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 3.0).all()), "a refused call must not touch the output"
    # the ordinary entry point takes the same shape with a workspace of that size
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    fc.fc_active_attention(h, 0, q, A, S, None, out, ws, need)
    torch.cuda.synchronize()
    assert bool((out == 0.0).all())  # zero queries over a zero cache: the mean of zero values
    fc.fc_cache_free(h)
