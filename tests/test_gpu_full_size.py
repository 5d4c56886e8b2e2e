"""GPU parity at the full sizes of the measurement configurations, in the launch configuration the
bench uses.  Where the whole problem is too large for the CPU oracle in seconds, one sampled
sequence is checked in full (every sequence is independent on this path)."""
import numpy as np
import pytest
import torch

from oracle import fc_oracle as orc
from paper_2505_21467_amd import binding as fc
from paper_2505_21467_amd import inputs
from tests.harness import GpuLayerCache, OracleLayerCache, assert_close

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def _window_rows(K, V, o, lo, hi, dtype, what):
    assert_close(K[:, :, lo:hi], o.Kc[:, :, lo:hi], dtype, what + " K window rows")
    assert_close(V[:, :, lo:hi], o.Vc[:, :, lo:hi], dtype, what + " V window rows")


def test_config2_dream_shaped_cached_step():
    w = inputs.C2
    L, A, S = w.cached_len, w.active, w.kv_len
    _say("config2 bf16 B1 d3584 28/4 Dh128 L1024 A32")
    g = GpuLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=A, fill=0.5)
    o = OracleLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, fill=0.5)
    K, V = inputs.kv_fill(w, 0, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, X = inputs.weights(w, 0), inputs.hidden_states(w, 0, A)
    Qg, Og = g.step(0, X, W, None, L, S)
    Qo, Oo = o.step(X, W, None, L, S)
    assert_close(Qg, Qo, w.dtype, "Q")
    assert_close(Og, Oo, w.dtype, "O")
    Kg, Vg = g.read_rows(0, 0, S)
    assert np.array_equal(Kg[:, :, :L], o.Kc[:, :, :L]) and np.array_equal(Vg[:, :, :L], o.Vc[:, :, :L])
    _window_rows(Kg, Vg, o, L, S, w.dtype, "config2")
    g.close()


def test_config2_prompt_refresh_then_cached_step():
    """The cache filled by a refresh of prompt activations (reduced prompt of 160 rows, full width)."""
    w = inputs.C2.scaled(cached_len=160)
    L, A, S = w.cached_len, w.active, w.kv_len
    _say("config2-shaped refresh of %d prompt rows (K/V only), then cached step" % L)
    g = GpuLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=L, fill=0.0)
    o = OracleLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, fill=0.0)
    W = inputs.weights(w, 0)
    Xp = inputs.hidden_states(w, 0, L, tag="x_prompt")
    g.refresh(0, Xp, W, None, 0, L, want_out=False)
    o.project_only(Xp, W, None, 0)
    Kg, Vg = g.read_rows(0, 0, S)
    _window_rows(Kg, Vg, o, 0, L, w.dtype, "prompt refresh")
    X = inputs.hidden_states(w, 0, A)
    Qg, Og = g.step(0, X, W, None, L, S)
    Qo, Oo = o.step(X, W, None, L, S)
    assert_close(Qg, Qo, w.dtype, "Q")
    assert_close(Og, Oo, w.dtype, "O")
    g.close()


def test_config3_llada_shaped_cached_step():
    w = inputs.C3
    B, L, A, S = w.batch, w.cached_len, w.active, w.kv_len
    _say("config3 bf16 B4 d4096 32/32 Dh128 L4096 A64 (direct K/V fill)")
    g = GpuLayerCache(w.dtype, B, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=A)
    o = OracleLayerCache(w.dtype, B, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S)
    K, V = inputs.kv_fill(w, 0, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, X = inputs.weights(w, 0), inputs.hidden_states(w, 0, A)
    Qg, Og = g.step(0, X, W, None, L, S)
    Qo, Oo = o.step(X, W, None, L, S)
    assert_close(Qg, Qo, w.dtype, "Q")
    assert_close(Og, Oo, w.dtype, "O")
    Kg, Vg = g.read_rows(0, L, A)
    assert_close(Kg, o.Kc[:, :, L:S], w.dtype, "K window rows")
    assert_close(Vg, o.Vc[:, :, L:S], w.dtype, "V window rows")
    g.close()


def test_config4_long_context_hundred_steps():
    """100 consecutive cached steps, window sliding by 32 every 8 steps; parity at steps 0, 7, 8, 99."""
    w = inputs.C4
    A, S, P = w.active, w.kv_len, w.cached_len
    check = (0, 7, 8, 99)
    _say("config4 bf16 28/4 Dh128 L16384 kv_len %d, 100 steps, parity at %s" % (S, check))
    g = GpuLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=A)
    o = OracleLayerCache(w.dtype, 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S)
    K, V = inputs.kv_fill(w, 0, S)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W = inputs.weights(w, 0)
    for s in range(100):
        ws, rows, _ = fc.fc_window(s, P, w.gen_len, w.block, w.steps_per_block)
        assert (ws, rows) == orc.window(s, P, w.gen_len, w.block, w.steps_per_block)[:2]
        assert ws == P + 32 * (s // 8) and rows == A
        X = inputs.hidden_states(w, 0, A, tag="x.%d" % s)
        Qg, Og = g.step(0, X, W, None, ws, S)
        if s in check:
            _say("  step %d" % s)
            Qo, Oo = o.step(X, W, None, ws, S)
            assert_close(Qg, Qo, w.dtype, "step %d Q" % s)
            assert_close(Og, Oo, w.dtype, "step %d O" % s)
        elif s % 8 == 7:
            # the last write to a finished block is what later steps attend to
            o.project_only(X, W, None, ws)
    assert ws + A == S
    Kg, Vg = g.read_rows(0, 0, S)
    assert np.array_equal(Kg[:, :, :P], o.Kc[:, :, :P]) and np.array_equal(Vg[:, :, :P], o.Vc[:, :, :P])
    _window_rows(Kg, Vg, o, P, S, w.dtype, "after 100 steps")
    g.close()


def test_config5_one_layer_of_28_cached_step_and_block_refresh():
    """Layer 27 of a 28-layer, batch-8 cache: one cached step and the periodic refresh of the
    generation region, all eight sequences against the oracle (queries, outputs and every written
    K/V row)."""
    w = inputs.C5
    B, P, G, A = w.batch, w.cached_len, w.gen_len, w.active
    S = P + G
    layer = 27
    _say("config5 bf16 B8 28 layers P2048 G256: layer %d, oracle on all %d sequences" % (layer, B))
    g = GpuLayerCache(w.dtype, B, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, n_layers=w.n_layers,
                      max_rows=G)
    o = OracleLayerCache(w.dtype, B, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S)
    K, V = inputs.kv_fill(w, 0, S)  # stands in for the initial full pass
    g.write_rows(layer, K, V, 0)
    o.write_rows(K, V, 0)
    Kf, Vf = inputs.as_oracle(K), inputs.as_oracle(V)
    W = inputs.weights(w, 0, layer=layer)
    s = 27  # block 3
    ws, rows, ra = fc.fc_window(s, P, G, w.block, w.steps_per_block, w.refresh_every)
    assert (ws, rows, ra) == (P + 96, 32, 0)
    X = inputs.hidden_states(w, 0, A, tag="x.%d" % s)
    Qg, Og = g.step(layer, X, W, None, ws, S)
    Qo, Oo = o.step(X, W, None, ws, S)
    for b in range(B):  # per sequence, so that one bad sequence cannot hide in the mean of eight
        assert_close(Qg[b], Qo[b], w.dtype, "cached Q, sequence %d" % b)
        assert_close(Og[b], Oo[b], w.dtype, "cached O, sequence %d" % b)
    Kg, Vg = g.read_rows(layer, 0, S)
    outside = np.ones(S, bool)
    outside[ws:ws + A] = False
    assert np.array_equal(Kg[:, :, outside], Kf[:, :, outside]) and np.array_equal(Vg[:, :, outside], Vf[:, :, outside])
    assert_close(Kg[:, :, ws:ws + A], o.Kc[:, :, ws:ws + A], w.dtype, "cached-step K rows")
    assert_close(Vg[:, :, ws:ws + A], o.Vc[:, :, ws:ws + A], w.dtype, "cached-step V rows")

    _say("  refresh of the generation region [2048, 2304) after step 31, all sequences")
    assert fc.fc_window(31, P, G, w.block, w.steps_per_block, w.refresh_every)[2] == 1
    Xr = inputs.hidden_states(w, 0, G, tag="x.refresh")
    Qg, Og = g.refresh(layer, Xr, W, None, P, S)
    Qo, Oo = o.step(Xr, W, None, P, S)
    for b in range(B):
        assert_close(Qg[b], Qo[b], w.dtype, "refresh Q, sequence %d" % b)
        assert_close(Og[b], Oo[b], w.dtype, "refresh O, sequence %d" % b)
    Kg, Vg = g.read_rows(layer, 0, S)
    assert np.array_equal(Kg[:, :, :P], Kf[:, :, :P]) and np.array_equal(Vg[:, :, :P], Vf[:, :, :P])
    for b in range(B):
        assert_close(Kg[b, :, P:], o.Kc[b, :, P:], w.dtype, "refresh K rows, sequence %d" % b)
        assert_close(Vg[b, :, P:], o.Vc[b, :, P:], w.dtype, "refresh V rows, sequence %d" % b)
    K0, V0 = g.read_rows(0, 0, 64)  # other layers untouched
    assert np.all(K0 == 0) and np.all(V0 == 0)
    g.close()


def _dev(t):
    return t.to("cuda:0").contiguous()


def test_refresh_width_linear_layers_sampled_rows():
    """The linear layers of the whole-layer refresh (2048 rows at the 7B widths) in the launch
    configuration the bench uses; the oracle checks sampled rows (the layers are row-wise)."""
    M, d, F = 2048, 3584, 18944
    rows = [0, 1, 255, 256, 1023, 1500, 2047]
    _say("refresh-width linear layers bf16 M2048 d3584 d_ff18944")
    x = inputs.normal(51, "x", (M, d), 1.0, "bf16")
    wg = inputs.normal(51, "wg", (F, d), 0.02, "bf16")
    wu = inputs.normal(51, "wu", (F, d), 0.02, "bf16")
    need = max(fc.fc_linear_workspace_bytes("bf16", M, d, 2 * F), fc.fc_linear_workspace_bytes("bf16", M, F, d))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda:0")
    act = torch.full((M, F), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    xd = _dev(x)
    fc.fc_ffn_gate_up("bf16", xd, _dev(wg), _dev(wu), M, d, F, act, ws, need)
    torch.cuda.synchronize()
    got = inputs.as_oracle(act)
    assert np.all(np.isfinite(got))
    ref = orc.ffn_gate_up(inputs.as_oracle(x)[rows], inputs.as_oracle(wg), inputs.as_oracle(wu), "bf16")
    assert_close(got[rows], ref, "bf16", "gated W_1, 2048 rows")
    del wg, wu
    wd = inputs.normal(51, "wd", (d, F), 0.02, "bf16")
    y = torch.full((M, d), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    fc.fc_linear_residual("bf16", act, _dev(wd), xd, M, F, d, y, ws, need)
    torch.cuda.synchronize()
    goty = inputs.as_oracle(y)
    assert np.all(np.isfinite(goty))
    refy = orc.linear_residual(got[rows], inputs.as_oracle(wd), inputs.as_oracle(x)[rows], "bf16")
    assert_close(goty[rows], refy, "bf16", "W_2 + residual, 2048 rows")


def test_vocabulary_projection_at_full_vocabulary():
    """fc_lm_head_argmax at the Dream-7B sizes (32 rows, hidden 3584, vocabulary 152064), as the bench
    runs it; the oracle computes three of the rows against the whole vocabulary."""
    M, K, V = 32, 3584, 152064
    rows = [0, 13, 31]
    _say("vocabulary projection bf16 M32 K3584 V152064")
    x = inputs.normal(52, "h", (M, K), 1.0, "bf16")
    w = inputs.normal(52, "w_vocab", (V, K), 0.02, "bf16")
    need = fc.fc_lm_head_workspace_bytes("bf16", M, K, V)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    tok = torch.full((M,), -1, dtype=torch.int32, device="cuda:0")
    conf = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda:0")
    fc.fc_lm_head_argmax("bf16", _dev(x), _dev(w), M, K, V, tok, conf, ws, need)
    torch.cuda.synchronize()
    tok, conf = tok.cpu().numpy(), conf.cpu().numpy()
    assert np.all((tok >= 0) & (tok < V)) and np.all(np.isfinite(conf)) and np.all(conf > 0) and np.all(conf <= 1)
    rt, rc, z = orc.lm_head_argmax(inputs.as_oracle(x)[rows], inputs.as_oracle(w), want_logits=True)
    top = z.max(axis=1)
    second = np.partition(z, -2, axis=1)[:, -2]
    clear = top - second > 2e-4
    assert np.array_equal(tok[rows][clear], rt[clear])
    assert np.all(top - z[np.arange(len(rows)), tok[rows]] <= 2e-4)
    assert np.allclose(conf[rows], rc, rtol=2e-3)
