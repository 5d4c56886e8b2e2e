"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bit-exact for which cache rows are written and for everything outside the window; float
outputs within the tolerances in tests/harness.py."""
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


def _pair(dtype, B, d, Hq, Hkv, Dh, Smax, max_rows, fill=None, n_layers=1, base=10000.0, scale=0.0):
    g = GpuLayerCache(dtype, B, d, Hq, Hkv, Dh, Smax, n_layers=n_layers, max_rows=max_rows,
                      rope_base=base, scale=scale, fill=fill)
    o = OracleLayerCache(dtype, B, d, Hq, Hkv, Dh, Smax, rope_base=base, scale=scale,
                         fill=0.0 if fill is None else fill)
    return g, o


def _compare_cache(g, o, dtype, layer=0, written=None, what="", before=None):
    """Rows in `written` (bool [B,Smax]) match the oracle within tolerance; all other rows are
    bit-identical to `before` (the GPU cache read back before the step) or, when the rows outside
    were placed by bit copies of the same inputs on both sides, to the oracle's cache."""
    K, V = g.read_rows(layer, 0, g.max_seq)
    if written is None:
        assert_close(K, o.Kc, dtype, what + " K cache")
        assert_close(V, o.Vc, dtype, what + " V cache")
        return
    w = np.broadcast_to(written[:, None, :, None], K.shape)
    Kref, Vref = before if before is not None else (o.Kc, o.Vc)
    assert np.array_equal(K[~w].view(np.uint32), Kref[~w].view(np.uint32)), what + ": K row outside window changed"
    assert np.array_equal(V[~w].view(np.uint32), Vref[~w].view(np.uint32)), what + ": V row outside window changed"
    assert_close(K[w], o.Kc[w], dtype, what + " K window rows")
    assert_close(V[w], o.Vc[w], dtype, what + " V window rows")


# ------------------------------------------------------------------------------------------------

def test_row_copies_are_bit_exact_and_layout_private():
    _say("row copy round trip bf16 B2 Hkv3 Dh128 Smax200")
    w = inputs.C2.scaled(batch=2, n_kv_heads=3, n_q_heads=6)
    g = GpuLayerCache("bf16", 2, 256, 6, 3, 128, 200, n_layers=2, fill=-7.25)
    K, V = inputs.kv_fill(w, 5, 77)
    g.write_rows(1, K, V, 60)
    Kr, Vr = g.read_rows(1, 0, 200)
    assert np.array_equal(Kr[:, :, 60:137], inputs.as_oracle(K)) and np.array_equal(Vr[:, :, 60:137], inputs.as_oracle(V))
    assert np.all(Kr[:, :, :60] == -7.25) and np.all(Vr[:, :, 137:] == -7.25)
    K0, V0 = g.read_rows(0, 0, 200)  # the other layer is untouched
    assert np.all(K0 == -7.25) and np.all(V0 == -7.25)
    g.close()


def test_config1_tiny_fp32_refresh_vs_cached():
    """Configuration 1: fp32, hidden 256, 4/4 heads, Dh 64, L=256, A=32, seed 0."""
    w = inputs.C1
    L, A, S = w.cached_len, w.active, w.kv_len
    _say("config1 fp32 full refresh of %d rows" % S)
    W = inputs.weights(w, 0)
    X = inputs.hidden_states(w, 0, S)
    g, o = _pair("f32", 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=S)
    Qg, Og = g.refresh(0, X, W, None, 0, S)
    Qo, Oo = o.step(X, W, None, 0, S)
    assert_close(Qg, Qo, "f32", "refresh Q")
    assert_close(Og, Oo, "f32", "refresh O")
    _compare_cache(g, o, "f32", what="refresh")
    g.close()

    _say("config1 fp32 refresh rows [0,256) then cached step on [256,288)")
    g, o2 = _pair("f32", 1, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=L, fill=3.0)
    g.refresh(0, X[:, :L], W, None, 0, L, want_out=False)
    o2.project_only(X[:, :L], W, None, 0)
    Qc, Oc = g.step(0, X[:, L:], W, None, L, S)
    Qo2, Oo2 = o2.step(X[:, L:], W, None, L, S)
    assert_close(Qc, Qo2, "f32", "cached Q")
    assert_close(Oc, Oo2, "f32", "cached O")
    assert_close(Oc, Oo[:, L:], "f32", "cached O vs window rows of the full recompute")
    _compare_cache(g, o2, "f32", what="cached")

    _say("config1 fp32 perturbed window: rows < 256 stay bit-identical")
    k_before, v_before = g.snapshot()
    Kb, Vb = g.read_rows(0, 0, S)
    X2 = inputs.hidden_states(w, 1, A, tag="x2")
    g.step(0, X2, W, None, L, S)
    o2.step(X2, W, None, L, S)
    Ka, Va = g.read_rows(0, 0, S)
    assert np.array_equal(Ka[:, :, :L].view(np.uint32), Kb[:, :, :L].view(np.uint32))
    assert np.array_equal(Va[:, :, :L].view(np.uint32), Vb[:, :, :L].view(np.uint32))
    assert not np.array_equal(Ka[:, :, L:], Kb[:, :, L:])
    written = np.zeros((1, S), bool)
    written[:, L:] = True
    _compare_cache(g, o2, "f32", written=written, what="perturbed", before=(Kb, Vb))
    # raw storage: exactly 2 * B * A * Hkv * Dh elements differ at most
    k_after, v_after = g.snapshot()
    assert int((k_after != k_before).sum()) <= A * w.n_kv_heads * w.head_dim
    assert int((v_after != v_before).sum()) <= A * w.n_kv_heads * w.head_dim
    g.close()


@pytest.mark.parametrize("dtype,B,d,Hq,Hkv,Dh,L,A", [
    ("bf16", 2, 256, 8, 2, 128, 333, 32),    # GQA g=4, ragged key tail
    ("bf16", 1, 512, 28, 4, 128, 1000, 32),  # g=7 like Dream
    ("bf16", 3, 256, 4, 4, 128, 130, 64),    # MHA like LLaDA, A=64
    ("bf16", 2, 128, 6, 3, 64, 97, 20),      # Dh 64, A not a multiple of 16
    ("f32", 2, 64, 6, 2, 128, 150, 17),      # fp32 with Dh 128, odd A
    ("bf16", 1, 256, 14, 2, 128, 64, 1),     # a single active row
    ("bf16", 1, 256, 8, 1, 128, 200, 40),    # 10 row tiles per kv head: two row groups of 8 tiles
    ("bf16", 2, 256, 16, 2, 128, 1500, 48),  # 12 row tiles, several key splits, ragged last stage
])
def test_cached_step_matches_oracle(dtype, B, d, Hq, Hkv, Dh, L, A):
    _say("cached step %s B%d d%d Hq%d Hkv%d Dh%d L%d A%d" % (dtype, B, d, Hq, Hkv, Dh, L, A))
    w = inputs.Workload("t", dtype, B, d, Hq, Hkv, Dh, L, A)
    S = L + A
    g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 9, max_rows=max(A, 64), fill=1.5)
    K, V = inputs.kv_fill(w, 7, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, b = inputs.weights(w, 7), inputs.bias(w, 7)
    X = inputs.hidden_states(w, 7, A)
    Qg, Og = g.step(0, X, W, b, L, S)
    Qo, Oo = o.step(X, W, b, L, S)
    assert_close(Qg, Qo, dtype, "Q")
    assert_close(Og, Oo, dtype, "O")
    written = np.zeros((B, S + 9), bool)
    written[:, L:S] = True
    _compare_cache(g, o, dtype, written=written, what="step")
    g.close()


def test_cached_step_seeded_shape_sweep():
    """20 seeded shapes of the bf16 / head_dim 128 path: 1..3 sequences, 1..4 KV heads, 1..7 query heads
    per KV head, windows of 1..80 rows, 1..2500 cached rows, hidden 128..512.  Between them they take
    every branch of the attention planner (eight- and four-wave workgroups, one or several row groups,
    one or many key splits, ragged last stage) and both projection paths (up to 32 rows, more)."""
    rng = np.random.default_rng(20250529)
    for case in range(20):
        B = int(rng.integers(1, 4))
        Hkv = int(rng.choice([1, 2, 4]))
        Hq = Hkv * int(rng.choice([1, 2, 4, 7]))
        A = int(rng.integers(1, 81))
        L = int(rng.integers(1, 2501))
        d = int(rng.choice([128, 256, 512]))
        dtype, Dh = "bf16", 128
        _say("sweep case %d: B%d d%d Hq%d Hkv%d L%d A%d" % (case, B, d, Hq, Hkv, L, A))
        w = inputs.Workload("sweep", dtype, B, d, Hq, Hkv, Dh, L, A)
        S = L + A
        g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 5, max_rows=max(A, 64), fill=1.5)
        K, V = inputs.kv_fill(w, 100 + case, L)
        g.write_rows(0, K, V, 0)
        o.write_rows(K, V, 0)
        W, b = inputs.weights(w, 100 + case), (inputs.bias(w, 100 + case) if case % 2 else None)
        X = inputs.hidden_states(w, 100 + case, A)
        Qg, Og = g.step(0, X, W, b, L, S)
        Qo, Oo = o.step(X, W, b, L, S)
        what = "sweep case %d (B%d d%d Hq%d Hkv%d L%d A%d)" % (case, B, d, Hq, Hkv, L, A)
        assert_close(Qg, Qo, dtype, what + " Q")
        assert_close(Og, Oo, dtype, what + " O")
        written = np.zeros((B, S + 5), bool)
        written[:, L:S] = True
        _compare_cache(g, o, dtype, written=written, what=what)
        g.close()


def test_refresh_seeded_shape_sweep():
    """10 seeded refreshes of a region in the middle of a filled cache (section 3.2.1: re-projection of a
    region): 33..500 rows from a random start, keys before and behind the region, one call."""
    rng = np.random.default_rng(20250530)
    for case in range(10):
        B = int(rng.integers(1, 3))
        Hkv = int(rng.choice([1, 2, 4]))
        Hq = Hkv * int(rng.choice([1, 2, 7]))
        R = int(rng.integers(33, 501))
        start = int(rng.integers(0, 300))
        tail = int(rng.integers(0, 200))
        d = int(rng.choice([256, 512, 768]))
        dtype, Dh = "bf16", 128
        S = start + R + tail
        _say("refresh sweep case %d: B%d d%d Hq%d Hkv%d start%d R%d kv_len%d" % (case, B, d, Hq, Hkv, start, R, S))
        w = inputs.Workload("rsweep", dtype, B, d, Hq, Hkv, Dh, S, R)
        g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 3, max_rows=R, fill=0.5)
        K, V = inputs.kv_fill(w, 200 + case, S)
        g.write_rows(0, K, V, 0)
        o.write_rows(K, V, 0)
        W, b = inputs.weights(w, 200 + case), (inputs.bias(w, 200 + case) if case % 2 else None)
        X = inputs.hidden_states(w, 200 + case, R)
        Qg, Og = g.refresh(0, X, W, b, start, S)
        Qo, Oo = o.step(X, W, b, start, S)
        what = "refresh sweep case %d (B%d d%d Hq%d Hkv%d start%d R%d kv_len%d)" % (case, B, d, Hq, Hkv, start, R, S)
        assert_close(Qg, Qo, dtype, what + " Q")
        assert_close(Og, Oo, dtype, what + " O")
        written = np.zeros((B, S + 3), bool)
        written[:, start:start + R] = True
        _compare_cache(g, o, dtype, written=written, what=what)
        g.close()


@pytest.mark.parametrize("B,d,Hq,Hkv,L,A", [
    (1, 1024, 4, 1, 50, 33),    # 33 window rows: one ragged row tile
    (3, 768, 6, 3, 90, 37),     # 111 rows
    (5, 512, 8, 2, 64, 51),     # 255 rows: one padding row
    (2, 1280, 2, 1, 40, 128),   # 256 rows exactly
])
def test_mid_window_projection(B, d, Hq, Hkv, L, A):
    """Windows of 33..256 rows with hidden sizes that are multiples of 256, default tile choice (every
    row and head checked)."""
    _say("mid-window projection B%d d%d Hq%d Hkv%d L%d A%d" % (B, d, Hq, Hkv, L, A))
    dtype, Dh = "bf16", 128
    w = inputs.Workload("t", dtype, B, d, Hq, Hkv, Dh, L, A)
    S = L + A
    g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 5, max_rows=A, fill=0.25)
    K, V = inputs.kv_fill(w, 13, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, b = inputs.weights(w, 13), inputs.bias(w, 13)
    X = inputs.hidden_states(w, 13, A)
    Qg, Og = g.step(0, X, W, b, L, S)
    Qo, Oo = o.step(X, W, b, L, S)
    assert_close(Qg, Qo, dtype, "Q")
    assert_close(Og, Oo, dtype, "O")
    written = np.zeros((B, S + 5), bool)
    written[:, L:S] = True
    _compare_cache(g, o, dtype, written=written, what="mid-window step")
    g.close()


@pytest.mark.parametrize("shape", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("B,d,Hq,Hkv,L,A", [
    (3, 192, 8, 2, 100, 23),   # 69 window rows: one ragged row tile, three hidden stages
    (2, 320, 4, 4, 70, 160),   # 320 window rows: several row tiles, the last one ragged
    (2, 64, 3, 1, 50, 40),     # an odd number of head slots (5), a single hidden stage
])
def test_wide_window_projection_tile_shapes(knob, shape, B, d, Hq, Hkv, L, A):
    """The tiled projection (more than 32 window rows) in each of its six tile shapes."""
    _say("wide-window projection, tile shape %d, B%d d%d Hq%d Hkv%d L%d A%d" % (shape, B, d, Hq, Hkv, L, A))
    knob("FC_PROJ_GEMM_SHAPE", str(shape))
    dtype, Dh = "bf16", 128
    w = inputs.Workload("t", dtype, B, d, Hq, Hkv, Dh, L, A)
    S = L + A
    g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 5, max_rows=A, fill=-0.75)
    K, V = inputs.kv_fill(w, 11, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, b = inputs.weights(w, 11), inputs.bias(w, 11)
    X = inputs.hidden_states(w, 11, A)
    Qg, Og = g.step(0, X, W, b, L, S)
    Qo, Oo = o.step(X, W, b, L, S)
    assert_close(Qg, Qo, dtype, "Q")
    assert_close(Og, Oo, dtype, "O")
    written = np.zeros((B, S + 5), bool)
    written[:, L:S] = True
    _compare_cache(g, o, dtype, written=written, what="wide step")
    g.close()


@pytest.mark.parametrize("B,d,Hq,Hkv,L,A", [
    (1, 512, 28, 4, 300, 32),    # 36 head slots (the 7B head geometry)
    (2, 512, 3, 1, 77, 10),      # 5 head slots, 20 window rows (two 16-row tiles, the second ragged)
    (1, 4096, 2, 2, 40, 7),      # hidden 4096, one 16-row tile
    (3, 3584, 4, 2, 50, 9),      # hidden 3584, 27 rows
])
def test_short_window_projection_bias_and_scattered_positions(B, d, Hq, Hkv, L, A):
    """Windows of at most 32 rows at hidden sizes 512 / 3584 / 4096, with bias and with scattered, padded
    and out-of-range positions: q, every written K / V row and the freeze rule."""
    _say("short-window projection B%d d%d Hq%d Hkv%d L%d A%d" % (B, d, Hq, Hkv, L, A))
    dtype, Dh = "bf16", 128
    w = inputs.Workload("t", dtype, B, d, Hq, Hkv, Dh, L, A)
    S = L + A
    g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S + 7, max_rows=32, fill=0.75)
    K, V = inputs.kv_fill(w, 19, L)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    W, b = inputs.weights(w, 19), inputs.bias(w, 19)
    X = inputs.hidden_states(w, 19, A)
    # contiguous window
    Qg, Og = g.step(0, X, W, b, L, S)
    Qo, Oo = o.step(X, W, b, L, S)
    assert_close(Qg, Qo, dtype, "Q")
    assert_close(Og, Oo, dtype, "O")
    written = np.zeros((B, S + 7), bool)
    written[:, L:S] = True
    _compare_cache(g, o, dtype, written=written, what="short-window step")
    # scattered positions, one padded row and one position beyond the cache per sequence
    gen = torch.Generator().manual_seed(5)
    pos = torch.stack([torch.randperm(S + 7, generator=gen)[:A] for _ in range(B)]).to(torch.int32)
    pos[:, 0] = -1
    pos_o = pos.clone()
    if A > 2:
        pos[:, 2] = S + 100
        pos_o[:, 2] = -1
    Qg, Og = g.step(0, X, W, b, 0, S + 7, pos=pos)
    Qo, Oo = o.step(X, W, b, 0, S + 7, pos=pos_o)
    assert_close(Qg, Qo, dtype, "Q scattered")
    assert_close(Og, Oo, dtype, "O scattered")
    for bb in range(B):
        for a in range(A):
            if 0 <= int(pos_o[bb, a]) < S + 7:
                written[bb, int(pos_o[bb, a])] = True
    _compare_cache(g, o, dtype, written=written, what="short-window scattered step")
    g.close()


def test_scattered_positions_padding_and_bit_exact_scatter():
    """Arbitrary pos lists, padded rows, and the scatter as a pure bit copy (identity weights)."""
    dtype, B, Dh, Smax, A = "bf16", 2, 128, 210, 24
    _say("identity-weight scatter bf16 B2 Dh128 A24 with scattered and padded positions")
    g, o = _pair(dtype, B, Dh, 1, 1, Dh, Smax, max_rows=64, fill=-2.0)
    w = inputs.Workload("t", dtype, B, Dh, 1, 1, Dh, 0, A)
    eye = torch.eye(Dh, dtype=torch.float32)
    W = torch.cat([eye, eye, eye], 0).to(torch.bfloat16)
    X = inputs.hidden_states(w, 3, A)
    pos = torch.stack([torch.randperm(Smax, generator=torch.Generator().manual_seed(s))[:A] for s in (1, 2)]).to(torch.int32)
    pos[0, 5] = -1
    pos[1, 0] = -1
    pos[1, 7] = 0  # position 0: the rotation is the identity, so K is an exact copy too
    pos[0, 3] = Smax + 5  # beyond the cache: treated as padded by the kernel, never written
    K0, V0 = inputs.kv_fill(w.scaled(n_kv_heads=1), 4, Smax)
    g.write_rows(0, K0, V0, 0)
    o.write_rows(K0, V0, 0)
    Qg, Og = g.step(0, X, W, None, 0, Smax, pos=pos)
    pos_o = pos.clone()
    pos_o[0, 3] = -1
    Qo, Oo = o.step(X, W, None, 0, Smax, pos=pos_o)
    assert_close(Qg, Qo, dtype, "Q")
    assert_close(Og, Oo, dtype, "O")
    assert np.all(Og[0, 5] == 0) and np.all(Og[1, 0] == 0) and np.all(Qg[0, :, 5] == 0)
    K, V = g.read_rows(0, 0, Smax)
    Xf = inputs.as_oracle(X)
    written = np.zeros((B, Smax), bool)
    for b in range(B):
        for a in range(A):
            p = int(pos_o[b, a])
            if p < 0:
                continue
            written[b, p] = True
            assert np.array_equal(V[b, 0, p], Xf[b, a]), "V row is not a bit copy of its input"
            if p == 0:
                assert np.array_equal(K[b, 0, p], Xf[b, a])
    _compare_cache(g, o, dtype, written=written, what="scatter")
    assert written.sum() == 2 * A - 3
    g.close()


@pytest.mark.parametrize("Hq,A", [(4, 8), (8, 24)])   # one row tile; three row tiles (four-wave workgroups)
def test_degenerate_attention_cases(Hq, A):
    dtype, B, Hkv, Dh = "bf16", 1, 2, 128
    w = inputs.Workload("t", dtype, B, 256, Hq, Hkv, Dh, 0, A)
    _say("kv_len = 1 returns the single value row")
    g, o = _pair(dtype, B, 256, Hq, Hkv, Dh, 70, max_rows=64)
    K, V = inputs.kv_fill(w, 9, 70)
    g.write_rows(0, K, V, 0)
    Q = inputs.normal(9, "q", (B, Hq, A, Dh), 1.0, dtype)
    O = inputs.as_oracle(g.attend(0, g.dev_t(Q), 1)).reshape(B, A, Hq, Dh)
    Vf = inputs.as_oracle(V)
    for h in range(Hq):
        assert np.array_equal(O[0, :, h], np.broadcast_to(Vf[0, h // (Hq // Hkv), 0], (A, Dh)))
    _say("zero queries give the mean of the values")
    O = inputs.as_oracle(g.attend(0, g.dev_t(torch.zeros_like(Q)), 70)).reshape(B, A, Hq, Dh)
    for h in range(Hq):
        assert np.max(np.abs(O[0, 0, h] - Vf[0, h // (Hq // Hkv)].astype(np.float64).mean(0))) < 4e-3
    _say("oracle agreement at kv_len 65 (one key past a 64-row tile) and 70")
    o.write_rows(K, V, 0)
    for S in (65, 70):
        Og = inputs.as_oracle(g.attend(0, g.dev_t(Q), S))
        Oo = orc.attend(o.cfg, inputs.as_oracle(Q), o.Kc, o.Vc, S)
        assert_close(Og, Oo, dtype, "O at kv_len %d" % S)
    g.close()


@pytest.mark.parametrize("Hq,A", [(6, 8), (12, 24)])   # one row tile (eight-wave workgroups); three (four-wave ones)
def test_split_partials_keep_extreme_value_scales(Hq, A):
    """Several key splits with value rows of very large, very small and zero magnitude: the partial
    results exchanged between the splits carry their own scale, so each head keeps its relative
    accuracy."""
    dtype, B, Hkv, Dh, S = "bf16", 1, 3, 128, 1500
    _say("split-KV partials with values scaled by 2^100, 2^-100 and 0")
    w = inputs.Workload("t", dtype, B, 256, Hq, Hkv, Dh, 0, A)
    g, o = _pair(dtype, B, 256, Hq, Hkv, Dh, S, max_rows=64)
    K, V = inputs.kv_fill(w, 13, S)
    V = V.clone()
    V[:, 0] = (V[:, 0].float() * 2.0 ** 100).to(V.dtype)
    V[:, 1] = (V[:, 1].float() * 2.0 ** -100).to(V.dtype)
    V[:, 2] = 0
    V[:, 2, 700] = 3.0  # one nonzero row in an otherwise zero head: most splits see only zeros
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    Q = inputs.normal(13, "q", (B, Hq, A, Dh), 1.0, dtype)
    Og = inputs.as_oracle(g.attend(0, g.dev_t(Q), S)).reshape(B, A, Hq, Dh).astype(np.float64)
    Oo = orc.attend(o.cfg, inputs.as_oracle(Q), o.Kc, o.Vc, S).reshape(B, A, Hq, Dh).astype(np.float64)
    assert np.all(np.isfinite(Og))
    for h in range(Hq):
        ref, got = Oo[0, :, h], Og[0, :, h]
        scale = np.abs(ref).mean()
        assert scale > 0
        err = np.abs(got - ref)
        # same bars as the bf16 tolerance, relative to the magnitude of this head's outputs
        assert err.mean() / scale < 5e-3, "head %d: mean-rel %g" % (h, err.mean() / scale)
        assert err.max() / np.abs(ref).max() < 2e-2, "head %d: max-rel %g" % (h, err.max() / np.abs(ref).max())
    g.close()


@pytest.mark.parametrize("S", [1500, 6000, 12000, 32000])
def test_merge_of_many_key_splits(S):
    """One KV head, one row tile, long cache: the planner cuts the keys into 12, 47, 94 and 250 splits,
    one for each launch variant of the merge kernel (2, 4 waves; 8, 16, 32 splits per wave and batch;
    two batches per wave at 250)."""
    dtype, B, Hq, Hkv, Dh, A = "bf16", 1, 2, 1, 128, 8
    _say("attention over %d keys, one KV head: many key splits" % S)
    w = inputs.Workload("t", dtype, B, 256, Hq, Hkv, Dh, 0, A)
    g, o = _pair(dtype, B, 256, Hq, Hkv, Dh, S, max_rows=64)
    K, V = inputs.kv_fill(w, 17, S)
    g.write_rows(0, K, V, 0)
    o.write_rows(K, V, 0)
    Q = inputs.normal(17, "q", (B, Hq, A, Dh), 1.0, dtype)
    Og = inputs.as_oracle(g.attend(0, g.dev_t(Q), S))
    Oo = orc.attend(o.cfg, inputs.as_oracle(Q), o.Kc, o.Vc, S)
    assert_close(Og, Oo, dtype, "O over %d keys" % S)
    g.close()


def test_multi_layer_caches_are_independent():
    dtype, B, d, Hq, Hkv, Dh, L, A = "bf16", 1, 256, 8, 2, 128, 96, 32
    _say("3 layers, step on layer 1 only")
    w = inputs.Workload("t", dtype, B, d, Hq, Hkv, Dh, L, A)
    g = GpuLayerCache(dtype, B, d, Hq, Hkv, Dh, L + A, n_layers=3, max_rows=64, fill=0.5)
    o = OracleLayerCache(dtype, B, d, Hq, Hkv, Dh, L + A, fill=0.5)
    K, V = inputs.kv_fill(w, 2, L)
    g.write_rows(1, K, V, 0)
    o.write_rows(K, V, 0)
    W, X = inputs.weights(w, 2, layer=1), inputs.hidden_states(w, 2, A)
    Qg, Og = g.step(1, X, W, None, L, L + A)
    Qo, Oo = o.step(X, W, None, L, L + A)
    assert_close(Og, Oo, dtype, "O")
    for layer in (0, 2):
        Kl, Vl = g.read_rows(layer, 0, L + A)
        assert np.all(Kl == 0.5) and np.all(Vl == 0.5)
    g.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,Dh", [("f32", 64), ("bf16", 128)])
def test_kv_drift_similarity_matches_oracle(dtype, Dh):
    """KV drift diagnostic: snapshot the window rows, re-project them from changed inputs, compare the
    similarity of the cache's new rows to the snapshot with the oracle's on the same bits; rows
    re-projected from unchanged inputs have similarity 1."""
    import torch
    from paper_2505_21467_amd import binding as fcb
    B, d, Hq, Hkv, S, A, start = 2, 256, 4, 2, 200, 40, 100
    w = inputs.Workload("drift", dtype, B, d, Hq, Hkv, Dh, S, A)
    g = GpuLayerCache(dtype, B, d, Hq, Hkv, Dh, S, max_rows=A)
    W = inputs.weights(w, 3)
    X0 = inputs.hidden_states(w, 3, S)
    g.refresh(0, X0, W, None, 0, S, want_out=False)
    tdt = inputs.TORCH_DTYPE[dtype]
    kp = torch.empty((B, Hkv, A, Dh), dtype=tdt, device=g.dev)
    vp = torch.empty_like(kp)
    fcb.fc_cache_read_rows(g.handle, 0, kp, vp, start, A)
    sk = torch.full((B, Hkv, A), float("nan"), dtype=torch.float32, device=g.dev)
    sv = torch.full_like(sk, float("nan"))

    def similarity():
        fcb.fc_kv_similarity(g.handle, 0, kp, vp, start, A, sk, sv)
        torch.cuda.synchronize()
        Kg, Vg = g.read_rows(0, 0, S)
        ocfg = orc.OracleConfig(B, d, Hq, Hkv, Dh, S, dtype)
        rk, rv = orc.kv_similarity(ocfg, Kg, Vg, inputs.as_oracle(kp), inputs.as_oracle(vp), start)
        assert np.allclose(sk.cpu().numpy(), rk, atol=2e-6) and np.allclose(sv.cpu().numpy(), rv, atol=2e-6)
        return sk.cpu().numpy(), sv.cpu().numpy()

    # unchanged inputs: the re-projection reproduces the rows bit for bit -> similarity 1
    g.project(0, X0[:, start:start + A].contiguous(), W, None, start)
    k1, v1 = similarity()
    assert np.allclose(k1, 1.0, atol=2e-6) and np.allclose(v1, 1.0, atol=2e-6)
    # half of the window rows get new inputs: those drift, the others stay at 1
    X1 = X0[:, start:start + A].clone()
    X1[:, ::2] = inputs.hidden_states(w, 4, A, tag="x.new")[:, ::2]
    g.project(0, X1.contiguous(), W, None, start)
    k2, v2 = similarity()
    assert np.all(k2[:, :, ::2] < 0.9) and np.all(v2[:, :, ::2] < 0.9)
    assert np.allclose(k2[:, :, 1::2], 1.0, atol=2e-6) and np.allclose(v2[:, :, 1::2], 1.0, atol=2e-6)
    g.close()


@pytest.mark.gpu
def test_wide_window_projection_cut_into_two_launches():
    """36 head slots x 8 row tiles of 256 rows are 288 workgroups of the 256-row shape: the projection
    runs as 7 row tiles of that shape plus the last 256 rows with a smaller tile.  Every row checked."""
    _say("wide-window projection in two launches, B8 A256 d192 28/4")
    dtype, B, d, Hq, Hkv, Dh, L, A = "bf16", 8, 192, 28, 4, 128, 40, 256
    w = inputs.Workload("t2", dtype, B, d, Hq, Hkv, Dh, L, A)
    S = L + A
    g, o = _pair(dtype, B, d, Hq, Hkv, Dh, S, max_rows=A, fill=0.5)
    W, b = inputs.weights(w, 12), inputs.bias(w, 12)
    X = inputs.hidden_states(w, 12, A)
    Qg = inputs.as_oracle(g.project(0, X, W, b, L))
    Qo = o.project_only(X, W, b, L)
    assert_close(Qg, Qo, dtype, "Q")
    written = np.zeros((B, S), bool)
    written[:, L:S] = True
    _compare_cache(g, o, dtype, written=written, what="two-launch projection")
    g.close()
