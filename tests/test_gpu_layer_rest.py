"""GPU parity of the rest of the layer on the window rows (RMSNorm, output projection + residual,
gated feed-forward network, and the whole cached layer step) against the CPU oracle, element by
element, through the C-ABI binding.  Tolerances as for the attention path (tests/harness.py)."""
import numpy as np
import pytest
import torch

from oracle import fc_oracle as orc
from paper_2505_21467_amd import binding as fc
from paper_2505_21467_amd import inputs
from tests.harness import GpuLayerCache, assert_chain_close as _chain_tolerance, assert_close, bf16_ulp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(t):
    return None if t is None else t.to(DEV).contiguous()


def _ws(nbytes):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("dtype,rows,hidden", [
    ("f32", 5, 200), ("bf16", 5, 200), ("bf16", 32, 3584), ("bf16", 3, 8), ("bf16", 4, 2048), ("bf16", 3, 4096),
    ("bf16", 2, 8192), ("bf16", 2, 8200), ("bf16", 3, 100),
])
def test_rmsnorm_matches_oracle(dtype, rows, hidden):
    x = inputs.normal(1, "x", (rows, hidden), 1.5, dtype)
    w = (1.0 + 0.1 * inputs.normal(1, "w", (hidden,), 1.0, "f32")).to(inputs.TORCH_DTYPE[dtype])
    ref = orc.rmsnorm(inputs.as_oracle(x), inputs.as_oracle(w), 1e-5, dtype)
    xd, wd = _dev(x), _dev(w)
    out = torch.full_like(xd, float("nan"))
    fc.fc_rmsnorm(dtype, xd, wd, 1e-5, rows, hidden, out)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, dtype, "rmsnorm")
    fc.fc_rmsnorm(dtype, xd, wd, 1e-5, rows, hidden, xd)  # in place
    torch.cuda.synchronize()
    assert torch.equal(xd, out)


LINEAR_SHAPES = [
    # dtype, M, K, N, residual
    ("f32", 9, 72, 50, True),          # plain kernel, ragged everything
    ("bf16", 5, 136, 72, True),        # bf16 shape the streaming kernels do not cover
    ("bf16", 32, 512, 128, False),     # one work item
    ("bf16", 7, 1024, 256, True),      # one 16-row tile, padded rows
    ("bf16", 32, 3584, 3584, True),    # the output projection of the 7B geometry
    ("bf16", 32, 4608, 1536, True),    # long rows: many slices per slab, runs that straddle slabs
    ("bf16", 40, 1024, 384, True),     # two passes of up to 32 rows, ragged second pass
    ("bf16", 17, 512, 408, True),      # whole-row kernel: 51 half items of 8 rows (the last item is half), ragged rows
    ("bf16", 32, 4096, 4096 + 24, False),  # whole-row kernel at hidden 4096, more items than workgroups, odd half item
    ("bf16", 3, 3584, 16 * 300, True),  # whole-row kernel, one 16-row tile of X, uneven runs (300 items over 256 workgroups)
]


@pytest.mark.parametrize("dtype,M,K,N,with_res", LINEAR_SHAPES)
def test_linear_residual_matches_oracle(dtype, M, K, N, with_res):
    x = inputs.normal(2, "x", (M, K), 1.0, dtype)
    w = inputs.normal(2, "w", (N, K), 0.05, dtype)
    r = inputs.normal(2, "r", (M, N), 1.0, dtype) if with_res else None
    ref = orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), None if r is None else inputs.as_oracle(r),
                              dtype)
    need = fc.fc_linear_workspace_bytes(dtype, M, K, N)
    ws = _ws(need)
    xd, wd, rd = _dev(x), _dev(w), _dev(r)
    out = torch.full((M, N), float("nan"), dtype=xd.dtype, device=DEV)
    fc.fc_linear_residual(dtype, xd, wd, rd, M, K, N, out, ws, need)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, dtype, "linear_residual")
    if with_res:  # out may be the residual buffer
        fc.fc_linear_residual(dtype, xd, wd, rd, M, K, N, rd, ws, need)
        torch.cuda.synchronize()
        assert torch.equal(rd, out)


@pytest.mark.parametrize("wgs", ["3", "100", "1000"])
def test_linear_residual_any_number_of_workgroups(wgs, knob):
    # the work items are dealt to however many workgroups the plan asks for; runs of every length
    knob("FC_LIN_WGS", wgs)
    M, K, N = 32, 2560, 640
    x = inputs.normal(3, "x", (M, K), 1.0, "bf16")
    w = inputs.normal(3, "w", (N, K), 0.05, "bf16")
    ref = orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), None, "bf16")
    need = fc.fc_linear_workspace_bytes("bf16", M, K, N)
    ws = _ws(need)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    fc.fc_linear_residual("bf16", _dev(x), _dev(w), None, M, K, N, out, ws, need)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, "bf16", "linear_residual wgs=" + wgs)


@pytest.mark.parametrize("dtype,M,K,F", [
    ("f32", 6, 40, 70), ("bf16", 5, 136, 72), ("bf16", 32, 1024, 320), ("bf16", 16, 512, 64),
    ("bf16", 32, 3584, 2368), ("bf16", 50, 1024, 192),
    ("bf16", 9, 512, 100),        # whole-row kernel: 25 half items of 4 features
    ("bf16", 32, 4096, 2052),     # whole-row kernel at hidden 4096, 513 half items over 256 workgroups
    ("bf16", 64, 1024, 12800),    # tiled GEMM, 200 slabs and at most 128 rows: 128-row tiles of half slabs
])
def test_ffn_gate_up_matches_oracle(dtype, M, K, F):
    x = inputs.normal(4, "x", (M, K), 1.0, dtype)
    wg = inputs.normal(4, "wg", (F, K), 0.05, dtype)
    wu = inputs.normal(4, "wu", (F, K), 0.05, dtype)
    ref = orc.ffn_gate_up(inputs.as_oracle(x), inputs.as_oracle(wg), inputs.as_oracle(wu), dtype)
    need = fc.fc_linear_workspace_bytes(dtype, M, K, 2 * F)
    ws = _ws(need)
    out = torch.full((M, F), float("nan"), dtype=inputs.TORCH_DTYPE[dtype], device=DEV)
    fc.fc_ffn_gate_up(dtype, _dev(x), _dev(wg), _dev(wu), M, K, F, out, ws, need)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, dtype, "ffn_gate_up")


def test_whole_row_kernel_seeded_shape_sweep():
    # hidden 512 (the whole-row kernel), 24 seeded shapes: 1..32 rows, 1..600 half items, with and without
    # residual, both epilogues; every output checked
    rng = np.random.default_rng(20250527)
    for case in range(24):
        M = int(rng.integers(1, 33))
        gated = case % 2 == 1
        N = int(rng.integers(1, 601)) * (4 if gated else 8)
        x = inputs.normal(30 + case, "x", (M, 512), 1.0, "bf16")
        w = inputs.normal(30 + case, "w", (N, 512), 0.05, "bf16")
        if gated:
            wu = inputs.normal(30 + case, "wu", (N, 512), 0.05, "bf16")
            ref = orc.ffn_gate_up(inputs.as_oracle(x), inputs.as_oracle(w), inputs.as_oracle(wu), "bf16")
            assert fc.fc_linear_workspace_bytes("bf16", M, 512, 2 * N) == 0
            out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
            fc.fc_ffn_gate_up("bf16", _dev(x), _dev(w), _dev(wu), M, 512, N, out, None, 0)
        else:
            r = inputs.normal(30 + case, "r", (M, N), 1.0, "bf16") if case % 4 == 0 else None
            ref = orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), None if r is None else inputs.as_oracle(r),
                                      "bf16")
            out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
            fc.fc_linear_residual("bf16", _dev(x), _dev(w), _dev(r), M, 512, N, out, None, 0)
        torch.cuda.synchronize()
        assert_close(inputs.as_oracle(out), ref, "bf16", "whole-row sweep case %d (M %d, N %d, gated %s)" % (case, M, N, gated))


@pytest.mark.parametrize("wgs", ["2", "7", "300"])
def test_whole_row_kernel_any_number_of_workgroups(wgs, knob):
    # runs of 1, 38 and 131 items: the staged outputs of a run are flushed every 16 items and at its end
    knob("FC_LIN_WGS", wgs)
    M, K = 27, 512
    x = inputs.normal(5, "x", (M, K), 1.0, "bf16")
    for gated, N in ((True, 4 * 523), (False, 8 * 523)):
        w = inputs.normal(5, "w", (N, K), 0.05, "bf16")
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        if gated:
            wu = inputs.normal(5, "wu", (N, K), 0.05, "bf16")
            ref = orc.ffn_gate_up(inputs.as_oracle(x), inputs.as_oracle(w), inputs.as_oracle(wu), "bf16")
            fc.fc_ffn_gate_up("bf16", _dev(x), _dev(w), _dev(wu), M, K, N, out, None, 0)
        else:
            r = inputs.normal(5, "r", (M, N), 1.0, "bf16")
            ref = orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), inputs.as_oracle(r), "bf16")
            fc.fc_linear_residual("bf16", _dev(x), _dev(w), _dev(r), M, K, N, out, None, 0)
        torch.cuda.synchronize()
        assert_close(inputs.as_oracle(out), ref, "bf16", "whole-row kernel, %s workgroups, gated %s" % (wgs, gated))


@pytest.mark.parametrize("shape", ["0", "1", "2"])
@pytest.mark.parametrize("ksplit", ["1", "3"])
def test_linear_residual_wide_window_tile_shapes(shape, ksplit, knob):
    # more than 32 rows: tiled GEMM, every tile shape, with and without a split of the hidden dimension;
    # ragged row count, an odd number of 128-row slabs
    knob("FC_LIN_WIDE_SHAPE", shape)
    knob("FC_LIN_KSPLIT", ksplit)
    M, K, N = 200, 1024, 384
    x = inputs.normal(12, "x", (M, K), 1.0, "bf16")
    w = inputs.normal(12, "w", (N, K), 0.05, "bf16")
    r = inputs.normal(12, "r", (M, N), 1.0, "bf16")
    ref = orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), inputs.as_oracle(r), "bf16")
    need = fc.fc_linear_workspace_bytes("bf16", M, K, N)
    assert (need > 0) == (ksplit != "1")
    ws = _ws(need)
    rd = _dev(r)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    fc.fc_linear_residual("bf16", _dev(x), _dev(w), rd, M, K, N, out, ws, need)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, "bf16", "wide linear_residual shape %s ksplit %s" % (shape, ksplit))
    fc.fc_linear_residual("bf16", _dev(x), _dev(w), rd, M, K, N, rd, ws, need)  # in place
    torch.cuda.synchronize()
    assert torch.equal(rd, out)


@pytest.mark.parametrize("shape", ["0", "1", "2", "4"])
def test_ffn_gate_up_wide_window_tile_shapes(shape, knob):
    knob("FC_LIN_WIDE_SHAPE", shape)
    M, K, F = 100, 1024, 320
    x = inputs.normal(13, "x", (M, K), 1.0, "bf16")
    wg = inputs.normal(13, "wg", (F, K), 0.05, "bf16")
    wu = inputs.normal(13, "wu", (F, K), 0.05, "bf16")
    ref = orc.ffn_gate_up(inputs.as_oracle(x), inputs.as_oracle(wg), inputs.as_oracle(wu), "bf16")
    need = fc.fc_linear_workspace_bytes("bf16", M, K, 2 * F)
    ws = _ws(need)
    out = torch.full((M, F), float("nan"), dtype=torch.bfloat16, device=DEV)
    fc.fc_ffn_gate_up("bf16", _dev(x), _dev(wg), _dev(wu), M, K, F, out, ws, need)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), ref, "bf16", "wide ffn_gate_up shape " + shape)


def test_wide_linear_layers_of_a_little_more_than_one_round():
    # 260 slabs x one row tile of the 256-row shape are 260 workgroups, a little more than one per compute
    # unit.  The plain layer is cut in two launches (256 slabs in that shape, the last 4 with a smaller
    # tile); the gated layer takes the shape of 80 dealt (gate, up) pairs in one launch, and with 330 slabs,
    # too many for that, two launches again.  Every output checked.
    M, K = 200, 256
    x = inputs.normal(15, "x", (M, K), 1.0, "bf16")
    N = 128 * 260
    w = inputs.normal(15, "w", (N, K), 0.05, "bf16")
    r = inputs.normal(15, "r", (M, N), 1.0, "bf16")
    assert fc.fc_linear_workspace_bytes("bf16", M, K, N) == 0
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    fc.fc_linear_residual("bf16", _dev(x), _dev(w), _dev(r), M, K, N, out, None, 0)
    torch.cuda.synchronize()
    assert_close(inputs.as_oracle(out), orc.linear_residual(inputs.as_oracle(x), inputs.as_oracle(w), inputs.as_oracle(r),
                                                            "bf16"), "bf16", "two-launch linear_residual")
    for slabs in (260, 330):
        F = 64 * slabs
        wg = inputs.normal(15, "wg%d" % slabs, (F, K), 0.05, "bf16")
        wu = inputs.normal(15, "wu%d" % slabs, (F, K), 0.05, "bf16")
        act = torch.full((M, F), float("nan"), dtype=torch.bfloat16, device=DEV)
        fc.fc_ffn_gate_up("bf16", _dev(x), _dev(wg), _dev(wu), M, K, F, act, None, 0)
        torch.cuda.synchronize()
        assert_close(inputs.as_oracle(act), orc.ffn_gate_up(inputs.as_oracle(x), inputs.as_oracle(wg), inputs.as_oracle(wu),
                                                            "bf16"), "bf16", "ffn_gate_up, %d slabs" % slabs)


def test_linear_calls_default_plan_at_block_widths():
    # the shapes of a 256-row block at the 7B widths, default plan: W_out and W_2 (28 slabs: hidden
    # dimension split), gated W_1 (296 slabs); rows sampled for the oracle
    M = 256
    for K, N, gated in ((3584, 3584, False), (18944, 3584, False), (3584, 18944, True)):
        x = inputs.normal(14, "x%d" % K, (M, K), 1.0, "bf16")
        w = inputs.normal(14, "w%d%d" % (K, N), (N, K), 0.02, "bf16")
        rows = [0, 31, 32, 127, 128, 200, 255]
        xo, wo = inputs.as_oracle(x)[rows], inputs.as_oracle(w)
        need = fc.fc_linear_workspace_bytes("bf16", M, K, 2 * N if gated else N)
        ws = _ws(need)
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        if gated:
            wu = inputs.normal(14, "wu", (N, K), 0.02, "bf16")
            fc.fc_ffn_gate_up("bf16", _dev(x), _dev(w), _dev(wu), M, K, N, out, ws, need)
            ref = orc.ffn_gate_up(xo, wo, inputs.as_oracle(wu), "bf16")
        else:
            r = inputs.normal(14, "r", (M, N), 1.0, "bf16")
            fc.fc_linear_residual("bf16", _dev(x), _dev(w), _dev(r), M, K, N, out, ws, need)
            ref = orc.linear_residual(xo, wo, inputs.as_oracle(r)[rows], "bf16")
        torch.cuda.synchronize()
        got = inputs.as_oracle(out)
        assert np.all(np.isfinite(got))
        assert_close(got[rows], ref, "bf16", "block-width linear K=%d N=%d" % (K, N))


class FullLayer:
    """One layer's weights on the GPU and on the oracle side."""

    def __init__(self, w: inputs.Workload, seed, with_bias=False, std=0.02):
        self.w = w
        self.host = inputs.layer_weights(w, seed, 0, with_bias, std)
        self.dev = {k: _dev(v) for k, v in self.host.items()}
        self.orc = {k: (None if v is None else inputs.as_oracle(v)) for k, v in self.host.items()}
        d = self.dev
        self.handle = fc.make_layer_weights(d["norm1"], d["w_qkv"], d["b_qkv"], d["w_out"], d["norm2"], d["w_gate"],
                                            d["w_up"], d["w_down"], w.d_ff, w.norm_eps)

    def gpu_step(self, cache: GpuLayerCache, X, win_start, kv_len, pos=None):
        """The whole layer through its one entry point."""
        A = X.shape[1]
        need = fc.fc_full_layer_workspace_bytes(cache.cfg, self.w.d_ff, A)
        ws = _ws(need)
        xd = _dev(X)
        y = torch.full_like(xd, float("nan"))
        fc.fc_full_layer_step(cache.handle, 0, self.handle, xd, win_start, A, _dev(pos), kv_len, y, ws, need)
        torch.cuda.synchronize()
        return y

    def gpu_chain(self, cache: GpuLayerCache, X, win_start, kv_len, pos=None):
        """The same modules called one by one; returns every tensor handed from module to module."""
        w, d, dt = self.w, self.dev, self.w.dtype
        B, A = X.shape[0], X.shape[1]
        M, E, F = B * A, w.n_q_heads * w.head_dim, w.d_ff
        new = lambda *shape: torch.full(shape, float("nan"), dtype=inputs.TORCH_DTYPE[dt], device=DEV)
        xd, posd = _dev(X), _dev(pos)
        t = {"h1": new(B, A, w.hidden), "q": new(B, w.n_q_heads, A, w.head_dim), "o": new(B, A, E),
             "x2": new(B, A, w.hidden), "h2": new(B, A, w.hidden), "act": new(B, A, F), "y": new(B, A, w.hidden)}
        need = max(fc.fc_linear_workspace_bytes(dt, M, E, w.hidden), fc.fc_linear_workspace_bytes(dt, M, w.hidden, 2 * F),
                   fc.fc_linear_workspace_bytes(dt, M, F, w.hidden))
        ws = _ws(need)
        fc.fc_rmsnorm(dt, xd, d["norm1"], w.norm_eps, M, w.hidden, t["h1"])
        fc.fc_qkv_project_scatter(cache.handle, 0, t["h1"], d["w_qkv"], d["b_qkv"], win_start, A, posd, t["q"])
        fc.fc_active_attention(cache.handle, 0, t["q"], A, kv_len, posd, t["o"], cache.workspace, cache.ws_bytes)
        fc.fc_linear_residual(dt, t["o"], d["w_out"], xd, M, E, w.hidden, t["x2"], ws, need)
        fc.fc_rmsnorm(dt, t["x2"], d["norm2"], w.norm_eps, M, w.hidden, t["h2"])
        fc.fc_ffn_gate_up(dt, t["h2"], d["w_gate"], d["w_up"], M, w.hidden, F, t["act"], ws, need)
        fc.fc_linear_residual(dt, t["act"], d["w_down"], t["x2"], M, F, w.hidden, t["y"], ws, need)
        torch.cuda.synchronize()
        return t


def _run_full_layer(w: inputs.Workload, L, A, seed, with_bias=False, pad=False, std=0.02):
    """Cache rows [0, L) filled directly, then one cached step of the whole layer on [L, L + A):
    (1) every module against the oracle's module on the GPU's own input to it, at the single-module
    tolerance; (2) the one-call entry point against the module-by-module chain, bit for bit;
    (3) the output against the oracle's whole layer (see _chain_tolerance)."""
    S = L + A
    dt = w.dtype
    layer = FullLayer(w, seed, with_bias, std)
    ocfg = orc.OracleConfig(w.batch, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, dt)
    K, V = inputs.kv_fill(w, seed, L)
    X = inputs.hidden_states(w, seed, A)
    pos = inputs.window_positions(w.batch, L, A)
    if pad:
        pos[:, 1] = -1
        pos[-1, A - 1] = -1
    pos_arg = pos if pad else None
    caches = []
    for _ in range(2):
        g = GpuLayerCache(dt, w.batch, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, max_rows=A)
        g.write_rows(0, K, V, 0)
        caches.append(g)
    t = layer.gpu_chain(caches[0], X, L, S, pos_arg)
    y = layer.gpu_step(caches[1], X, L, S, pos_arg)

    # (2) one call == the chain of calls
    assert torch.equal(y, t["y"])
    assert torch.equal(caches[0].k_store, caches[1].k_store) and torch.equal(caches[0].v_store, caches[1].v_store)

    # (1) module by module, each on the GPU's own input
    o = {k: inputs.as_oracle(v) for k, v in t.items()}
    W, M = layer.orc, w.batch * A
    Xo, po = inputs.as_oracle(X), inputs.as_oracle(pos)
    Kc = np.zeros((w.batch, w.n_kv_heads, S, w.head_dim), np.float32)
    Vc = np.zeros_like(Kc)
    Kc[:, :, :L], Vc[:, :, :L] = inputs.as_oracle(K), inputs.as_oracle(V)
    assert_close(o["h1"], orc.rmsnorm(Xo, W["norm1"], w.norm_eps, dt), dt, "h1")
    K1, V1 = Kc.copy(), Vc.copy()
    q_ref, o_ref = orc.layer_step(ocfg, o["h1"], W["w_qkv"], W["b_qkv"], po, S, K1, V1)
    Kg, Vg = caches[0].read_rows(0, 0, S)
    assert_close(o["q"], q_ref, dt, "q")
    assert_close(Kg[:, :, L:], K1[:, :, L:], dt, "fresh K rows")
    assert_close(Vg[:, :, L:], V1[:, :, L:], dt, "fresh V rows")
    assert np.array_equal(Kg[:, :, :L], Kc[:, :, :L]) and np.array_equal(Vg[:, :, :L], Vc[:, :, :L])
    # attention on the GPU's own q and cache rows
    assert_close(o["o"], orc.attend(ocfg, o["q"], Kg, Vg, S, po), dt, "attention output")
    E, F, d = w.n_q_heads * w.head_dim, w.d_ff, w.hidden
    assert_close(o["x2"].reshape(M, d), orc.linear_residual(o["o"].reshape(M, E), W["w_out"], Xo.reshape(M, d), dt),
                 dt, "x2")
    assert_close(o["h2"], orc.rmsnorm(o["x2"], W["norm2"], w.norm_eps, dt), dt, "h2")
    assert_close(o["act"].reshape(M, F), orc.ffn_gate_up(o["h2"].reshape(M, d), W["w_gate"], W["w_up"], dt), dt, "act")
    assert_close(o["y"].reshape(M, d),
                 orc.linear_residual(o["act"].reshape(M, F), W["w_down"], o["x2"].reshape(M, d), dt), dt, "y")

    # (3) end to end
    ref = orc.full_layer_step(ocfg, Xo, W, po, S, Kc, Vc, w.norm_eps)
    _chain_tolerance(o["y"], ref, dt, "full layer output")
    for g in caches:
        g.close()


def test_full_layer_step_tiny_f32():
    _run_full_layer(inputs.C1.scaled(cached_len=100), 100, 32, seed=5, with_bias=True, std=0.06)


def test_full_layer_step_small_bf16_generic_shapes():
    # shapes none of the matrix-core kernels cover: every module runs on the plain kernels
    w = inputs.Workload("small", "bf16", 2, 136, 6, 2, 64, 0, 0, d_ff=200)
    _run_full_layer(w, 50, 12, seed=6, with_bias=True, pad=True, std=0.08)


def test_full_layer_step_streaming_kernels_bf16():
    # a narrow model that still takes the matrix-core path everywhere (hidden 512, d_ff 1024)
    w = inputs.Workload("narrow", "bf16", 1, 512, 4, 2, 128, 0, 0, d_ff=1024)
    _run_full_layer(w, 300, 32, seed=7, std=0.04)
    _run_full_layer(w.scaled(batch=2), 130, 16, seed=8, pad=True, std=0.04)
    _run_full_layer(w.scaled(batch=3), 90, 40, seed=10, pad=True, std=0.04)   # 120 rows: tiled GEMM everywhere


def test_full_layer_step_dream7b_geometry():
    # the 7B geometry at its real widths (hidden 3584, 28/4 heads, d_ff 18944), window of 32 rows
    _run_full_layer(inputs.C2.scaled(cached_len=480), 480, 32, seed=9)
