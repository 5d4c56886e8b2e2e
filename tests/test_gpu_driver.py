"""The decoding loop (section 3.2.1) on a tiny synthetic diffusion LM, driven through the C-ABI ops and
mirrored on the CPU oracle, in two schedules: the paper's literal reducing window, described below, and
the block window with a refresh of the generation region after every block.

Initial pass: every layer projects and caches all rows of prompt + generation region.  Then, block by
block, the active window is the current block and all later ones: its rows are re-embedded, run
through every layer (`fc_full_layer_step`), the rows of the current block go through the final norm
and the vocabulary projection, and the most confident masked positions are filled (section 3.1).  When
a block is complete the window shrinks past it and its cache rows are never written again.

The per-op parity is tested elsewhere at the stated tolerances; this test checks the orchestration:
the schedule, which rows are recomputed, the freeze rule (bitwise), the integer bookkeeping (bit-exact
given the same confidences), and that the GPU's hidden states and token choices stay within the chained
float bound of the oracle's."""
import numpy as np
import pytest
import torch

from oracle import fc_oracle as orc
from paper_2505_21467_amd import binding as fc
from paper_2505_21467_amd import inputs
from tests.harness import GpuLayerCache, assert_chain_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("mode", ["reducing", "block"])
def test_decoding_loop_on_a_tiny_model(mode):
    """mode "reducing": the paper's literal window (the current block and all later ones).  mode "block":
    the window is the current block only, and after the last step of a block the whole generation
    region is refreshed (the schedule of the 28-layer bench configuration)."""
    B, d, Hq, Hkv, Dh, F, V, NL = 2, 512, 4, 2, 128, 1024, 1024, 2
    P, G, Bk, spb = 24, 64, 16, 4          # 4 blocks of 16 tokens, 4 steps per block, 4 tokens per step
    S, MASK, k, eps, dt = P + G, V + 7, Bk // spb, 1e-6, "bf16"
    w = inputs.Workload("tiny_dlm", dt, B, d, Hq, Hkv, Dh, P, Bk, n_layers=NL, gen_len=G, block=Bk,
                        steps_per_block=spb, d_ff=F)
    tdt = torch.bfloat16

    # model: embedding, NL layers, final norm, vocabulary matrix
    emb = inputs.normal(41, "emb", (V + 8, d), 1.0, dt)           # rows V.. hold the mask embedding
    w_vocab = inputs.normal(41, "w_vocab", (V, d), 0.05, dt)
    final_norm = (1.0 + 0.1 * inputs.normal(41, "fn", (d,), 1.0, "f32")).to(tdt)
    host_layers = [inputs.layer_weights(w, 41, layer, std=0.04) for layer in range(NL)]
    dev_layers, handles = [], []
    for hl in host_layers:
        t = {kk: (None if v is None else v.to(DEV)) for kk, v in hl.items()}
        dev_layers.append(t)
        handles.append(fc.make_layer_weights(t["norm1"], t["w_qkv"], t["b_qkv"], t["w_out"], t["norm2"], t["w_gate"],
                                             t["w_up"], t["w_down"], F, eps))
    orc_layers = [{kk: (None if v is None else inputs.as_oracle(v)) for kk, v in hl.items()} for hl in host_layers]
    emb_d, w_vocab_d, fn_d = emb.to(DEV), w_vocab.to(DEV), final_norm.to(DEV)
    emb_o, w_vocab_o, fn_o = inputs.as_oracle(emb), inputs.as_oracle(w_vocab), inputs.as_oracle(final_norm)

    tokens = np.full((B, S), MASK, np.int32)
    tokens[:, :P] = inputs.integers(41, "prompt", (B, P), 0, V).numpy()
    tok_d = torch.from_numpy(tokens.copy()).to(DEV)
    tok_o = tokens.copy()

    g = GpuLayerCache(dt, B, d, Hq, Hkv, Dh, S, n_layers=NL, max_rows=S)
    ocfg = orc.OracleConfig(B, d, Hq, Hkv, Dh, S, dt)
    Kc = [np.zeros((B, Hkv, S, Dh), np.float32) for _ in range(NL)]
    Vc = [np.zeros((B, Hkv, S, Dh), np.float32) for _ in range(NL)]
    ws_bytes = fc.fc_full_layer_workspace_bytes(g.cfg, F, S)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=DEV)
    lm_bytes = fc.fc_lm_head_workspace_bytes(dt, B * Bk, d, V)
    lm_ws = torch.empty(lm_bytes, dtype=torch.uint8, device=DEV)

    def forward(win_start, rows, first_layer_bound=None):
        """Embed the window rows and run them through every layer, on both sides; returns (x_gpu, x_oracle).
        first_layer_bound: name of the pass whose first layer sees the same input rows on both sides; its
        output is then held to the per-tensor bound of a whole layer (largest error and mean relative
        error), not only to the loose mean used further down the chain."""
        idx = (torch.arange(B, device=DEV)[:, None] * S + win_start + torch.arange(rows, device=DEV)[None, :])
        ids = tok_d.view(-1)[idx.reshape(-1)].contiguous()
        x = torch.empty((B, rows, d), dtype=tdt, device=DEV)
        fc.fc_gather_rows(dt, emb_d, V + 8, d, ids, B * rows, x)
        xo = orc.gather_rows(emb_o, tok_o[:, win_start:win_start + rows].reshape(-1)).reshape(B, rows, d)
        pos = np.tile(np.arange(win_start, win_start + rows, dtype=np.int32), (B, 1))
        for layer in range(NL):
            y = torch.empty_like(x)
            fc.fc_full_layer_step(g.handle, layer, handles[layer], x, win_start, rows, None, S, y, ws, ws_bytes)
            x = y
            xo = orc.full_layer_step(ocfg, xo, orc_layers[layer], pos, S, Kc[layer], Vc[layer], eps)
            if layer == 0 and first_layer_bound:
                torch.cuda.synchronize()
                assert_chain_close(inputs.as_oracle(x), xo, dt, first_layer_bound + ", first layer")
        torch.cuda.synchronize()
        return x, xo

    # Past the first layer of a pass the two sides no longer see the same inputs: each feeds its own
    # rounded hidden states to the next layer and attends over its own cache rows, so differences of
    # one storage ulp are amplified layer by layer and step by step.  There only a mean bound (four
    # times the single-tensor one) is applied; the per-tensor bounds are applied where the inputs are
    # the same (first layer of the initial pass and of step 0) and, op by op, in the other test files.
    def close(gpu, ref, what, mean_rel=2e-2):
        gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
        assert np.all(np.isfinite(gpu)), what
        err = np.mean(np.abs(gpu - ref)) / max(np.mean(np.abs(ref)), 1e-30)
        assert err <= mean_rel, "%s: mean-rel %.3e" % (what, err)

    # initial pass over prompt + all blocks
    x, xo = forward(0, S, first_layer_bound="initial pass")
    close(inputs.as_oracle(x), xo, "initial pass output")
    n_blocks, rows_projected = G // Bk, 0
    for step in range(n_blocks * spb):
        if mode == "reducing":
            win_start, rows, refresh_after = fc.fc_window(step, P, G, Bk, spb, 0, 1)
            assert win_start + rows == S
        else:
            win_start, rows, refresh_after = fc.fc_window(step, P, G, Bk, spb, spb, 0)
            assert rows == Bk and refresh_after == (1 if step % spb == spb - 1 else 0)
        blk = step // spb
        assert win_start == P + blk * Bk
        before_k, before_v = g.snapshot()
        x, xo = forward(win_start, rows, first_layer_bound="step 0" if step == 0 else None)
        rows_projected += rows
        close(inputs.as_oracle(x), xo, "step %d window output" % step)
        # freeze rule: cache rows before the window are bit-identical, in every layer
        after_k, after_v = g.snapshot()
        frozen = _frozen_equal(g, before_k, after_k, before_v, after_v, win_start, NL)
        assert frozen, "step %d: a cache row before the window changed" % step

        # rows of the current block -> final norm -> vocabulary projection -> fill
        idx = (torch.arange(B, device=DEV, dtype=torch.int32)[:, None] * rows +
               torch.arange(Bk, device=DEV, dtype=torch.int32)[None, :]).reshape(-1).contiguous()
        hb = torch.empty((B * Bk, d), dtype=tdt, device=DEV)
        fc.fc_gather_rows(dt, x, B * rows, d, idx, B * Bk, hb)
        fc.fc_rmsnorm(dt, hb, fn_d, eps, B * Bk, d, hb)
        tok_blk = torch.empty((B * Bk,), dtype=torch.int32, device=DEV)
        conf_blk = torch.empty((B * Bk,), dtype=torch.float32, device=DEV)
        fc.fc_lm_head_argmax(dt, hb, w_vocab_d, B * Bk, d, V, tok_blk, conf_blk, lm_ws, lm_bytes)
        pos_next = torch.empty((B, Bk), dtype=torch.int32, device=DEV)
        count = torch.empty((B,), dtype=torch.int32, device=DEV)
        fc.fc_unmask_select(tok_blk, conf_blk, None, win_start, B, Bk, k, MASK, tok_d, S, pos_next, count)
        torch.cuda.synchronize()

        # oracle: its own hidden states give its own logits; the GPU's choice must be (near) the largest
        ho = orc.rmsnorm(xo[:, :Bk].reshape(B * Bk, d), fn_o, eps, dt)
        _, _, z = orc.lm_head_argmax(ho, w_vocab_o, want_logits=True)
        tg, cg = tok_blk.cpu().numpy(), conf_blk.cpu().numpy()
        assert np.all((tg >= 0) & (tg < V))
        assert np.all(z.max(axis=1) - z[np.arange(B * Bk), tg] <= 0.25), "step %d: token far from the arg-max" % step
        # integer bookkeeping: exact, given the GPU's tokens and confidences
        pos_blk = np.tile(np.arange(win_start, win_start + Bk, dtype=np.int32), (B, 1))
        want_next, want_count = orc.unmask_select(tg.reshape(B, Bk), cg.reshape(B, Bk).astype(np.float64), pos_blk, k,
                                                  MASK, tok_o)
        assert np.array_equal(tok_d.cpu().numpy(), tok_o)
        assert np.array_equal(pos_next.cpu().numpy(), want_next) and np.array_equal(count.cpu().numpy(), want_count)
        assert np.all(want_count == Bk - k * (step % spb + 1))
        assert np.all(tok_o[:, win_start + Bk:] == MASK)                   # later blocks stay masked

        if mode == "block" and refresh_after:
            # the block is complete: re-project the whole generation region in every layer; the prompt
            # rows stay frozen
            before_k, before_v = g.snapshot()
            x, xo = forward(P, G)
            close(inputs.as_oracle(x), xo, "refresh after step %d" % step)
            after_k, after_v = g.snapshot()
            assert _frozen_equal(g, before_k, after_k, before_v, after_v, P, NL), "a prompt row changed in a refresh"

    assert not np.any(tok_o == MASK)
    if mode == "reducing":
        assert rows_projected == spb * Bk * n_blocks * (n_blocks + 1) // 2  # closed form of the reducing window
    else:
        assert rows_projected == spb * Bk * n_blocks
    g.close()


def _frozen_equal(g, before_k, after_k, before_v, after_v, win_start, n_layers):
    """Bitwise comparison of the raw cache storage of all rows before win_start, every layer."""
    if win_start == 0:
        return True
    cfg = g.cfg
    spad = (cfg.max_seq + 63) // 64 * 64
    B, Hkv, Dh = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    kb = before_k.view(n_layers, B, Hkv, spad, Dh)[:, :, :, :win_start]
    ka = after_k.view(n_layers, B, Hkv, spad, Dh)[:, :, :, :win_start]
    if not torch.equal(kb, ka):
        return False
    # V is stored as 64-row transposed tiles [tile][Dh][64]: whole tiles before the window, then the
    # leading key columns of the tile that straddles it
    vb = before_v.view(n_layers, B, Hkv, spad // 64, Dh, 64)
    va = after_v.view(n_layers, B, Hkv, spad // 64, Dh, 64)
    full, part = win_start // 64, win_start % 64
    if full and not torch.equal(vb[:, :, :, :full], va[:, :, :, :full]):
        return False
    return part == 0 or torch.equal(vb[:, :, :, full, :, :part], va[:, :, :, full, :, :part])
