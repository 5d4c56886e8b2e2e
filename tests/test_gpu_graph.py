"""The cached step recorded into a HIP graph: the entry points allocate nothing, clear nothing with a
memset and never synchronize, so a caller may capture them on its stream and replay the graph.  The test
records one denoising step of a tiny model (embedding gather, two whole layers of section 3.2.1's cached
step, final norm, vocabulary projection with arg-max, confidence-ranked fill of section 3.1) and checks
several replays, with eager work and synchronizations between them, bit for bit against the same step
launched eagerly from the same state."""
import pytest
import torch

from paper_2505_21467_amd import binding as fc
from paper_2505_21467_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_cached_step_replayed_from_a_graph():
    B, d, Hq, Hkv, Dh, F, V, NL = 2, 512, 4, 2, 128, 1024, 1024, 2
    P, G, A, k_fill = 40, 64, 16, 4
    S, MASK, eps, dt, tdt = P + G, V, 1e-6, "bf16", torch.bfloat16
    w = inputs.Workload("tiny_dlm_graph", dt, B, d, Hq, Hkv, Dh, P, A, n_layers=NL, gen_len=G, block=A,
                        steps_per_block=4, d_ff=F)
    emb = inputs.normal(43, "emb", (V + 1, d), 1.0, dt).to(DEV)
    w_vocab = inputs.normal(43, "w_vocab", (V, d), 0.05, dt).to(DEV)
    final_norm = (1.0 + 0.1 * inputs.normal(43, "fn", (d,), 1.0, "f32")).to(tdt).to(DEV)
    keep, handles = [], []
    for layer in range(NL):
        t = {kk: (None if v is None else v.to(DEV)) for kk, v in inputs.layer_weights(w, 43, layer, std=0.04).items()}
        keep.append(t)
        handles.append(fc.make_layer_weights(t["norm1"], t["w_qkv"], t["b_qkv"], t["w_out"], t["norm2"], t["w_gate"],
                                             t["w_up"], t["w_down"], F, eps))
    cfg = fc.make_config(NL, B, d, Hq, Hkv, Dh, S, dt, w.rope_base)
    n_el = fc.fc_cache_storage_bytes(cfg) // 2
    k_store = inputs.normal(43, "k0", (n_el,), 0.5, dt).to(DEV)
    v_store = inputs.normal(43, "v0", (n_el,), 0.5, dt).to(DEV)
    cache = fc.fc_cache_alloc(cfg, k_store, v_store)
    ws_bytes = fc.fc_full_layer_workspace_bytes(cfg, F, S)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
    lm_bytes = fc.fc_lm_head_workspace_bytes(dt, B * A, d, V)
    lm_ws = torch.empty(max(lm_bytes, 16), dtype=torch.uint8, device=DEV)

    tokens0 = torch.full((B, S), MASK, dtype=torch.int32, device=DEV)
    tokens0[:, :P] = inputs.integers(43, "prompt", (B, P), 0, V).to(DEV)
    tokens = tokens0.clone()
    x, y = (torch.empty((B, A, d), dtype=tdt, device=DEV) for _ in range(2))
    tok = torch.empty((B * A,), dtype=torch.int32, device=DEV)
    conf = torch.empty((B * A,), dtype=torch.float32, device=DEV)
    pos_next = torch.empty((B, A), dtype=torch.int32, device=DEV)
    count = torch.empty((B,), dtype=torch.int32, device=DEV)
    pos = (P + 16 + torch.arange(A, dtype=torch.int32, device=DEV)).repeat(B, 1).contiguous()   # the window, on the device
    idx = torch.empty((B, A), dtype=torch.int32, device=DEV)

    def step(stream):
        a, b = x, y
        idx.copy_(torch.gather(tokens, 1, pos.long()))       # token ids of the window's rows (a torch copy kernel)
        for s in range(B):
            fc.fc_gather_rows(dt, emb, V + 1, d, idx[s], A, a[s], stream)
        for layer in range(NL):
            fc.fc_full_layer_step(cache, layer, handles[layer], a, 0, A, pos, S, b, ws, ws_bytes, stream)
            a, b = b, a
        h = a.view(B * A, d)
        fc.fc_rmsnorm(dt, h, final_norm, eps, B * A, d, h, stream)
        fc.fc_lm_head_argmax(dt, h, w_vocab, B * A, d, V, tok, conf, lm_ws, lm_bytes, stream)
        fc.fc_unmask_select(tok, conf, pos, 0, B, A, k_fill, MASK, tokens, S, pos_next, count, stream)
        return a

    def state():
        return [t.clone() for t in (x, y, tok, conf, tokens, pos_next, count, k_store, v_store)]

    # warm-up on a side stream (what torch asks for before a capture), then the capture itself
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    tokens.copy_(tokens0)
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()

    for replay in range(4):
        # the window moves by a block every second replay: the graph reads `pos` and `tokens` anew
        pos.copy_((P + 16 * (replay // 2) + torch.arange(A, dtype=torch.int32, device=DEV)).repeat(B, 1))
        tokens.copy_(tokens0)
        step(torch.cuda.current_stream().cuda_stream)        # eager, from this state
        torch.cuda.synchronize()
        want = state()
        filled = int((want[4] != tokens0).sum())
        assert filled == B * k_fill, "the eager step fills k tokens per sequence"
        tokens.copy_(tokens0)
        for t in (x, y, conf):
            t.zero_()
        tok.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = state()
        for name, g_, w_ in zip(("x", "y", "tok", "conf", "tokens", "pos_next", "count", "k", "v"), got, want):
            same = torch.equal(g_.view(torch.int16) if g_.dtype == tdt else g_, w_.view(torch.int16) if w_.dtype == tdt else w_)
            assert same, "replay %d: %s differs from the eager step" % (replay, name)
