"""Benchmark of the FreeCache cached denoising layer-step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers N]
                    [--workload c4|c2|c3|c5|c5_refresh|c4_layer|c2_layer|c3_layer|c5_layer|c5_refresh_layer|
                                c4_unmask|c5_unmask|c4_accept|c5_drift|c5_decode|c5_decode_model]

A "step" is one pass of the whole hot path for one layer: QKV projection + RoPE + scatter of the
active window, then attention of the window's queries over the cache.  The default workload is the
long-context Dream-7B-shaped configuration (prompt 16384, window of 32 rows sliding by 32 every 8
steps, 28/4 GQA heads, head_dim 128, bf16), on which the metric's bandwidth target is quoted.

`value` is the time of exactly `--steps` steps recorded once into a HIP graph and replayed (the library's
calls allocate nothing, issue no memset node and never synchronise, so they are captured as they
are); the same steps launched one by one from the host are reported beside it (`eager_us_per_step`).
The default run also carries the other configurations in compact form (`others`: C2, C3, the cached
step and the refresh of C5, and the 28-layer block schedule of C5 in decoded tokens/s).

So that the key/value stream really comes from HBM and not from the 256 MB memory-side cache, the
timed loop rotates over `--layers` distinct layer caches and weight matrices (default: enough for
more than 1.5 GB of working set), as a 28-layer model does between two visits of one layer.  The
same loop on a single layer is reported as `single_cache_us` (cache-resident figure).

`--workload c5_refresh` times the periodic refresh of configuration 5 instead (one `fc_refresh` of the
256-row generation region of 8 sequences per step: a dense, matrix-core-bound pass).

`--workload <c>_layer` time the whole transformer layer on the window rows instead (RMSNorm, the path
above, output projection + residual, RMSNorm, gated feed-forward network + residual: one
`fc_full_layer_step` per step), the next row after the attention path; `c5_refresh_layer` does so for
the 256-row refresh of 8 sequences (2048 rows).

`--workload c4_unmask` / `c5_unmask` time the unmasking step of a block (vocabulary projection of the
block's rows with arg-max and confidence, `fc_lm_head_argmax`, then `fc_unmask_select`; vocabulary
152064 x hidden 3584, the Dream-7B sizes).  `--workload c4_accept` times the Guided Diffusion acceptance of
one 32-token speculation block on synthetic DLM / AR logits (`fc_guided_accept`, Top-2 match, tau 0.5).
`--workload c5_drift` times the KV drift diagnostic around a step (snapshot of the window rows with
`fc_cache_read_rows`, then `fc_kv_similarity`) for the 256-row generation region of 8 sequences.

`--workload c5_decode` runs the whole block schedule of configuration 5 on the hot path: 28 layers, 8
sequences, prompt 2048 + 256 generated tokens in blocks of 32; a step is one denoising step of all 28
layers (projection + scatter + attention of the active block, per-layer synthetic inputs) plus, after
every 8th step, the refresh of the generation region in all layers; value = decoded tokens/s.
`--workload c5_decode_model` does the same with whole layers and the unmasking step (token embeddings,
28 x `fc_full_layer_step`, final norm, vocabulary projection, confidence-ranked fill): the decoding loop
of a synthetic 7B-shaped model.

Prints ONE JSON line (see the fields below).  Inputs are seeded and synthetic.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the attention call (main kernel + merge kernel) on the default workload,
# from `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs of this command, scaled by what the same
# counters read for the plain 256 MiB copy at the end of this file (profiles/ holds the summary).
# HBM bytes per launch of the gated W_1 at 32 rows and the 7B widths (k_linear_rows), same method
# (profiles/c4_whole_layer_step.md): 273.8 MB fetched + 3.1 MB written.
MEASURED_GATE_UP_TRAFFIC_BYTES = {(32, 3584, 18944): 274_990_000}

# The vocabulary projection of 32 rows (k_linear_rows, profiles/unmask_step.md): 1091.94 MB fetched, 0.1 MB written.
MEASURED_LM_HEAD_TRAFFIC_BYTES = {(32, 3584, 152064): 1_092_040_000}

# HBM bytes per launch of the attention call (main kernel + merge kernel), from `rocprofv3 --pmc
# FETCH_SIZE` / `--pmc WRITE_SIZE` runs of this command, scaled by what the same counters read for the
# plain 256 MiB copy at the end of the run.  Each figure is tied to the launch plan it was measured
# with (fc_attention_plan) and to the summary under profiles/ that holds the counter values; a run
# whose planner picks another plan reports null instead.
MEASURED_ATTENTION_TRAFFIC = {
    "c4_dream7b_long_L16384_A32": {
        "bytes": 53_010_000,   # 35.08 MB read + 7.31 MB written (main kernel), 10.39 + 0.23 MB (merge)
        "plan": {"kind": 1, "splits": 30, "keys_per_split": 576, "tiles_per_wg": 4, "waves": 8},
        "kernels": "k_attn_mfma<1,8,2> + k_attn_combine<8,4>",
        "profile": "profiles/c4_long_context_layer_step.md"},
    "c3_llada8b_B4_L4096_A64": {
        "bytes": 287_800_000,  # 274.9 + 4.46 MB, 6.34 + 2.10 MB
        "plan": {"kind": 1, "splits": 2, "keys_per_split": 2112, "tiles_per_wg": 2, "waves": 8},
        "kernels": "k_attn_mfma<1,8,4> + k_attn_combine<2,1>",
        "profile": "profiles/other_workloads_layer_step.md"},
}


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 100; 64 for the decode workloads)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4",
                    choices=["c2", "c3", "c4", "c5", "c5_refresh", "c4_layer", "c2_layer", "c3_layer", "c5_layer",
                             "c5_refresh_layer", "c4_unmask", "c5_unmask", "c4_accept", "c5_drift", "c5_decode",
                             "c5_decode_model"])
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single", action="store_true",
                    help="skip the single-cache loops (for counter runs: every dispatch then streams from HBM)")
    ap.add_argument("--no-others", action="store_true",
                    help="default workload only: skip the compact figures of the other configurations")
    ap.add_argument("--repeats", type=int, default=5, help="timed repetitions; the median is reported")
    return ap.parse_args()


def _graph_of(torch, n, fn):
    """Record n calls of fn(s) into one HIP graph (the library issues no memset node and never
    synchronises, so its calls can be captured as they are).  Returns the graph."""
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for s in range(min(n, 3)):
            fn(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            for s in range(n):
                fn(s)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    return g


def _time_replays(torch, g, n, repeats):
    """Median over repeats of the per-step time (us) of one replay of a graph of n steps, between two
    events on the stream the graph is launched on."""
    res = []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        res.append(e0.elapsed_time(e1) * 1000.0 / n)
    res.sort()
    return res[len(res) // 2]


def hot_path(torch, fc, inputs, dev, wname, steps, warmup, repeats, layers=0, no_single=False):
    """The hot path (projection + RoPE + scatter, then attention) of one configuration, rotating over
    distinct layers.  Returns the measured figures as a dict."""
    refresh = wname == "c5_refresh"
    w = {"c2": inputs.C2, "c3": inputs.C3, "c4": inputs.C4, "c5": inputs.C5, "c5_refresh": inputs.C5}[wname]
    B, Dh, Hq, Hkv = w.batch, w.head_dim, w.n_q_heads, w.n_kv_heads
    A = w.gen_len if refresh else w.active  # a refresh re-projects the whole generation region
    S = w.kv_len
    esz = 2
    kv_bytes_layer = 2 * B * S * Hkv * Dh * esz
    w_bytes_layer = w.qkv_width * w.hidden * esz
    n_layers = layers or max(4, math.ceil(1.6e9 / (kv_bytes_layer + w_bytes_layer)))
    tdt = inputs.TORCH_DTYPE[w.dtype]

    cfg = fc.make_config(n_layers, B, w.hidden, Hq, Hkv, Dh, S, w.dtype, w.rope_base)
    nbytes = fc.fc_cache_storage_bytes(cfg)
    k_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    v_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    cache = fc.fc_cache_alloc(cfg, k_store, v_store)
    ws_bytes = fc.fc_workspace_bytes(cfg, A)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    # seeded inputs: layer 0 from the shared generators, the other layers are device copies of it
    # (distinct memory, same statistics)
    K0, V0 = inputs.kv_fill(w, 0, S)
    K0d, V0d = K0.to(dev), V0.to(dev)
    W0 = inputs.weights(w, 0).to(dev)
    Ws = [W0] + [W0.clone() for _ in range(n_layers - 1)]
    for layer in range(n_layers):
        fc.fc_cache_write_rows(cache, layer, K0d, V0d, 0, S)
    n_x = 8
    Xs = [inputs.hidden_states(w, 0, A, tag="x.%d" % i).to(dev) for i in range(n_x)]
    Q = torch.empty((B, Hq, A, Dh), dtype=tdt, device=dev)
    O = torch.empty((B, A, Hq * Dh), dtype=tdt, device=dev)
    torch.cuda.synchronize()

    if refresh:
        sched = [w.cached_len]
    elif w.gen_len:
        n_sched = -(-w.gen_len // w.block) * w.steps_per_block
        sched = [fc.fc_window(s, w.cached_len, w.gen_len, w.block, w.steps_per_block)[0] for s in range(n_sched)]
    else:
        sched = [w.cached_len]

    def step(s, rotate=True, do_proj=True, do_attn=True):
        layer = s % n_layers if rotate else 0
        if do_proj:
            fc.fc_qkv_project_scatter(cache, layer, Xs[s % n_x], Ws[layer], None, sched[s % len(sched)], A, None, Q)
        if do_attn:
            fc.fc_active_attention(cache, layer, Q, A, S, None, O, ws, ws_bytes)

    def timed_eager(n, **kw):
        res = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for s in range(n):
                step(s, **kw)
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1000.0 / n)
        res.sort()
        return res[len(res) // 2]

    for s in range(warmup):
        step(s)
    torch.cuda.synchronize()

    # Eager: exactly `steps` steps launched one by one from the host (four kernels per step).
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_host0 = time.perf_counter()
    e0.record()
    for s in range(steps):
        step(s)
    e1.record()
    torch.cuda.synchronize()
    t_host = time.perf_counter() - t_host0
    us_step_eager = e0.elapsed_time(e1) * 1000.0 / steps

    # The headline: the same `steps` steps (rotating layers, the window moving as scheduled) recorded
    # once into a HIP graph and replayed, so the host's launch rate is out of the figure; one replay =
    # exactly `steps` steps between two events, synchronised on both sides.
    g_all = _graph_of(torch, steps, step)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    g_all.replay()
    e1.record()
    torch.cuda.synchronize()
    us_step = e0.elapsed_time(e1) * 1000.0 / steps
    us_step_med = _time_replays(torch, g_all, steps, repeats)

    # per-call figures, same launch configuration, each its own replayed loop
    g_attn = _graph_of(torch, steps, lambda s: step(s, do_proj=False))
    us_attn = _time_replays(torch, g_attn, steps, repeats)
    g_proj = _graph_of(torch, steps, lambda s: step(s, do_attn=False))
    us_proj = _time_replays(torch, g_proj, steps, repeats)
    us_attn_eager = timed_eager(steps, do_proj=False)
    us_single = us_attn_single = float("nan")
    if not no_single:
        us_single = timed_eager(steps, rotate=False)
        us_attn_single = timed_eager(steps, rotate=False, do_proj=False)
    del g_all, g_attn, g_proj

    plan = fc.fc_attention_plan(cfg, A, S)
    res = dict(w=w, refresh=refresh, B=B, A=A, S=S, Hq=Hq, Hkv=Hkv, Dh=Dh, n_layers=n_layers, steps=steps, warmup=warmup,
               us_step=us_step, us_step_med=us_step_med, us_step_eager=us_step_eager, us_attn=us_attn, us_proj=us_proj,
               us_attn_eager=us_attn_eager, us_single=us_single, us_attn_single=us_attn_single,
               host_us=t_host * 1e6 / steps, plan=plan,
               attn_bytes=kv_bytes_layer + 2 * B * A * Hq * Dh * esz,
               proj_bytes=w_bytes_layer + B * A * (w.hidden + w.qkv_width) * esz,
               proj_flops=2.0 * B * A * w.hidden * w.qkv_width, attn_flops=4.0 * B * A * Hq * S * Dh)
    torch.cuda.synchronize()
    fc.fc_cache_free(cache)
    del k_store, v_store, Ws, W0, K0d, V0d, Xs, Q, O, ws
    torch.cuda.empty_cache()
    return res


def _traffic(r):
    """HBM bytes of the attention call, if a counter run of this workload with this launch plan is on
    file (profiles/): otherwise null rather than a figure of another kernel or plan."""
    rec = MEASURED_ATTENTION_TRAFFIC.get(r["w"].name)
    if rec is None or r["refresh"]:
        return None, None
    same = all(r["plan"][k] == v for k, v in rec["plan"].items())
    if not same:
        return None, "no counter run on file for plan %s" % r["plan"]
    return rec["bytes"], {"profile": rec["profile"], "plan": rec["plan"], "kernels": rec["kernels"]}


def hot_path_json(r, args_layers_note=""):
    w, refresh = r["w"], r["refresh"]
    us_step, us_attn, us_proj = r["us_step"], r["us_attn"], r["us_proj"]
    attn_gbs = r["attn_bytes"] / us_attn * 1e-3
    traffic, traffic_src = _traffic(r)
    nan_none = lambda v, nd=3: None if v != v else round(v, nd)
    out = {
        "metric": "us per cached denoising layer-step + achieved KV-read HBM GB/s (fraction of peak)",
        "value": round(us_step, 3),
        "unit": "us",
        "n_gpus": 1,
        "steps": r["steps"],
        "warmup": r["warmup"],
        "ms_per_step": round(us_step / 1000.0, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": w.name + ("/refresh" if refresh else ""), "batch": r["B"], "hidden": w.hidden,
            "n_q_heads": r["Hq"], "n_kv_heads": r["Hkv"], "head_dim": r["Dh"], "kv_len": r["S"], "active_rows": r["A"],
            "layers_rotated": r["n_layers"],
            "window_schedule": "start %d, +%d every %d steps" % (w.cached_len, w.block, w.steps_per_block)
            if w.gen_len else "fixed at %d" % w.cached_len,
            "launch": "the timed steps are recorded into one HIP graph and replayed once",
        },
        "roofline": {
            "kernel": "fc_active_attention (k_attn_mfma + k_attn_combine)",
            "bound": "hbm",
            "achieved": round(attn_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(attn_gbs / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_src,
            "algorithmic_bytes_per_launch": r["attn_bytes"],
            "us_per_launch": round(us_attn, 3),
            "us_per_launch_eager": round(r["us_attn_eager"], 3),
            "launch_plan": r["plan"],
        },
        "projection": {
            "kernel": "fc_qkv_project_scatter",
            "us_per_launch": round(us_proj, 3),
            "weight_stream_gbs": round(r["proj_bytes"] / us_proj * 1e-3, 1),
            "frac_of_hbm_peak": round(r["proj_bytes"] / us_proj * 1e-3 / HBM_PEAK_GBS, 4),
            "tflops": round(r["proj_flops"] / us_proj * 1e-6, 1),
            "frac_of_mfma_peak": round(r["proj_flops"] / us_proj * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
        },
        "active_rows_per_s": round(r["B"] * r["A"] / (us_step * 1e-6), 1),
        "tflops": round((r["proj_flops"] + r["attn_flops"]) / us_step * 1e-6, 2),
        "graph_us_per_step_median": round(r["us_step_med"], 3),
        "eager_us_per_step": round(r["us_step_eager"], 3),
        "host_wall_us_per_step": round(r["host_us"], 2),
        "single_cache_us": nan_none(r["us_single"]),
        "single_cache_attention_us": nan_none(r["us_attn_single"]),
        "single_cache_attention_gbs": None if r["us_attn_single"] != r["us_attn_single"]
        else round(r["attn_bytes"] / r["us_attn_single"] * 1e-3, 1),
    }
    if refresh:
        # the refresh is a dense pass: both calls are bound by the matrix cores, the projection GEMM
        # being the longer one
        out["roofline"] = {
            "kernel": "fc_qkv_project_scatter (k_proj_gemm)",
            "bound": "mfma",
            "achieved": round(r["proj_flops"] / us_proj * 1e-6, 1),
            "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(r["proj_flops"] / us_proj * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": None,
            "algorithmic_flops_per_launch": r["proj_flops"],
            "us_per_launch": round(us_proj, 3),
        }
        out["attention"] = {
            "kernel": "fc_active_attention",
            "us_per_launch": round(us_attn, 3),
            "tflops": round(r["attn_flops"] / us_attn * 1e-6, 1),
            "frac_of_mfma_peak": round(r["attn_flops"] / us_attn * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
        }
    return out


def others_summary(args, torch, fc, inputs, dev):
    """The other configurations in the same run, compact: value and roofline fraction each."""
    res = {}
    for name in ("c2", "c3", "c5", "c5_refresh"):
        r = hot_path(torch, fc, inputs, dev, name, steps=20 if name == "c5_refresh" else 40, warmup=8, repeats=3,
                     no_single=True)
        j = hot_path_json(r)
        res[name] = {"workload": j["config"]["workload"], "us_per_step": j["value"],
                     "attention_us": round(r["us_attn"], 3), "projection_us": round(r["us_proj"], 3),
                     "roofline_bound": j["roofline"]["bound"], "roofline_kernel": j["roofline"]["kernel"],
                     "roofline_frac": j["roofline"]["frac"],
                     "attention_kv_gbs": round(r["attn_bytes"] / r["us_attn"] * 1e-3, 1)}
    sub = argparse.Namespace(**vars(args))
    sub.workload, sub.steps, sub.warmup, sub.repeats, sub.no_cpu_baseline = "c5_decode", 64, 8, 3, True
    d = main_decode(sub, torch, fc, inputs, dev)
    res["c5_decode"] = {"workload": d["config"]["workload"], "tokens_per_s": d["value"], "ms_per_28_layer_step": d["ms_per_step"],
                        "roofline_frac": d["roofline"]["frac"], "initial_pass_ms": d["initial_pass_ms"]}
    return res


def main():
    args = _parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_21467_amd import binding as fc
    from paper_2505_21467_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fc.lib()
    dev = torch.device("cuda:0")
    if args.workload.startswith("c5_decode"):
        args.steps = 64 if args.steps is None else args.steps
        print(json.dumps(main_decode(args, torch, fc, inputs, dev)))
        return
    args.steps = 100 if args.steps is None else args.steps
    if args.workload.endswith("_layer"):
        return main_layer(args, torch, fc, inputs, dev)
    if args.workload.endswith("_unmask"):
        return main_unmask(args, torch, fc, inputs, dev)
    if args.workload.endswith("_accept"):
        return main_accept(args, torch, fc, inputs, dev)
    if args.workload.endswith("_drift"):
        return main_drift(args, torch, fc, inputs, dev)

    r = hot_path(torch, fc, inputs, dev, args.workload, args.steps, args.warmup, args.repeats, args.layers, args.no_single)
    out = hot_path_json(r)

    # A plain elementwise copy kernel of known size, so that a counter run of this same command
    # (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) can be scaled: 256 MiB read and 256 MiB written.
    cal_src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        torch.add(cal_src, 1.0, out=cal_dst)  # an elementwise kernel: reads 256 MiB, writes 256 MiB
    torch.cuda.synchronize()
    out["calibration_copy_bytes"] = cal_src.numel() * 4
    del cal_src, cal_dst

    if args.workload == "c4" and not args.no_others:
        out["others"] = others_summary(args, torch, fc, inputs, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(r["w"], inputs, r["A"], r["refresh"])
    print(json.dumps(out))


def main_layer(args, torch, fc, inputs, dev):
    """Whole-layer workloads: one fc_full_layer_step per step, rotating over distinct layers."""
    w = {"c4_layer": inputs.C4, "c2_layer": inputs.C2, "c3_layer": inputs.C3, "c5_layer": inputs.C5,
         "c5_refresh_layer": inputs.C5}[args.workload]
    refresh = args.workload == "c5_refresh_layer"
    B, Dh, Hq, Hkv, d, F = w.batch, w.head_dim, w.n_q_heads, w.n_kv_heads, w.hidden, w.d_ff
    A, S, E, esz = (w.gen_len if refresh else w.active), w.kv_len, w.n_q_heads * w.head_dim, 2
    M = B * A
    tdt = inputs.TORCH_DTYPE[w.dtype]
    w_bytes = {"w_qkv": w.qkv_width * d * esz, "w_out": d * E * esz, "gate_up": 2 * F * d * esz, "w_down": d * F * esz}
    kv_bytes_layer = 2 * B * S * Hkv * Dh * esz
    layer_bytes = sum(w_bytes.values()) + kv_bytes_layer
    n_layers = args.layers or max(4, math.ceil(2.4e9 / layer_bytes))
    steps = min(args.steps, 60)

    cfg = fc.make_config(n_layers, B, d, Hq, Hkv, Dh, S, w.dtype, w.rope_base)
    nbytes = fc.fc_cache_storage_bytes(cfg)
    k_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    v_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    cache = fc.fc_cache_alloc(cfg, k_store, v_store)
    K0, V0 = inputs.kv_fill(w, 0, S)
    K0d, V0d = K0.to(dev), V0.to(dev)
    for layer in range(n_layers):
        fc.fc_cache_write_rows(cache, layer, K0d, V0d, 0, S)
    # layer 0 from the shared generators, the other layers are device copies (distinct memory)
    host = inputs.layer_weights(w, 0)
    layers = []
    for layer in range(n_layers):
        t = {k: (None if v is None else (v.to(dev) if layer == 0 else layers[0][0][k].clone())) for k, v in host.items()}
        h = fc.make_layer_weights(t["norm1"], t["w_qkv"], t["b_qkv"], t["w_out"], t["norm2"], t["w_gate"], t["w_up"],
                                  t["w_down"], F, w.norm_eps)
        layers.append((t, h))
    ws_bytes = fc.fc_full_layer_workspace_bytes(cfg, F, A)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    n_x = 8
    Xs = [inputs.hidden_states(w, 0, A, tag="x.%d" % i).to(dev) for i in range(n_x)]
    Y = torch.empty((B, A, d), dtype=tdt, device=dev)
    if w.gen_len and not refresh:
        n_sched = -(-w.gen_len // w.block) * w.steps_per_block
        sched = [fc.fc_window(s, w.cached_len, w.gen_len, w.block, w.steps_per_block)[0] for s in range(n_sched)]
    else:
        sched = [w.cached_len]
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()

    def step(s):
        layer = s % n_layers
        fc.fc_full_layer_step(cache, layer, layers[layer][1], Xs[s % n_x], sched[s % len(sched)], A, None, S, Y, ws,
                              ws_bytes, stream)

    def timed(fn, n):
        res = []
        for _ in range(args.repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for s in range(n):
                fn(s)
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1000.0 / n)
        res.sort()
        return res[len(res) // 2]

    for s in range(min(args.warmup, 2 * n_layers)):
        step(s)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_host0 = time.perf_counter()
    e0.record()
    for s in range(steps):
        step(s)
    e1.record()
    torch.cuda.synchronize()
    t_host = time.perf_counter() - t_host0
    us_step = e0.elapsed_time(e1) * 1000.0 / steps

    # the three weight-streaming calls on their own, same rotation (each is GPU-bound at these sizes)
    lin_ws_bytes = max(fc.fc_linear_workspace_bytes(w.dtype, M, E, d), fc.fc_linear_workspace_bytes(w.dtype, M, d, 2 * F),
                       fc.fc_linear_workspace_bytes(w.dtype, M, F, d))
    lws = torch.empty(max(lin_ws_bytes, 16), dtype=torch.uint8, device=dev)
    h = Xs[0].view(M, d)
    o = torch.randn((M, E), device=dev).to(tdt)
    act = torch.randn((M, F), device=dev).to(tdt)
    x2 = torch.empty((M, d), dtype=tdt, device=dev)
    actb = torch.empty((M, F), dtype=tdt, device=dev)
    L = lambda s: layers[s % n_layers][0]
    us_out = timed(lambda s: fc.fc_linear_residual(w.dtype, o, L(s)["w_out"], h, M, E, d, x2, lws, lin_ws_bytes, stream), steps)
    us_gate = timed(lambda s: fc.fc_ffn_gate_up(w.dtype, h, L(s)["w_gate"], L(s)["w_up"], M, d, F, actb, lws,
                                                lin_ws_bytes, stream), steps)
    us_down = timed(lambda s: fc.fc_linear_residual(w.dtype, act, L(s)["w_down"], h, M, F, d, x2, lws, lin_ws_bytes,
                                                    stream), steps)

    total_w = sum(w_bytes.values())
    flops = 2.0 * M * (d * w.qkv_width + E * d + 3 * d * F) + 4.0 * M * Hq * S * Dh
    gate_flops = 4.0 * M * d * F
    gbs = lambda nbytes, us: round(nbytes / us * 1e-3, 1)
    # the gated W_1 is the longest call: bound by the weight stream for a block of rows, by the matrix
    # cores for a refresh of thousands of rows
    if M >= 1024:
        roof = {"kernel": "fc_ffn_gate_up (k_proj_gemm, SiLU-gate epilogue)", "bound": "mfma",
                "achieved": round(gate_flops / us_gate * 1e-6, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(gate_flops / us_gate * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "algorithmic_flops_per_launch": gate_flops, "us_per_launch": round(us_gate, 3)}
    else:
        roof = {"kernel": "fc_ffn_gate_up (%s)" % ("k_linear_rows" if M <= 32 else
                                                   "k_proj_gemm, SiLU-gate epilogue"), "bound": "hbm",
                "achieved": gbs(w_bytes["gate_up"], us_gate), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(w_bytes["gate_up"] / us_gate * 1e-3 / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_GATE_UP_TRAFFIC_BYTES.get((M, d, F)),
                "algorithmic_bytes_per_launch": w_bytes["gate_up"] + M * (d + F) * esz,
                "us_per_launch": round(us_gate, 3), "tflops": round(gate_flops / us_gate * 1e-6, 1)}
    out = {
        "metric": "us per cached denoising step of one whole transformer layer on the window rows",
        "value": round(us_step, 3), "unit": "us", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 2 * n_layers),
        "ms_per_step": round(us_step / 1000.0, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + ("/refresh" if refresh else "") + "/whole-layer", "batch": B, "hidden": d, "d_ff": F, "n_q_heads": Hq,
                   "n_kv_heads": Hkv, "head_dim": Dh, "kv_len": S, "active_rows": A, "layers_rotated": n_layers,
                   "weight_bytes_per_layer": total_w, "kv_bytes_per_layer": kv_bytes_layer},
        "roofline": roof,
        "linear_calls": {
            "w_out": {"us_per_launch": round(us_out, 3), "weight_stream_gbs": gbs(w_bytes["w_out"], us_out),
                      "tflops": round(2.0 * M * E * d / us_out * 1e-6, 1)},
            "gate_up": {"us_per_launch": round(us_gate, 3), "weight_stream_gbs": gbs(w_bytes["gate_up"], us_gate),
                        "tflops": round(gate_flops / us_gate * 1e-6, 1)},
            "w_down": {"us_per_launch": round(us_down, 3), "weight_stream_gbs": gbs(w_bytes["w_down"], us_down),
                       "tflops": round(2.0 * M * F * d / us_down * 1e-6, 1)},
        },
        "layer_stream_gbs": gbs(total_w + kv_bytes_layer, us_step),
        "layer_frac_of_hbm_peak": round((total_w + kv_bytes_layer) / us_step * 1e-3 / HBM_PEAK_GBS, 4),
        "active_rows_per_s": round(M / (us_step * 1e-6), 1),
        "tflops": round(flops / us_step * 1e-6, 2),
        "host_wall_us_per_step": round(t_host * 1e6 / steps, 2),
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import fc_oracle as orc
        # bounded sample: the first sequence of the batch and at most 32 of its window rows (the layer is
        # row-wise apart from attention, whose cost per row does not depend on the row count); the value
        # is the sample's time scaled to all B * A rows
        As = min(A, 32)
        ocfg = orc.OracleConfig(1, d, Hq, Hkv, Dh, S, w.dtype, w.rope_base)
        Kc, Vc = inputs.as_oracle(K0)[:1].copy(), inputs.as_oracle(V0)[:1].copy()
        wts = {k: (None if v is None else inputs.as_oracle(v)) for k, v in host.items()}
        pos = inputs.as_oracle(inputs.window_positions(1, w.cached_len, As))
        X = inputs.as_oracle(inputs.hidden_states(w, 0, A, tag="x.0"))[:1, :As].copy()
        n_sample, dt = 0, 0.0
        while n_sample < 20 and dt < 12.0:
            t0 = time.perf_counter()
            orc.full_layer_step(ocfg, X, wts, pos, S, Kc, Vc, w.norm_eps)
            dt += time.perf_counter() - t0
            n_sample += 1
        scale = M / float(As)
        out["cpu_baseline"] = {"value": round(dt * 1e6 / n_sample * scale, 1), "unit": "us", "cores": orc.get_threads(),
                               "kind": "oracle",
                               "sample": "%d whole-layer step(s) of %d row(s) of one sequence of %s, fp64, OpenMP; "
                                         "scaled by %g to the %d rows of a step" % (n_sample, As, w.name, scale, M)}
        del np
    torch.cuda.synchronize()
    fc.fc_cache_free(cache)
    print(json.dumps(out))


def main_decode(args, torch, fc, inputs, dev):
    """The block schedule of configuration 5 over all 28 layers; value = decoded tokens/s.

    A step is one denoising step (section 3.2.1: the active block of 32 rows in every layer) and, when
    the step completes a block (every 8th), the refresh of the 256-row generation region in every
    layer.  `c5_decode`: projection + scatter + attention only, per-layer synthetic activations.
    `c5_decode_model`: token embeddings -> 28 whole layers -> final norm -> vocabulary projection with
    arg-max -> confidence-ranked fill of 4 tokens per sequence (section 3.1)."""
    w = inputs.C5
    whole = args.workload == "c5_decode_model"
    B, Dh, Hq, Hkv, d, F, NL = w.batch, w.head_dim, w.n_q_heads, w.n_kv_heads, w.hidden, w.d_ff, w.n_layers
    P, G, Bk, spb = w.cached_len, w.gen_len, w.block, w.steps_per_block
    S, A, esz, V = P + G, Bk, 2, 152064
    k_fill, MASK = Bk // spb, V
    n_sched = (G // Bk) * spb
    tdt = inputs.TORCH_DTYPE[w.dtype]
    stream = torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device=dev)
    gen.manual_seed(20250521)
    rnd = lambda shape, std: (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(tdt)

    cfg = fc.make_config(NL, B, d, Hq, Hkv, Dh, S, w.dtype, w.rope_base)
    nbytes = fc.fc_cache_storage_bytes(cfg)
    k_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    v_store = torch.zeros(nbytes // esz, dtype=tdt, device=dev)
    cache = fc.fc_cache_alloc(cfg, k_store, v_store)

    if whole:
        layers = []
        for layer in range(NL):
            t = {"norm1": (1.0 + 0.1 * torch.randn(d, generator=gen, device=dev)).to(tdt), "w_qkv": rnd((w.qkv_width, d), 0.02),
                 "w_out": rnd((d, Hq * Dh), 0.02), "norm2": (1.0 + 0.1 * torch.randn(d, generator=gen, device=dev)).to(tdt),
                 "w_gate": rnd((F, d), 0.02), "w_up": rnd((F, d), 0.02), "w_down": rnd((d, F), 0.02)}
            layers.append((t, fc.make_layer_weights(t["norm1"], t["w_qkv"], None, t["w_out"], t["norm2"], t["w_gate"],
                                                    t["w_up"], t["w_down"], F, w.norm_eps)))
        emb = rnd((V + 1, d), 1.0)                     # row V = the mask embedding
        w_vocab = rnd((V, d), 0.02)
        final_norm = (1.0 + 0.1 * torch.randn(d, generator=gen, device=dev)).to(tdt)
        tokens0 = torch.full((B, S), MASK, dtype=torch.int32, device=dev)
        tokens0[:, :P] = torch.randint(0, V, (B, P), generator=gen, device=dev, dtype=torch.int32)
        tokens = tokens0.clone()
        ws_bytes = fc.fc_full_layer_workspace_bytes(cfg, F, S)
        lm_bytes = fc.fc_lm_head_workspace_bytes(w.dtype, B * A, d, V)
        lm_ws = torch.empty(max(lm_bytes, 16), dtype=torch.uint8, device=dev)
        tok = torch.empty((B * A,), dtype=torch.int32, device=dev)
        conf = torch.empty((B * A,), dtype=torch.float32, device=dev)
        pos_next = torch.empty((B, A), dtype=torch.int32, device=dev)
        count = torch.empty((B,), dtype=torch.int32, device=dev)
        bufs = {r: (torch.empty((B, r, d), dtype=tdt, device=dev), torch.empty((B, r, d), dtype=tdt, device=dev))
                for r in (A, G, S)}
    else:
        W0 = inputs.weights(w, 0).to(dev)
        Ws = [W0] + [W0.clone() for _ in range(NL - 1)]
        Xs = [inputs.hidden_states(w, 0, A, tag="x.%d" % i).to(dev) for i in range(8)]
        Xr = [rnd((B, G, d), 1.0) for _ in range(2)]
        Xall = rnd((B, S, d), 1.0)
        ws_bytes = fc.fc_workspace_bytes(cfg, S)
        Q = {r: torch.empty((B, Hq, r, Dh), dtype=tdt, device=dev) for r in (A, G, S)}
        O = {r: torch.empty((B, r, Hq * Dh), dtype=tdt, device=dev) for r in (A, G, S)}
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def forward(start, rows, n):
        """All layers on the window [start, start + rows) of every sequence; returns the last hidden states."""
        if not whole:
            x = Xs[n % 8] if rows == A else (Xr[n % 2] if rows == G else Xall)
            for layer in range(NL):
                fc.fc_qkv_project_scatter(cache, layer, x, Ws[layer], None, start, rows, None, Q[rows], stream)
                fc.fc_active_attention(cache, layer, Q[rows], rows, S, None, O[rows], ws, ws_bytes, stream)
            return None
        x, y = bufs[rows]
        for b in range(B):  # the window's token ids of a sequence are contiguous: one embedding gather each
            fc.fc_gather_rows(w.dtype, emb, V + 1, d, tokens[b, start:start + rows], rows, x[b], stream)
        for layer in range(NL):
            fc.fc_full_layer_step(cache, layer, layers[layer][1], x, start, rows, None, S, y, ws, ws_bytes, stream)
            x, y = y, x
        return x

    def step(n):
        s_idx = n % n_sched
        if whole and s_idx == 0:
            tokens.copy_(tokens0)                                  # a new generation: everything masked again
        start, rows, _ = fc.fc_window(s_idx, P, G, Bk, spb, 0, 0)
        h = forward(start, rows, n)
        if whole:
            hb = h.view(B * A, d)
            fc.fc_rmsnorm(w.dtype, hb, final_norm, w.norm_eps, B * A, d, hb, stream)
            fc.fc_lm_head_argmax(w.dtype, hb, w_vocab, B * A, d, V, tok, conf, lm_ws, lm_bytes, stream)
            fc.fc_unmask_select(tok, conf, None, start, B, A, k_fill, MASK, tokens, S, pos_next, count, stream)
        if s_idx % spb == spb - 1:
            forward(P, G, n)                                       # the block is complete: refresh the generation region

    # initial pass over prompt + generation region (all rows projected and cached), untimed but reported
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    forward(0, S, 0)
    torch.cuda.synchronize()
    init_ms = (time.perf_counter() - t0) * 1e3

    for n in range(args.warmup):
        step(n)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    e0.record()
    for n in range(args.steps):
        step(n)
    e1.record()
    torch.cuda.synchronize()
    t_host = time.perf_counter() - t_host0
    ms_total = e0.elapsed_time(e1)
    tokens_done = args.steps * B * k_fill
    n_refresh = sum(1 for n in range(args.steps) if (n % n_sched) % spb == spb - 1)

    # the attention call of the cached step on its own (rotating over the 28 layers), for the roofline
    if whole:
        Qa = torch.randn((B, Hq, A, Dh), generator=gen, device=dev).to(tdt)
        Oa = torch.empty((B, A, Hq * Dh), dtype=tdt, device=dev)
    else:
        Qa, Oa = Q[A], O[A]
    res = []
    for _ in range(args.repeats):
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a0.record()
        for n in range(2 * NL):
            fc.fc_active_attention(cache, n % NL, Qa, A, S, None, Oa, ws, ws_bytes, stream)
        a1.record()
        torch.cuda.synchronize()
        res.append(a0.elapsed_time(a1) * 1000.0 / (2 * NL))
    us_attn = sorted(res)[len(res) // 2]
    attn_bytes = 2 * B * S * Hkv * Dh * esz + 2 * B * A * Hq * Dh * esz
    roof = {"kernel": "fc_active_attention of the cached step (k_attn_mfma + k_attn_combine)", "bound": "hbm",
            "achieved": round(attn_bytes / us_attn * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(attn_bytes / us_attn * 1e-3 / HBM_PEAK_GBS, 4), "traffic": None,
            "algorithmic_bytes_per_launch": attn_bytes, "us_per_launch": round(us_attn, 3)}
    if whole:
        # the longest call of a whole-layer cached step is the gated W_1 on the 256 window rows
        M = B * A
        lin_bytes = fc.fc_linear_workspace_bytes(w.dtype, M, d, 2 * F)
        lws = torch.empty(max(lin_bytes, 16), dtype=torch.uint8, device=dev)
        hx, actb = bufs[A][0].view(M, d), torch.empty((M, F), dtype=tdt, device=dev)
        res = []
        for _ in range(args.repeats):
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a0.record()
            for n in range(2 * NL):
                t = layers[n % NL][0]
                fc.fc_ffn_gate_up(w.dtype, hx, t["w_gate"], t["w_up"], M, d, F, actb, lws, lin_bytes, stream)
            a1.record()
            torch.cuda.synchronize()
            res.append(a0.elapsed_time(a1) * 1000.0 / (2 * NL))
        us_gate = sorted(res)[len(res) // 2]
        gate_bytes = 2 * F * d * esz + M * (d + F) * esz
        roof = {"kernel": "fc_ffn_gate_up of the cached step (k_proj_gemm, SiLU-gate epilogue, 256 rows)", "bound": "hbm",
                "achieved": round(gate_bytes / us_gate * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gate_bytes / us_gate * 1e-3 / HBM_PEAK_GBS, 4), "traffic": None,
                "algorithmic_bytes_per_launch": gate_bytes, "us_per_launch": round(us_gate, 3),
                "tflops": round(4.0 * M * d * F / us_gate * 1e-6, 1), "attention_us_per_launch": round(us_attn, 3)}

    if whole:
        # bookkeeping check: every step of the last generation filled 4 tokens per sequence
        done = (args.steps - 1) % n_sched + 1
        assert int((tokens[:, P:] == MASK).sum()) == B * G - done * B * k_fill, "fill bookkeeping"
    out = {
        "metric": "decoded tokens/s, 28-layer block schedule (%s)" % (
            "whole layers + unmasking, synthetic 7B-shaped model" if whole else "projection + scatter + attention per layer"),
        "value": round(tokens_done / (ms_total * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_total / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + ("/decode-model" if whole else "/decode"), "batch": B, "layers": NL, "prompt": P,
                   "generated": G, "block": Bk, "steps_per_block": spb, "tokens_per_step_and_sequence": k_fill,
                   "refreshes_in_timed_region": n_refresh, "hidden": d, "d_ff": F if whole else None,
                   "vocab": V if whole else None},
        "roofline": roof,
        "initial_pass_ms": round(init_ms, 2),
        "host_wall_ms_per_step": round(t_host * 1e3 / args.steps, 4),
    }
    if not args.no_cpu_baseline:
        # bounded sample: cached layer-steps of the hot path (projection + scatter + attention) on the
        # oracle, scaled to 28 layers; the refreshes and (for the model variant) the rest of the layer and
        # the vocabulary projection are left out, so the oracle's real rate is lower still
        cb = cpu_baseline(w, inputs, A, False)
        out["cpu_baseline"] = {"value": round(B * k_fill / (NL * cb["value"] * 1e-6), 3), "unit": "tokens/s",
                               "cores": cb["cores"], "kind": "oracle",
                               "sample": cb["sample"] + "; scaled to 28 layers per step, refreshes not included"}
    torch.cuda.synchronize()
    fc.fc_cache_free(cache)
    return out


def main_unmask(args, torch, fc, inputs, dev):
    """Unmasking step of one block: vocabulary projection (arg-max + confidence) and confidence-ranked fill."""
    w = {"c4_unmask": inputs.C4, "c5_unmask": inputs.C5}[args.workload]
    B, A, d, V, esz = w.batch, w.active, w.hidden, 152064, 2
    M, L, MASK, k = B * A, w.kv_len, V - 1, 4
    tdt = inputs.TORCH_DTYPE[w.dtype]
    n_mats = args.layers or 3                      # 1.09 GB each: the stream always comes from HBM
    steps = min(args.steps, 30)
    W0 = inputs.normal(0, "w_vocab", (V, d), 0.02, w.dtype).to(dev)
    Ws = [W0] + [W0.clone() for _ in range(n_mats - 1)]
    Xs = [inputs.hidden_states(w, 0, A, tag="h.%d" % i).to(dev).view(M, d) for i in range(4)]
    need = fc.fc_lm_head_workspace_bytes(w.dtype, M, d, V)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    tok = torch.empty((M,), dtype=torch.int32, device=dev)
    conf = torch.empty((M,), dtype=torch.float32, device=dev)
    tokens = torch.full((B, L), MASK, dtype=torch.int32, device=dev)
    pos_next = torch.empty((B, A), dtype=torch.int32, device=dev)
    count = torch.empty((B,), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()

    def step(s, head=True, select=True):
        if head:
            fc.fc_lm_head_argmax(w.dtype, Xs[s % 4], Ws[s % n_mats], M, d, V, tok, conf, ws, need, stream)
        if select:
            fc.fc_unmask_select(tok, conf, None, w.cached_len, B, A, k, MASK, tokens, L, pos_next, count, stream)

    def timed(n, **kw):
        res = []
        for _ in range(args.repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for s in range(n):
                step(s, **kw)
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1000.0 / n)
        res.sort()
        return res[len(res) // 2]

    for s in range(min(args.warmup, 6)):
        step(s)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for s in range(steps):
        step(s)
    e1.record()
    torch.cuda.synchronize()
    us_step = e0.elapsed_time(e1) * 1000.0 / steps
    us_head = timed(steps, select=False)
    us_sel = timed(steps, head=False)
    w_bytes = V * d * esz
    out = {
        "metric": "us per unmasking step of one block (vocabulary projection with arg-max + confidence-ranked fill)",
        "value": round(us_step, 3), "unit": "us", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 6),
        "ms_per_step": round(us_step / 1000.0, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "/unmask", "batch": B, "block_rows": A, "hidden": d, "vocab": V,
                   "unmasked_per_step": k, "matrices_rotated": n_mats},
        "roofline": {"kernel": "fc_lm_head_argmax (%s + k_lmhead_reduce)" % (
                         "k_linear_rows" if M <= 32 else "k_proj_gemm with the arg-max epilogue"),
                     "bound": "hbm",
                     "achieved": round(w_bytes / us_head * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(w_bytes / us_head * 1e-3 / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_LM_HEAD_TRAFFIC_BYTES.get((M, d, V)),
                     "algorithmic_bytes_per_launch": w_bytes + M * d * esz + M * 8, "us_per_launch": round(us_head, 3),
                     "tflops": round(2.0 * M * d * V / us_head * 1e-6, 1)},
        "unmask_select_us": round(us_sel, 3),
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import fc_oracle as orc
        rows = 2   # bounded sample: two rows of the block against the whole vocabulary, scaled to M rows
        X = inputs.as_oracle(inputs.hidden_states(w, 0, A, tag="h.0")).reshape(M, d)[:rows].copy()
        Wv = inputs.as_oracle(inputs.normal(0, "w_vocab", (V, d), 0.02, w.dtype))
        t0 = time.perf_counter()
        orc.lm_head_argmax(X, Wv)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(dt * 1e6 * M / rows, 1), "unit": "us", "cores": orc.get_threads(),
                               "kind": "oracle", "sample": "vocabulary projection + arg-max of %d rows of %s, fp64, "
                               "OpenMP over rows; scaled by %g to the %d rows of a step" % (rows, w.name, M / rows, M)}
        del np
    print(json.dumps(out))


def main_accept(args, torch, fc, inputs, dev):
    """Guided Diffusion acceptance of one speculation block on synthetic logits (fp32, vocabulary 152064)."""
    w = inputs.C4
    B, A, V, topk, tau = w.batch, 32, 152064, 2, 0.5
    L, P, MASK = 64, 16, V + 1
    n_sets = args.layers or 16                     # 38.9 MB of logits each: 620 MB rotated
    steps = min(args.steps, 64)
    dlm0 = inputs.normal(0, "dlm_logits", (B, A, V), 3.0, "f32")
    ar0 = dlm0 + inputs.normal(0, "ar_noise", (B, A, V), 1.5, "f32")
    dlm = [dlm0.to(dev)] + [None] * (n_sets - 1)
    ar = [ar0.to(dev)] + [None] * (n_sets - 1)
    for i in range(1, n_sets):
        dlm[i], ar[i] = dlm[0].clone(), ar[0].clone()
    tokens0 = torch.full((B, L), MASK, dtype=torch.int32, device=dev)
    tokens0[:, :P] = 1
    tokens = tokens0.clone()
    need = fc.fc_guided_accept_workspace_bytes(B, A, V)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    pos_next = torch.empty((B, A), dtype=torch.int32, device=dev)
    count = torch.empty((B,), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()

    def step(s):
        # every call sees the whole block masked (the timed work does not shrink from step to step)
        tokens.copy_(tokens0)
        fc.fc_guided_accept(dlm[s % n_sets], ar[s % n_sets], None, P, B, A, V, topk, tau, MASK, tokens, L, n_acc,
                            pos_next, count, ws, need, stream)

    def run(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for s in range(n):
            step(s)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1000.0 / n

    for s in range(min(args.warmup, n_sets)):
        step(s)
    us_step = run(steps)
    # the token reset alone, to subtract it
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for s in range(steps):
        tokens.copy_(tokens0)
    e1.record()
    torch.cuda.synchronize()
    us_reset = e0.elapsed_time(e1) * 1000.0 / steps
    us_call = sorted(run(steps) for _ in range(args.repeats))[args.repeats // 2] - us_reset
    nbytes = 2 * B * A * V * 4
    out = {
        "metric": "us per Guided Diffusion acceptance step of one speculation block (synthetic logits)",
        "value": round(us_step, 3), "unit": "us", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, n_sets),
        "ms_per_step": round(us_step / 1000.0, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "c4_guided_accept_B%d_block%d_V%d" % (B, A, V), "batch": B, "block_rows": A, "vocab": V,
                   "topk": topk, "tau": tau, "logit_sets_rotated": n_sets, "includes_token_reset_us": round(us_reset, 3)},
        "roofline": {"kernel": "fc_guided_accept (k_accept_scan + k_accept_rowmerge + k_accept_seq)", "bound": "hbm",
                     "achieved": round(nbytes / us_call * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(nbytes / us_call * 1e-3 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": nbytes, "us_per_launch": round(us_call, 3)},
        "accepted_first_call": int(n_acc.sum().item()),
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import fc_oracle as orc
        host_tokens = tokens0.cpu().numpy().copy()
        pos = inputs.as_oracle(inputs.window_positions(B, P, A))
        t0 = time.perf_counter()
        orc.guided_accept(dlm0.numpy(), ar0.numpy(), pos, topk, tau, MASK, host_tokens)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(dt * 1e6, 1), "unit": "us", "cores": 1, "kind": "oracle",
                               "sample": "one acceptance step of the same block and logits, single thread"}
        del np
    print(json.dumps(out))


def main_drift(args, torch, fc, inputs, dev):
    """KV drift diagnostic of the generation region: snapshot before a step, similarity after it."""
    w = inputs.C5
    B, Hkv, Dh, S, rows, start, esz = w.batch, w.n_kv_heads, w.head_dim, w.kv_len, w.gen_len, w.cached_len, 2
    n_layers = args.layers or 28
    tdt = inputs.TORCH_DTYPE[w.dtype]
    cfg = fc.make_config(n_layers, B, w.hidden, w.n_q_heads, Hkv, Dh, S, w.dtype, w.rope_base)
    nbytes = fc.fc_cache_storage_bytes(cfg)
    k_store = torch.randn(nbytes // esz, device=dev).to(tdt)
    v_store = torch.randn(nbytes // esz, device=dev).to(tdt)
    cache = fc.fc_cache_alloc(cfg, k_store, v_store)
    kp = torch.empty((B, Hkv, rows, Dh), dtype=tdt, device=dev)
    vp = torch.empty_like(kp)
    sk = torch.empty((B, Hkv, rows), dtype=torch.float32, device=dev)
    sv = torch.empty_like(sk)
    stream = torch.cuda.current_stream().cuda_stream
    steps = args.steps

    def timed(fn):
        res = []
        for _ in range(args.repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for s in range(steps):
                fn(s % n_layers)
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1000.0 / steps)
        res.sort()
        return res[len(res) // 2]

    snap = lambda l: fc.fc_cache_read_rows(cache, l, kp, vp, start, rows, stream)
    sim = lambda l: fc.fc_kv_similarity(cache, l, kp, vp, start, rows, sk, sv, stream)
    for l in range(min(args.warmup, n_layers)):
        snap(l)
        sim(l)
    us_both = timed(lambda l: (snap(l), sim(l)))
    us_snap, us_sim = timed(snap), timed(sim)
    row_bytes = 2 * B * Hkv * rows * Dh * esz          # K and V rows of the region
    out = {
        "metric": "us per layer for the KV drift diagnostic of the generation region (snapshot + similarity)",
        "value": round(us_both, 3), "unit": "us", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, n_layers),
        "ms_per_step": round(us_both / 1000.0, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "/kv-drift", "batch": B, "n_kv_heads": Hkv, "head_dim": Dh, "rows": rows,
                   "layers_rotated": n_layers},
        "roofline": {"kernel": "fc_kv_similarity (k_kv_similarity)", "bound": "hbm",
                     "achieved": round(2 * row_bytes / us_sim * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(2 * row_bytes / us_sim * 1e-3 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": 2 * row_bytes, "us_per_launch": round(us_sim, 3)},
        "snapshot_us": round(us_snap, 3),
    }
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import fc_oracle as orc
        ocfg = orc.OracleConfig(B, w.hidden, w.n_q_heads, Hkv, Dh, S, w.dtype)
        Kg = np.zeros((B, Hkv, S, Dh), np.float32)
        Kg[:] = np.random.default_rng(0).normal(size=Kg.shape)
        prev = Kg[:, :, start:start + rows].copy()
        t0 = time.perf_counter()
        orc.kv_similarity(ocfg, Kg, Kg, prev, prev, start)
        out["cpu_baseline"] = {"value": round((time.perf_counter() - t0) * 1e6, 1), "unit": "us", "cores": 1,
                               "kind": "oracle", "sample": "similarity of the same 256-row region of one layer, single thread"}
    torch.cuda.synchronize()
    fc.fc_cache_free(cache)
    print(json.dumps(out))


def cpu_baseline(w, inputs, A, refresh):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import fc_oracle as orc

    max_samples, budget_s = 100, 10.0  # stop after about 10 s of oracle work
    S = w.kv_len
    cfg = orc.OracleConfig(w.batch, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, S, w.dtype, w.rope_base)
    K0, V0 = inputs.kv_fill(w, 0, S)
    Kc, Vc = inputs.as_oracle(K0).copy(), inputs.as_oracle(V0).copy()
    W = inputs.as_oracle(inputs.weights(w, 0))
    threads = orc.get_threads()
    pos = inputs.as_oracle(inputs.window_positions(w.batch, w.cached_len, A))
    Xs = [inputs.as_oracle(inputs.hidden_states(w, 0, A, tag="x.%d" % s)) for s in range(4)]
    n_sample, dt = 0, 0.0
    while n_sample < max_samples and dt < budget_s:
        t0 = time.perf_counter()
        orc.layer_step(cfg, Xs[n_sample % 4], W, None, pos, S, Kc, Vc)
        dt += time.perf_counter() - t0
        n_sample += 1
    return {
        "value": round(dt * 1e6 / n_sample, 1),
        "unit": "us",
        "cores": threads,
        "kind": "oracle",
        "sample": "%d layer-step(s) of %s%s (projection + scatter + attention), fp64, OpenMP" % (
            n_sample, w.name, "/refresh" if refresh else ""),
    }


if __name__ == "__main__":
    main()
