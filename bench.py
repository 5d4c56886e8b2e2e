"""Benchmark of the FreeCache cached denoising layer-step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c2|c3|c5|c5_refresh] [--layers N]

A "step" is one pass of the whole hot path for one layer: QKV projection + RoPE + scatter of the
active window, then attention of the window's queries over the cache.  The default workload is the
long-context Dream-7B-shaped configuration (prompt 16384, window of 32 rows sliding by 32 every 8
steps, 28/4 GQA heads, head_dim 128, bf16), on which the metric's bandwidth target is quoted.

So that the key/value stream really comes from HBM and not from the 256 MB memory-side cache, the
timed loop rotates over `--layers` distinct layer caches and weight matrices (default: enough for
more than 1.5 GB of working set), as a 28-layer model does between two visits of one layer.  The
same loop on a single layer is reported as `single_cache_us` (cache-resident figure).

`--workload c5_refresh` times the periodic refresh of configuration 5 instead (one `fc_refresh` of the
256-row generation region of 8 sequences per step: a dense, matrix-core-bound pass).

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
MEASURED_ATTENTION_TRAFFIC_BYTES = {
    "c4_dream7b_long_L16384_A32": 54_470_000,   # 36.47 + 7.31 MB (main kernel), 10.47 + 0.23 MB (merge)
    "c3_llada8b_B4_L4096_A64": 289_900_000,     # 277.0 + 4.46 MB, 6.35 + 2.10 MB
}


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5", "c5_refresh"])
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single", action="store_true",
                    help="skip the single-cache loops (for counter runs: every dispatch then streams from HBM)")
    ap.add_argument("--repeats", type=int, default=5, help="timed repetitions; the median is reported")
    return ap.parse_args()


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
    refresh = args.workload == "c5_refresh"
    w = {"c2": inputs.C2, "c3": inputs.C3, "c4": inputs.C4, "c5": inputs.C5, "c5_refresh": inputs.C5}[args.workload]
    B, Dh, Hq, Hkv = w.batch, w.head_dim, w.n_q_heads, w.n_kv_heads
    A = w.gen_len if refresh else w.active  # a refresh re-projects the whole generation region
    S = w.kv_len
    esz = 2
    kv_bytes_layer = 2 * B * S * Hkv * Dh * esz
    w_bytes_layer = w.qkv_width * w.hidden * esz
    n_layers = args.layers or max(4, math.ceil(1.6e9 / (kv_bytes_layer + w_bytes_layer)))
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

    def timed(n, **kw):
        """Median over repeats of the per-step time (us) of n back-to-back steps on the current stream."""
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

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()

    # the headline: exactly --steps steps between two events, barrier (sync) on both sides
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_host0 = time.perf_counter()
    e0.record()
    for s in range(args.steps):
        step(s)
    e1.record()
    torch.cuda.synchronize()
    t_host = time.perf_counter() - t_host0
    us_step = e0.elapsed_time(e1) * 1000.0 / args.steps

    # per-kernel figures, same launch configuration, each its own back-to-back loop
    us_attn = timed(args.steps, do_proj=False)
    us_proj = timed(args.steps, do_attn=False)
    us_single = us_attn_single = float("nan")
    if not args.no_single:
        us_single = timed(args.steps, rotate=False)
        us_attn_single = timed(args.steps, rotate=False, do_proj=False)

    attn_bytes = kv_bytes_layer + 2 * B * A * Hq * Dh * esz
    proj_bytes = w_bytes_layer + B * A * (w.hidden + w.qkv_width) * esz
    attn_gbs = attn_bytes / us_attn * 1e-3
    proj_flops = 2.0 * B * A * w.hidden * w.qkv_width
    attn_flops = 4.0 * B * A * Hq * S * Dh
    flops = proj_flops + attn_flops

    out = {
        "metric": "us per cached denoising layer-step + achieved KV-read HBM GB/s (fraction of peak)",
        "value": round(us_step, 3),
        "unit": "us",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(us_step / 1000.0, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": w.name + ("/refresh" if refresh else ""), "batch": B, "hidden": w.hidden, "n_q_heads": Hq, "n_kv_heads": Hkv,
            "head_dim": Dh, "kv_len": S, "active_rows": A, "layers_rotated": n_layers,
            "window_schedule": "start %d, +%d every %d steps" % (w.cached_len, w.block, w.steps_per_block)
            if w.gen_len else "fixed at %d" % w.cached_len,
        },
        "roofline": {
            "kernel": "fc_active_attention (k_attn_mfma + k_attn_combine)",
            "bound": "hbm",
            "achieved": round(attn_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(attn_gbs / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_ATTENTION_TRAFFIC_BYTES.get(w.name) if not refresh else None,
            "algorithmic_bytes_per_launch": attn_bytes,
            "us_per_launch": round(us_attn, 3),
        },
        "projection": {
            "kernel": "fc_qkv_project_scatter",
            "us_per_launch": round(us_proj, 3),
            "weight_stream_gbs": round(proj_bytes / us_proj * 1e-3, 1),
            "frac_of_hbm_peak": round(proj_bytes / us_proj * 1e-3 / HBM_PEAK_GBS, 4),
            "tflops": round(proj_flops / us_proj * 1e-6, 1),
            "frac_of_mfma_peak": round(proj_flops / us_proj * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
        },
        "active_rows_per_s": round(B * A / (us_step * 1e-6), 1),
        "tflops": round(flops / us_step * 1e-6, 2),
        "single_cache_us": None if args.no_single else round(us_single, 3),
        "single_cache_attention_us": None if args.no_single else round(us_attn_single, 3),
        "single_cache_attention_gbs": None if args.no_single else round(attn_bytes / us_attn_single * 1e-3, 1),
        "host_wall_us_per_step": round(t_host * 1e6 / args.steps, 2),
    }

    # A plain elementwise copy kernel of known size, so that a counter run of this same command
    # (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) can be scaled: 256 MiB read and 256 MiB written.
    cal_src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        torch.add(cal_src, 1.0, out=cal_dst)  # an elementwise kernel: reads 256 MiB, writes 256 MiB
    torch.cuda.synchronize()
    out["calibration_copy_bytes"] = cal_src.numel() * 4

    if refresh:
        # the refresh is a dense pass: both calls are bound by the matrix cores, the projection GEMM
        # being the longer one
        out["roofline"] = {
            "kernel": "fc_qkv_project_scatter (k_proj_gemm)",
            "bound": "mfma",
            "achieved": round(proj_flops / us_proj * 1e-6, 1),
            "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(proj_flops / us_proj * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": None,
            "algorithmic_flops_per_launch": proj_flops,
            "us_per_launch": round(us_proj, 3),
        }
        out["attention"] = {
            "kernel": "fc_active_attention",
            "us_per_launch": round(us_attn, 3),
            "tflops": round(attn_flops / us_attn * 1e-6, 1),
            "frac_of_mfma_peak": round(attn_flops / us_attn * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
        }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inputs, A, refresh)

    torch.cuda.synchronize()
    fc.fc_cache_free(cache)
    print(json.dumps(out))


def cpu_baseline(w, inputs, A, refresh):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import fc_oracle as orc

    max_samples, budget_s = 100, 12.0  # stop after about 12 s of oracle work
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
