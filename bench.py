#!/usr/bin/env python3
"""Benchmark of the MoC FFN hot path on one MI355X.

A step is one training forward + backward of one MoC FFN layer (all kernels of moc_ffn_fwd and
moc_ffn_bwd) over one batch of seeded synthetic tokens at the "1B shape" (T 8192, d 2048,
d_ff 5461, K 683, bf16 with fp32 accumulation), inputs resident in HBM.  The JSON line also
carries the decode leg at the "7B shape" (effective HBM GB/s, cold weights, with the dense FFN through
the same entry point beside it), a per-kernel breakdown (durations from HIP events that the library
records around every launch on the launch stream), the roofline object of the dominant kernel with
entries for the gate GEMM and the whole decode call, the two small configurations, the prefill
stack, the grouped and MoE-expert variants, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA: 256 CU x 4096 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-stack", action="store_true")
    ap.add_argument("--no-grouped", action="store_true", help="skip the MoC 2:8 (grouped Top-K) legs")
    ap.add_argument("--no-experts", action="store_true", help="skip the MoC-in-MoE-experts leg")
    ap.add_argument("--no-dense-decode", action="store_true", help="skip the dense FFN (K = d_ff) decode comparison")
    ap.add_argument("--no-small", action="store_true", help="skip the cfg0 (fp32 forward) and cfg1 (small fwd+bwd) legs")
    ap.add_argument("--no-clocks", action="store_true",
                    help="do not start rocm-smi after the run (a child process of a profiled run is refused on the GPU boxes)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--calibrate-traffic", action="store_true",
                    help="run only moc_residual_add on 2 x 512 MiB (known traffic: 1 GiB read, 512 MiB written per "
                         "launch) so that rocprofv3 FETCH_SIZE / WRITE_SIZE can be scaled")
    return ap.parse_args()


def source_hash():
    from paper_2511_09323_amd.build import source_hash as h
    return h()


def committed_traffic(kernel_key, lib_version):
    """HBM bytes per launch of `kernel_key` from the committed rocprofv3 counter summary, or None when that
    summary was not taken on the sources this library was built from."""
    tpath = os.path.join(ROOT, "profiles", "cfg2_traffic.json")
    if not os.path.exists(tpath):
        return None, "no committed counter summary"
    tj = json.load(open(tpath))
    here = source_hash()
    if tj.get("_source_hash") != here:
        return None, "committed counter summary is for other sources (%s, these are %s)" % (tj.get("_source_hash"), here)
    if ("src:" + here) not in lib_version:
        return None, "the library was not built from these sources (%s)" % lib_version
    ent = tj.get(kernel_key)
    if not ent:
        return None, "kernel not in the committed counter summary"
    return ent["hbm_read_bytes"] + ent["hbm_written_bytes"], "profiles/cfg2_traffic.json, same source hash %s" % here


def gemm_flops(T, d, F, K):
    """Executed and algorithmic FLOPs per launch of every GEMM-shaped kernel of one step."""
    ex = 2.0 * T * d * F
    al = 2.0 * T * d * K
    return {
        "gemm_gate": (ex, ex),                       # truly dense: algorithmic == executed
        "gemm_up": (ex, al),
        "gemm_down": (ex, al),
        "gemm_dz_pointwise": (ex, al),
        "gemm_dz": (ex, al),
        "gemm_dwd": (ex, al),
        "gemm_dwg": (ex, al),
        "gemm_dwu": (ex, al),
        "gemm_dw3": (3 * ex, 3 * al),                # dW_down, dW_gate, dW_up in one launch
        "gemm_gate_up": (2 * ex, ex + al),           # gate and up projection in one launch (when that saves a round)
        "gemm_dx": (2 * ex, 2 * al),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over tokens and needs no second GPU to be measured); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2511_09323_amd as moc
    from paper_2511_09323_amd import inputs
    from paper_2511_09323_amd.configs import CONFIGS, DECODE_BATCHES

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    moc.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_traffic:
        n_rows, n_cols = 65536, 4096                       # 512 MiB of bf16 per array
        h = torch.zeros((n_rows, n_cols), dtype=torch.bfloat16, device=dev)
        yv = torch.ones((n_rows, n_cols), dtype=torch.bfloat16, device=dev)
        for _ in range(4):
            moc.moc_residual_add(h, yv)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "moc_residual_add", "read_bytes": 2 * h.numel() * 2, "write_bytes": h.numel() * 2}))
        return
    cfg = CONFIGS[args.workload]
    cfg_index = int(args.workload[-1])
    T, d, F, K = cfg.T, cfg.d, cfg.F, cfg.K
    bf = torch.bfloat16

    def dev_bf16(a):
        return torch.from_numpy(a).to(dev).to(bf).contiguous()

    L = inputs.make_layer(cfg_index, T, d, F, "bf16", with_dy=True)
    G = {k: dev_bf16(v) for k, v in L.items()}
    ws_f = torch.empty(moc.workspace_bytes(T, d, F, K, bf, 0), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(moc.workspace_bytes(T, d, F, K, bf, 1), dtype=torch.uint8, device=dev)
    out_f = (torch.empty((T, d), dtype=bf, device=dev), torch.empty((T, K), dtype=torch.int32, device=dev),
             torch.empty((T, K), dtype=bf, device=dev), torch.empty((T, K), dtype=bf, device=dev))
    out_b = (torch.empty((T, d), dtype=bf, device=dev), torch.empty((F, d), dtype=bf, device=dev),
             torch.empty((F, d), dtype=bf, device=dev), torch.empty((F, d), dtype=bf, device=dev))

    def step():
        y, idx, gv, uv = moc.moc_ffn_fwd(G["x"], G["wg"], G["wu"], G["wd"], K, ws=ws_f, out=out_f)
        moc.moc_ffn_bwd(G["x"], G["wg"], G["wu"], G["wd"], idx, gv, uv, G["dy"], ws=ws_b, out=out_b)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = T / (ms_per_step * 1e-3)

    # per-kernel durations: the same steps again with HIP events around every launch, recorded
    # by the library on the stream the kernels run on
    moc.timing_reset()
    moc.timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    timing = moc.timing_read()
    moc.timing_enable(False)
    moc.timing_reset()
    flops = gemm_flops(T, d, F, K)
    ldF = (F + 63) // 64 * 64
    # algorithmic HBM bytes per launch of the two streaming kernels (bf16 activations):
    #   Top-K + SiLU.U: reads G fp32 and U, writes the dense Z' row and the stored set (idx, gvals, uvals);
    #   pointwise + expansion: reads the stored set and the dense dZ' row, writes Z', dG, dU rows.
    # executed: what these kernels move in this design (dense U in, dense-masked rows out);
    # algorithmic: what the method needs (gate row in + stored set out; stored set + dZ' at the selected
    # channels in, z', dG, dU at the selected channels out)
    hbm_bytes = {"topk_select_act": T * (4 * F + 2 * F + 2 * ldF + K * 8),
                 "bwd_pointwise_expand": T * (K * 8 + 2 * ldF + 3 * 2 * ldF)}
    hbm_algo = {"topk_select_act": T * (4 * F + K * (4 + 2)),
                "bwd_pointwise_expand": T * (K * (4 + 2 * 2) + K * 2 + 3 * K * 2)}
    kernels = []
    for name, (ms, n) in sorted(timing.items(), key=lambda kv: -kv[1][0]):
        avg_ms = ms / max(n, 1)
        row = {"kernel": name, "avg_ms": round(avg_ms, 5), "launches": n}
        if name in flops:
            ex, al = flops[name]
            row["executed_tflops"] = round(ex / (avg_ms * 1e-3) / 1e12, 2)
            row["algorithmic_tflops"] = round(al / (avg_ms * 1e-3) / 1e12, 2)
            row["frac_executed"] = round(row["executed_tflops"] / PEAK_BF16_TFLOPS, 4)
        if name in hbm_bytes:
            row["executed_GBs"] = round(hbm_bytes[name] / (avg_ms * 1e-3) / 1e9, 1)
            row["frac_hbm_peak_executed"] = round(row["executed_GBs"] / PEAK_HBM_GBS, 4)
            row["algorithmic_GBs"] = round(hbm_algo[name] / (avg_ms * 1e-3) / 1e9, 1)
            row["frac_hbm_peak_algorithmic"] = round(row["algorithmic_GBs"] / PEAK_HBM_GBS, 4)
        kernels.append(row)
    # roofline: the top-level keys describe the dominant kernel of the step (largest share of the time);
    # `entries` adds the gate GEMM (the one contraction whose algorithmic FLOPs, 2 d F per token, equal
    # the executed ones) and, further down, the whole decode call.  `achieved` / `frac` are ALGORITHMIC
    # FLOP/s (2 d K per token and product for the gathered contractions); the executed (dense-tile)
    # rate stands beside them.  HBM traffic per launch comes from the committed rocprofv3 counter
    # summary, and only when that summary was taken on the sources this library was built from.
    traffic_keys = {"gemm_gate": "gemm_bf16_mfma<256,256,KC,KC,tail0,EpiStore<float>>",
                    "gemm_dw3": "gemm_bf16_mfma_batch3<256,192,KM,KM,tail0,EpiStore<bf16>>"}

    def roofline_entry(row):
        name = row["kernel"]
        ex, al = flops[name]
        traffic, note = (None, "not measured for this kernel")
        if args.workload == "cfg2" and name in traffic_keys:
            traffic, note = committed_traffic(traffic_keys[name], moc.version())
        return {"kernel": name, "bound": "mfma", "achieved": row["algorithmic_tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(row["algorithmic_tflops"] / PEAK_BF16_TFLOPS, 4),
                "achieved_executed": row["executed_tflops"], "frac_executed": row["frac_executed"],
                "traffic": traffic, "traffic_source": note, "avg_ms": row["avg_ms"],
                "flops_per_launch": al, "executed_flops_per_launch": ex,
                "timing": "HIP events around every launch, recorded by the library on the launch stream"}

    gemm_rows = [r for r in kernels if r["kernel"] in flops]
    roofline = None
    if gemm_rows:
        dominant = max(gemm_rows, key=lambda r: r["avg_ms"])
        roofline = roofline_entry(dominant)
        roofline["entries"] = [roofline_entry(r) for r in gemm_rows if r["kernel"] in ("gemm_gate", "gemm_gate_up") and r is not dominant]
    gemm_ms = sum(r["avg_ms"] for r in kernels if r["kernel"] in flops)
    gemm_ex = sum(flops[r["kernel"]][0] for r in kernels if r["kernel"] in flops)
    gemm_al = sum(flops[r["kernel"]][1] for r in kernels if r["kernel"] in flops)
    all_gemms = {"sum_avg_ms": round(gemm_ms, 4),
                 "executed_tflops": round(gemm_ex / (gemm_ms * 1e-3) / 1e12, 2) if gemm_ms else None,
                 "algorithmic_tflops": round(gemm_al / (gemm_ms * 1e-3) / 1e12, 2) if gemm_ms else None}

    # dense SwiGLU through the same library, for the paper's dense-vs-MoC comparison
    dense = None
    if not args.no_dense:
        ws_df = torch.empty(moc.workspace_bytes(T, d, F, F, bf, 3), dtype=torch.uint8, device=dev)
        ws_db = torch.empty(moc.workspace_bytes(T, d, F, F, bf, 4), dtype=torch.uint8, device=dev)
        out_df = (out_f[0], torch.empty((T, F), dtype=bf, device=dev), torch.empty((T, F), dtype=bf, device=dev))

        def dense_step():
            y, gs, us = moc.moc_swiglu_fwd(G["x"], G["wg"], G["wu"], G["wd"], ws=ws_df, out=out_df)
            moc.moc_swiglu_bwd(G["x"], G["wg"], G["wu"], G["wd"], gs, us, G["dy"], ws=ws_db, out=out_b)

        for _ in range(max(2, args.warmup // 2)):
            dense_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_dense = max(3, args.steps // 2)
        for _ in range(n_dense):
            dense_step()
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t0) * 1e3 / n_dense
        dense = {"ms_per_step": round(dense_ms, 4), "tokens_per_s": round(T / (dense_ms * 1e-3), 1),
                 "saved_activation_bytes": 2 * T * F * 2, "moc_saved_activation_bytes": T * K * (4 + 2 * 2)}
        del ws_df, ws_db, out_df

    # decode leg: 7B shape, cold weights (rotating through independent weight sets); the dense FFN through
    # the same entry point (K = d_ff: every channel selected) is the in-library comparison
    decode = None
    if not args.no_decode:
        decode = decode_leg(torch, moc, inputs, CONFIGS["cfg3"], DECODE_BATCHES, dev)
        if not args.no_dense_decode:
            decode["dense_K_equals_F"] = decode_leg(torch, moc, inputs, CONFIGS["cfg3"], DECODE_BATCHES, dev, dense=True)["batches"]
        if roofline is not None:
            roofline["entries"] += [
                {"kernel": "moc_ffn_decode, whole call, B=%d" % b["B"], "bound": "hbm", "achieved": b["effective_GBs"],
                 "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": b["frac_hbm_peak"], "traffic": None,
                 "bytes_per_call": int(b["algorithmic_MB"] * 1e6), "us_per_call": b["cold_us_median"],
                 "timing": "HIP events around the whole call, cold weights"} for b in decode["batches"]]

    # the two small configurations: cfg0 (fp32 forward) and cfg1 (bf16 forward + backward)
    small = None
    if not args.no_small:
        small = {"cfg0": small_leg(torch, moc, inputs, CONFIGS["cfg0"], 0, dev, backward=False),
                 "cfg1": small_leg(torch, moc, inputs, CONFIGS["cfg1"], 1, dev, backward=True)}

    # prefill-stack leg: 32 x [RMSNorm -> MoC FFN forward -> residual add] at the 7B shape
    stack = None
    if not args.no_stack:
        stack = stack_leg(torch, moc, CONFIGS["cfg4"], dev)

    # MoC_{2:8} (grouped Top-K): training step at the 1B shape with d_ff rounded up to a multiple of 8,
    # and cold decode at the 7B shape
    grouped = None
    if not args.no_grouped:
        grouped = {"train": grouped_train_leg(torch, moc, inputs, cfg, 2, 8, args.steps, args.warmup, dev),
                   "decode": decode_leg(torch, moc, inputs, CONFIGS["cfg3"], DECODE_BATCHES, dev, group=(2, 8)),
                   "decode_1of8": decode_leg(torch, moc, inputs, CONFIGS["cfg3"], DECODE_BATCHES, dev, group=(1, 8))}

    # MoC inside MoE experts (the paper's Mixtral shapes: 8 experts, 2 per token)
    experts = None
    if not args.no_experts:
        experts = [experts_leg(torch, moc, 512, 1376, 256, dev), experts_leg(torch, moc, 768, 2048, 384, dev)]

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(L, K, args.cpu_sample_tokens)

    line_clocks = None if args.no_clocks else gpu_clocks()
    line = {
        "metric": "MoC FFN fwd+bwd tokens/s (1B shape) + decode effective HBM GB/s vs peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: one MoC FFN layer fwd+bwd, T=%d d_model=%d d_ff=%d K=%d" % (args.workload, T, d, F, K),
                   "T": T, "d_model": d, "d_ff": F, "K": K},
        "roofline": roofline, "cpu_baseline": cpu, "all_gemms": all_gemms, "kernels": kernels, "dense_swiglu": dense,
        "decode": decode, "small_configs": small, "prefill_stack": stack, "grouped_2of8": grouped, "moe_experts": experts,
        "clocks_after_run": line_clocks, "library": moc.version(), "source_hash": source_hash(),
    }
    print(json.dumps(line))


def gpu_clocks():
    """Shader and memory clock as rocm-smi reports them right after the timed work (best effort)."""
    import re
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
        got = {}
        for key in ("sclk", "mclk", "fclk"):
            m = re.search(key + r" clock level: \d+: \((\d+)Mhz\)", out)
            if m:
                got[key + "_MHz"] = int(m.group(1))
        return got or None
    except Exception:
        return None


def stack_leg(torch, moc, cfg, dev, layers=32):
    """The cfg4 prefill stack: `layers` x [h <- h + MoC(RMSNorm(h))] with independent weights per layer
    (32 x 270 MB), timed as a whole and per kernel."""
    from paper_2511_09323_amd.configs import RMSNORM_EPS
    T, d, F, K = cfg.T, cfg.d, cfg.F, cfg.K
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(40_000)
    h0 = torch.randn((T, d), generator=gen, device=dev, dtype=torch.float32).to(bf)
    w = [[(torch.randn((F, d), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(bf) for _ in range(3)]
         for _ in range(layers)]
    gain = torch.ones((d,), dtype=bf, device=dev)
    h = torch.empty_like(h0)
    xn = torch.empty_like(h0)
    ws = torch.empty(moc.workspace_bytes(T, d, F, K, bf, 0), dtype=torch.uint8, device=dev)
    out = (torch.empty((T, d), dtype=bf, device=dev), torch.empty((T, K), dtype=torch.int32, device=dev),
           torch.empty((T, K), dtype=bf, device=dev), torch.empty((T, K), dtype=bf, device=dev))

    def stack():
        h.copy_(h0)
        for l in range(layers):
            moc.moc_rmsnorm(h, gain, RMSNORM_EPS, out=xn)
            y, _, _, _ = moc.moc_ffn_fwd(xn, w[l][0], w[l][1], w[l][2], K, ws=ws, out=out)
            moc.moc_residual_add(h, y)

    stack()
    torch.cuda.synchronize()
    n = 3
    t0 = time.perf_counter()
    for _ in range(n):
        stack()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    moc.timing_reset()
    moc.timing_enable(True)
    stack()
    torch.cuda.synchronize()
    kern = {k: round(v / max(c, 1), 4) for k, (v, c) in moc.timing_read().items()}
    moc.timing_enable(False)
    moc.timing_reset()
    ex = 2.0 * T * d * F
    row_bytes = T * d * 2
    return {"workload": "cfg4 stack: %d layers, T=%d d_model=%d d_ff=%d K=%d bf16, independent weights per layer" % (layers, T, d, F, K),
            "ms_per_stack": round(ms, 3), "ms_per_layer": round(ms / layers, 4), "tokens_per_s": round(T / (ms * 1e-3), 1),
            "kernels_ms": kern,
            "gemm_executed_tflops": {k: round(m * ex / (kern[k] * 1e-3) / 1e12, 1)
                                     for k, m in (("gemm_gate", 1), ("gemm_up", 1), ("gemm_gate_up", 2), ("gemm_down", 1)) if k in kern},
            "rmsnorm_GBs": round(2 * row_bytes / (kern["rmsnorm"] * 1e-3) / 1e9, 1) if "rmsnorm" in kern else None,
            "residual_add_GBs": round(3 * row_bytes / (kern["residual_add"] * 1e-3) / 1e9, 1) if "residual_add" in kern else None}


def experts_leg(torch, moc, d, F, K, dev, tokens=16384, n_exp=8, per_token=2):
    """Forward + backward of MoC as the MLP of MoE experts on `tokens` tokens routed to `per_token` of
    `n_exp` experts each (seeded, uneven split): one grouped launch per projection, against the same
    work done with one moc_ffn_fwd / moc_ffn_bwd call per expert."""
    bf = torch.bfloat16
    A = tokens * per_token
    rng = np.random.default_rng(60_000 + d)
    counts = rng.multinomial(A, rng.dirichlet(np.full(n_exp, 8.0)))
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    gen = torch.Generator(device=dev)
    gen.manual_seed(60_000 + d)
    x = torch.randn((A, d), generator=gen, device=dev, dtype=torch.float32).to(bf)
    dy = torch.randn((A, d), generator=gen, device=dev, dtype=torch.float32).to(bf)
    w = [(torch.randn((n_exp, F, d), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(bf) for _ in range(3)]
    ws_f = torch.empty(moc.workspace_bytes(A, d, F, K, bf, 0), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(moc.workspace_bytes(A, d, F, K, bf, 1), dtype=torch.uint8, device=dev)
    out_f = (torch.empty((A, d), dtype=bf, device=dev), torch.empty((A, K), dtype=torch.int32, device=dev),
             torch.empty((A, K), dtype=bf, device=dev), torch.empty((A, K), dtype=bf, device=dev))
    out_b = (torch.empty((A, d), dtype=bf, device=dev),) + tuple(torch.empty((n_exp, F, d), dtype=bf, device=dev) for _ in range(3))

    def grouped():
        y, idx, gv, uv = moc.moc_ffn_fwd_experts(x, offsets, w[0], w[1], w[2], K, ws=ws_f, out=out_f)
        moc.moc_ffn_bwd_experts(x, offsets, w[0], w[1], w[2], idx, gv, uv, dy, ws=ws_b, out=out_b)

    def looped():
        for e in range(n_exp):
            lo, hi = int(offsets[e]), int(offsets[e + 1])
            if hi == lo:
                continue
            o_f = tuple(t[lo:hi] for t in out_f)
            o_b = (out_b[0][lo:hi], out_b[1][e], out_b[2][e], out_b[3][e])
            y, idx, gv, uv = moc.moc_ffn_fwd(x[lo:hi], w[0][e], w[1][e], w[2][e], K, ws=ws_f, out=o_f)
            moc.moc_ffn_bwd(x[lo:hi], w[0][e], w[1][e], w[2][e], idx, gv, uv, dy[lo:hi], ws=ws_b, out=o_b)

    res = {}
    for name, fn in (("grouped", grouped), ("looped", looped)):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        n = 30
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) * 1e3 / n
    moc.timing_reset()
    moc.timing_enable(True)
    for _ in range(10):
        grouped()
    torch.cuda.synchronize()
    kern = {k: round(v / max(c, 1), 4) for k, (v, c) in moc.timing_read().items()}
    moc.timing_enable(False)
    moc.timing_reset()
    executed = 18.0 * A * d * F            # dense-equivalent FLOPs of forward + backward over all routed rows
    return {"workload": "MoC in MoE experts: %d tokens x %d of %d experts, d_model=%d d_ff=%d K=%d bf16, rows per expert %s" % (
                tokens, per_token, n_exp, d, F, K, [int(c) for c in counts]),
            "ms_per_step_grouped": round(res["grouped"], 4), "ms_per_step_one_call_per_expert": round(res["looped"], 4),
            "tokens_per_s": round(tokens / (res["grouped"] * 1e-3), 1),
            "executed_tflops": round(executed / (res["grouped"] * 1e-3) / 1e12, 1), "kernels_ms": kern}


def grouped_train_leg(torch, moc, inputs, cfg, a, b, steps, warmup, dev):
    """Forward (grouped selection) + backward of one MoC_{a:b} layer; d_ff rounded up to a multiple of b."""
    T, d = cfg.T, cfg.d
    F = (cfg.F + b - 1) // b * b
    K = F // b * a
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(50_000)
    x = torch.randn((T, d), generator=gen, device=dev, dtype=torch.float32).to(bf)
    dy = torch.randn((T, d), generator=gen, device=dev, dtype=torch.float32).to(bf)
    w = [(torch.randn((F, d), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(bf) for _ in range(3)]
    ws_f = torch.empty(moc.workspace_bytes(T, d, F, K, bf, 0), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(moc.workspace_bytes(T, d, F, K, bf, 1), dtype=torch.uint8, device=dev)
    out_f = (torch.empty((T, d), dtype=bf, device=dev), torch.empty((T, K), dtype=torch.int32, device=dev),
             torch.empty((T, K), dtype=bf, device=dev), torch.empty((T, K), dtype=bf, device=dev))
    out_b = (torch.empty((T, d), dtype=bf, device=dev), torch.empty((F, d), dtype=bf, device=dev),
             torch.empty((F, d), dtype=bf, device=dev), torch.empty((F, d), dtype=bf, device=dev))

    def step():
        y, idx, gv, uv = moc.moc_ffn_fwd_grouped(x, w[0], w[1], w[2], a, b, ws=ws_f, out=out_f)
        moc.moc_ffn_bwd(x, w[0], w[1], w[2], idx, gv, uv, dy, ws=ws_b, out=out_b)

    for _ in range(max(2, warmup // 2)):
        step()
    torch.cuda.synchronize()
    n = max(3, steps // 2)
    t0 = time.perf_counter()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    moc.timing_reset()
    moc.timing_enable(True)
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    kern = {k: round(v / max(c, 1), 4) for k, (v, c) in moc.timing_read().items()}
    moc.timing_enable(False)
    moc.timing_reset()
    sel_bytes = T * (4 * F + 2 * F + 2 * ((F + 63) // 64 * 64) + K * (4 + 2 + 2))     # G, U in; Z' and the stored set out
    sel = kern.get("group_select_act")
    return {"workload": "1B shape, MoC %d:%d: T=%d d_model=%d d_ff=%d K=%d bf16" % (a, b, T, d, F, K),
            "ms_per_step": round(ms, 4), "tokens_per_s": round(T / (ms * 1e-3), 1), "kernels_ms": kern,
            "group_select_GBs": round(sel_bytes / (sel * 1e-3) / 1e9, 1) if sel else None,
            "group_select_frac_hbm_peak": round(sel_bytes / (sel * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if sel else None}


def small_leg(torch, moc, inputs, cfg, cfg_index, dev, backward):
    """cfg0 / cfg1: far too small for any roofline (a few GFLOP); time and tokens/s only."""
    T, d, F, K = cfg.T, cfg.d, cfg.F, cfg.K
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    L = inputs.make_layer(cfg_index, T, d, F, cfg.dtype, with_dy=backward)
    G = {k: torch.from_numpy(v).to(dev).to(dt).contiguous() for k, v in L.items()}
    ws_f = torch.empty(moc.workspace_bytes(T, d, F, K, dt, 0), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(moc.workspace_bytes(T, d, F, K, dt, 1), dtype=torch.uint8, device=dev) if backward else None
    out_f = (torch.empty((T, d), dtype=dt, device=dev), torch.empty((T, K), dtype=torch.int32, device=dev),
             torch.empty((T, K), dtype=dt, device=dev), torch.empty((T, K), dtype=dt, device=dev))
    out_b = (torch.empty((T, d), dtype=dt, device=dev),) + tuple(torch.empty((F, d), dtype=dt, device=dev) for _ in range(3))

    def step():
        y, idx, gv, uv = moc.moc_ffn_fwd(G["x"], G["wg"], G["wu"], G["wd"], K, ws=ws_f, out=out_f)
        if backward:
            moc.moc_ffn_bwd(G["x"], G["wg"], G["wu"], G["wd"], idx, gv, uv, G["dy"], ws=ws_b, out=out_b)

    for _ in range(20):
        step()
    torch.cuda.synchronize()
    n = 200
    t0 = time.perf_counter()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    executed = (18.0 if backward else 6.0) * T * d * F
    return {"workload": "%s: %s, T=%d d_model=%d d_ff=%d K=%d %s" % (cfg.name, "forward + backward" if backward else "forward",
                                                                    T, d, F, K, cfg.dtype),
            "ms_per_step": round(ms, 4), "tokens_per_s": round(T / (ms * 1e-3), 1),
            "executed_tflops": round(executed / (ms * 1e-3) / 1e12, 2)}


def decode_leg(torch, moc, inputs, cfg, batches, dev, group=None, dense=False):
    d, F, K = cfg.d, cfg.F, cfg.K
    if dense:
        K = F
    if group is not None:
        K = F // group[1] * group[0]
    bf = torch.bfloat16

    def decode(x, w, ws, out):
        if group is None:
            moc.moc_ffn_decode(x, *w, K, ws=ws, out=out)
        else:
            moc.moc_ffn_decode_grouped(x, *w, group[0], group[1], ws=ws, out=out)

    R = 8        # independent weight sets: 8 x 270 MB >> the 256 MB last-level cache, so every call is cold
    gen = torch.Generator(device=dev)
    gen.manual_seed(30_000)
    sets = []
    for r in range(R):
        sets.append(tuple((torch.randn((F, d), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(bf)
                          for _ in range(3)))
    out = []
    for B in batches:
        xs = [torch.randn((B, d), generator=gen, device=dev, dtype=torch.float32).to(bf) for _ in range(R)]
        ws = torch.empty(moc.workspace_bytes(B, d, F, K, bf, 2), dtype=torch.uint8, device=dev)
        y = torch.empty((B, d), dtype=bf, device=dev)
        idx = torch.empty((B, K), dtype=torch.int32, device=dev)
        unions = []
        for r in range(R):
            decode(xs[r], sets[r], ws, (y, idx))
            torch.cuda.synchronize()
            unions.append(int(torch.unique(idx).numel()))
        union = float(np.mean(unions))
        algo_bytes = d * F * 2 + 2 * union * d * 2 + 2 * B * d * 2
        iters = 7 * R                   # 56 cold calls
        start = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
        stop = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
        for i in range(iters):
            r = i % R
            start[i].record()
            decode(xs[r], sets[r], ws, (y, idx))
            stop[i].record()
        torch.cuda.synchronize()
        us = sorted(s.elapsed_time(e) * 1e3 for s, e in zip(start, stop))
        med = us[len(us) // 2]
        # per-kernel durations of the cold calls (library-side HIP events, separate pass)
        moc.timing_reset()
        moc.timing_enable(True)
        for i in range(2 * R):
            r = i % R
            decode(xs[r], sets[r], ws, (y, idx))
        torch.cuda.synchronize()
        kern_us = {k: round(ms * 1e3 / max(n, 1), 2) for k, (ms, n) in moc.timing_read().items()}
        moc.timing_enable(False)
        moc.timing_reset()
        # warm: the same weight set every call (cache-resident, reported separately)
        for _ in range(3):
            decode(xs[0], sets[0], ws, (y, idx))
        torch.cuda.synchronize()
        s0, e0 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for _ in range(20):
            decode(xs[0], sets[0], ws, (y, idx))
        e0.record()
        torch.cuda.synchronize()
        warm_us = s0.elapsed_time(e0) * 1e3 / 20
        gbs = algo_bytes / (med * 1e-6) / 1e9
        out.append({"B": B, "cold_us_median": round(med, 2), "cold_us_min": round(us[0], 2), "warm_us": round(warm_us, 2),
                    "union_channels": round(union, 1), "algorithmic_MB": round(algo_bytes / 1e6, 2),
                    "effective_GBs": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
                    "kernels_us_event_bracketed": kern_us})
    sel = "row-wide Top-K" if group is None else "grouped Top-K %d:%d" % group
    if dense:
        sel = "dense FFN through moc_ffn_decode (K = d_ff)"
    return {"workload": "cfg3: d_model=%d d_ff=%d K=%d bf16, %s, cold weights (8 rotating sets)" % (d, F, K, sel),
            "timing": "cold_us_*: HIP events around the whole call; kernels_us_event_bracketed: a separate pass with events around "
                      "every launch, which adds 2-3 us per launch, so their sum exceeds the call time (rocprofv3 durations are "
                      "in profiles/cfg3_decode_kernel_stats.md)",
            "batches": out}


def cpu_baseline(L, K, sample_tokens):
    """The CPU oracle as it stands (numpy float64), timed on the first `sample_tokens` tokens of the
    same workload: forward (own selection) + backward, full-size weights."""
    from oracle import moc_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    n = min(sample_tokens, L["x"].shape[0])
    X = L["x"][:n].astype(np.float64)
    dY = L["dy"][:n].astype(np.float64)
    Wg, Wu, Wd = L["wg"].astype(np.float64).T, L["wu"].astype(np.float64).T, L["wd"].astype(np.float64)
    t0 = time.perf_counter()
    D, M, Gm, U = O.moc_forward(X, Wg, Wu, Wd, K)
    O.moc_backward(X, Wg, Wu, Wd, M, Gm * M, U * M, dY)
    dt = time.perf_counter() - t0
    return {"value": round(n / dt, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d tokens of the same layer, forward + backward, numpy float64, %.1f s" % (n, dt)}


if __name__ == "__main__":
    main()
