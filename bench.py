#!/usr/bin/env python3
"""Benchmark of the TurboBoA hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic attention block: Hessian build (Table 1, with the
deviation correlations R), quantization of W_Q, W_K, W_V (Algorithm 1 with Algorithms 2 and 3), the output-projection
Hessian, quantization of W_O.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_bf16_hv_syrk_llama2-7b_hbm_traffic.txt")


def measured_traffic(cfg_name):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of
    `bench.py --roofline-probe` (counters cannot be read from inside the timed run); None for other workloads."""
    if cfg_name != "llama2-7b" or not os.path.exists(TRAFFIC_FILE):
        return None
    for line in open(TRAFFIC_FILE):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def cpu_baseline(blk, cfg, hessians, budget_note):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload, scaled to one attention block:
    (1) Algorithm 1 for ONE head of W_Q (128 out-channels, all d in-channels) with the Hessians given, times the number of
        head-sized row groups in the four layers (Hq + 2 Hkv + d/dh);
    (2) the Table 1 sums of ONE (sequence, query head) pair (A_h, Y = A_h X_s, Y^T Y, and the same for the deviation term),
        times n_seqs * Hq, plus X_s^T X_s and dX_s^T X_s of one sequence times n_seqs.  The output-projection Hessian
        (another attention forward per sequence and head) is not sampled and not counted."""
    import numpy as np
    from oracle import turboboa_ref as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    dh = cfg.head_dim
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    W = f(blk["Wq"][:dh]); Hin = f(hessians["Hin_qk"]); Hout = f(hessians["Hout_q"][:1])
    R = f(hessians["R_qk"]) if hessians["R_qk"] is not None else None
    t = time.perf_counter()
    O.quantize_layer(W, Hin, Hout, R, 1, bits=cfg.bits, block=cfg.block, group=cfg.group)
    dt_q = time.perf_counter() - t
    heads_equiv = cfg.n_q_heads + 2 * cfg.n_kv_heads + cfg.d_model // dh
    xs = f(blk["X"][0]) if blk["X"] is not None else f(blk["X_fp"][0])
    xf = f(blk["X_fp"][0]); wq = f(blk["Wq"][:dh]); wk = f(blk["Wk"][:dh])
    t = time.perf_counter()
    A, _, _ = O.attention_probs(xs, wq, wk)
    Y = A @ xs; Hv = Y.T @ Y
    if R is not None:
        Af, _, _ = O.attention_probs(xf, wq, wk)
        Rv = (Y - Af @ xf).T @ Y
    dt_pair = time.perf_counter() - t
    t = time.perf_counter()
    Hs = xs.T @ xs
    if R is not None:
        Rs = (xs - xf).T @ xs
    dt_seq = time.perf_counter() - t
    hess = dt_pair * cfg.n_seqs * cfg.n_q_heads + dt_seq * cfg.n_seqs
    return {"value": dt_q * heads_equiv + hess, "unit": "s per attention block (extrapolated)", "cores": int(cores), "kind": "oracle",
            "sample": "oracle quantize_layer on head 0 of W_Q (%d x %d, Hessians given): %.1f s measured, x %d head-sized row groups in "
                      "W_Q, W_K, W_V, W_O = %.0f s; oracle Table 1 sums of one (sequence, head) pair: %.1f s, x %d pairs, and of one "
                      "sequence for H_in, R: %.2f s, x %d = %.0f s; output-projection Hessian not counted%s"
                      % (dh, cfg.d_model, dt_q, heads_equiv, dt_q * heads_equiv, dt_pair, cfg.n_seqs * cfg.n_q_heads, dt_seq, cfg.n_seqs, hess,
                         budget_note)}


def roofline_probe(ctx, cfg, torch, zero=False, reps=0):
    """The command the HBM-traffic counter runs are made with: one plain copy of 1 GiB (a kernel of known traffic, to scale
    the counters), then ONE launch of the dominant kernel in the launch shape the benchmark times: H_in^V += Y^T (Y^T)^T for
    all KV heads over a chunk of 8 sequences (lower tiles, accumulating into fp32), operands at the benchmark's row pitch and,
    as in the benchmark, read as 16 x 32 blocks (the values are random either way).
    zero: all-zero operands instead of random ones (same launch, same addresses: what the operand values alone do to the
    rate).  reps > 0: that many further launches, timed with events on the context's stream, their mean printed."""
    import paper_2602_04929_amd as tb
    rep, G = cfg.n_q_heads // cfg.n_kv_heads, 8
    ky = rep * G * cfg.seq_len
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    src = torch.randn(1 << 28, generator=g, device="cuda")                    # 1 GiB
    dst = torch.empty_like(src)
    YT = torch.empty(cfg.n_kv_heads, cfg.d_model, ky + 256, dtype=torch.bfloat16, device="cuda")
    for h in range(cfg.n_kv_heads):
        YT[h] = torch.randn(cfg.d_model, ky + 256, generator=g, device="cuda").to(torch.bfloat16)
    if zero:
        YT.zero_()
    Hv = torch.zeros(cfg.n_kv_heads, cfg.d_model, cfg.d_model, device="cuda")
    torch.cuda.synchronize()
    torch.mul(src, 1.0, out=dst)                                              # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    Y = YT[:, :, :ky]
    ctx.gemm_bf16_nt(Y, Y, C_out=Hv, accumulate=True, flags=tb.GEMM_LOWER | tb.GEMM_A_TILED | tb.GEMM_B_TILED)
    torch.cuda.synchronize()
    n = cfg.d_model
    alg = cfg.n_kv_heads * (n * ky * 2 + 2 * 4 * n * (n + 1) // 2)            # Y^T read once, lower half of H read + written
    rec = {"probe": "copy 1 GiB, then gemm_bf16_nt LOWER accumulate, blocked operands", "copy_bytes_read": src.numel() * 4,
           "copy_bytes_written": src.numel() * 4, "gemm_batch": cfg.n_kv_heads, "gemm_M": n, "gemm_K": ky,
           "gemm_algorithmic_bytes": alg, "operands": "zero" if zero else "random"}
    if reps > 0:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]    # the context runs on torch's current stream
        ev[0].record()
        for i in range(reps):
            ctx.gemm_bf16_nt(Y, Y, C_out=Hv, accumulate=True, flags=tb.GEMM_LOWER | tb.GEMM_A_TILED | tb.GEMM_B_TILED)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
        flops = 2.0 * cfg.n_kv_heads * (n * (n + 1) // 2) * ky                  # the lower triangle, as the library counts this launch
        rec.update({"reps": reps, "median_launch_ms": ms[reps // 2], "min_launch_ms": ms[0],
                    "median_tflops": flops / (ms[reps // 2] * 1e-3) / 1e12})
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="llama2-7b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-R", action="store_true", help="first-block setting: no upstream deviation (R = 0)")
    ap.add_argument("--n-seqs", type=int, default=0, help="override the number of calibration sequences (profiling runs)")
    ap.add_argument("--correlated", action="store_true", help="correlated channels: X <- X (I + 0.3 low-rank); reported separately")
    ap.add_argument("--seq-chunk", type=int, default=0, help="sequences per pass of the W_V Hessian build (0 = library default)")
    ap.add_argument("--serial-layers", action="store_true", help="quantize W_Q, W_K, W_V one after the other on one stream")
    ap.add_argument("--with-mlp", action="store_true",
                    help="also time the gated MLP of the same transformer block (reported beside the metric, never inside `value`)")
    ap.add_argument("--roofline-probe", action="store_true",
                    help="run one plain 1 GiB copy and one launch of the dominant kernel in the benchmark's launch shape, nothing else "
                         "(the command for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--probe-zero", action="store_true", help="with --roofline-probe: all-zero operands (same launch otherwise)")
    ap.add_argument("--probe-reps", type=int, default=0, help="with --roofline-probe: time this many further launches of the kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (heads would shard across GPUs, see DESIGN.md); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_04929_amd as tb
    from paper_2602_04929_amd import synth
    from paper_2602_04929_amd.pipeline import quantize_attention_block

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(2)
    cfg = synth.CONFIGS[args.config]
    if args.n_seqs:
        cfg = synth.scaled(cfg, n_seqs=args.n_seqs)
    torch.cuda.set_device(0)
    if args.roofline_probe:
        ctx = tb.Context()
        roofline_probe(ctx, cfg, torch, zero=args.probe_zero, reps=args.probe_reps)
        ctx.close()
        return
    blk = synth.make_block(cfg, seed=0, device="cuda:0")
    if args.correlated:
        synth.apply_mix(blk, synth.correlated_mix(cfg.d_model, seed=0, device="cuda:0"))
    ctx = tb.Context()
    use_R = not args.no_R

    from paper_2602_04929_amd.pipeline import make_side_contexts
    side = None if args.serial_layers else make_side_contexts(2)

    def step(timings=None):
        return quantize_attention_block(ctx, blk, cfg, alpha=0.25, use_R=use_R, timings=timings, side_contexts=side, seq_chunk=args.seq_chunk)

    for _ in range(args.warmup):
        out = step()
    torch.cuda.synchronize()
    ctx.profile(True)
    stages = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(stages)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sec_per_block = dt / args.steps

    prof = {k: ctx.profile_read(k) for k in ctx.PROF_TAGS}
    ctx.profile(False)
    dom = prof["hv_syrk"]
    achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12 if dom["ms"] > 0 else 0.0
    roofline = {"bound": "mfma", "kernel": "gemm_bf16_nt_fast_kernel (H_in^V += Y^T Y, lower tiles)", "achieved": achieved,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": dom["ms"] / max(1, dom["launches"]), "launches": dom["launches"], "traffic": measured_traffic(cfg.name if not args.n_seqs else ""),
                "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy)"}
    kernels = {k: {"ms_per_step": v["ms"] / args.steps, "launches_per_step": v["launches"] // args.steps,
                   "tflops": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["ms"] > 0 else 0.0} for k, v in prof.items()}
    mfma_ms = sum(v["ms"] for v in prof.values()) / args.steps

    rec = {
        "metric": "sec per attention block (Wq,Wk,Wv,Wo) quantized INT%d; MFMA util %%" % cfg.bits,
        "value": sec_per_block, "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_block * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (Hessian contractions, fp32 accumulate) + f64 (quantization)", "data": "synthetic",
        "config": {"workload": "%s attention block: d_model=%d, %d q-heads / %d kv-heads x %d, %d seqs x %d tokens, INT%d, N=%d, "
                               "group=%d, alpha=0.25, R %s, adaptive grid, 1 CD sweep"
                               % (cfg.name, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_seqs, cfg.seq_len, cfg.bits,
                                  cfg.block, cfg.group, "on" if use_R else "off") + (", correlated channels" if args.correlated else "")},
        "mfma_util_pct": 100.0 * achieved / PEAK_BF16_TFLOPS,
        "stage_seconds": {k: v / args.steps for k, v in stages.items()},
        "bf16_gemm_seconds_per_step": mfma_ms * 1e-3,
        "kernels": kernels,
        "losses": {k: out[k]["loss"] for k in ("q", "k", "v", "o")},
        "workspace_gib": (ctx.workspace_bytes() + sum(c.workspace_bytes() for c in side or [])) / 2 ** 30,
        "grid_search": {"two_phase_passes": ctx.counter(0), "passes_fully_exact": ctx.counter(1), "rows_fully_exact": ctx.counter(2)},
        "roofline": roofline,
    }
    if args.with_mlp:
        from paper_2602_04929_amd.pipeline import quantize_mlp
        mlp = synth.make_mlp(cfg, seed=0, device="cuda:0")
        quantize_mlp(ctx, mlp, cfg, use_R=use_R)
        tm = {}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        quantize_mlp(ctx, mlp, cfg, use_R=use_R, timings=tm)
        torch.cuda.synchronize()
        rec["mlp"] = {"seconds": time.perf_counter() - t0, "d_ff": cfg.d_ff, "stage_seconds": tm,
                      "note": "gate, up, down projections of the same block (H_out = I), outside `value`"}
        del mlp
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(blk, cfg, out["hessians"], "")
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
