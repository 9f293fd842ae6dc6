#!/usr/bin/env python3
"""Benchmark of the TurboBoA hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic attention block: Hessian build (Table 1, with the
deviation correlations R), quantization of W_Q, W_K, W_V (Algorithm 1 with Algorithms 2 and 3), the output-projection
Hessian, quantization of W_O.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
The default workload is the Llama-2-70B-shaped grouped-query block (the largest named configuration; it fits one GPU).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 MFMA, published
PEAK_F64_TFLOPS = 78.6         # MI355X fp64 MFMA, published
BF16_TAGS = ("hv_syrk", "rv", "ax", "ata", "gram", "proj", "scores", "pv", "grid")
F64_TAGS = ("f64_factor", "f64_sweep", "f64_comp", "f64_cd", "f64_grid")
KERNEL_OF = {"hv_syrk": "gemm_bf16_nt_fast_kernel (H_in^V += T1^T X, lower tiles)", "rv": "gemm_bf16_nt_fast_kernel (R_v += alpha Z^T X)",
             "ax": "gemm_bf16_nt_stream_kernel (T1 = B1 X, Z = B1 dX + B2^T X~; per-head form: A X)", "ata": "gemm_bf16_nt_stream_kernel (sum_h A_h^T A_h)",
             "gram": "gemm_bf16_nt_fast_kernel (X^T X, dX^T X, O^T O)", "proj": "gemm_bf16_nt_stream_kernel (projections X W^T)", "scores": "gemm_bf16_nt_stream_kernel (Q K^T, fp32 out)",
             "pv": "gemm_bf16_nt_stream_kernel (O^T = V^T A^T)",
             "grid": "gemm_bf16_nt_fast_kernel (approximate grid-search costs)"}


def traffic_file(cfg_name, tag):
    return os.path.join(ROOT, "profiles", "gemm_bf16_%s_%s_hbm_traffic.txt" % (tag, cfg_name))


def measured_traffic(cfg_name, tag):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of
    `bench.py --roofline-probe` for this workload and launch (counters cannot be read from inside the timed run); None when
    no summary exists for them."""
    path = traffic_file(cfg_name, tag)
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def cpu_baseline(blk, cfg, hessians, out):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload, scaled to one attention block, by stage:
    quantize:  the oracle's set-up of one in-channel Hessian (U = Chol(H^-1)^T, P, S = R H^-1), times the number of distinct
               H_in of the block (1 for W_Q and W_K, one per KV head for W_V, 1 for W_O); plus Algorithm 1 on ONE step of N
               out-channels of W_Q (a pseudo-head of N rows with the matching corner of H_out; set-up time subtracted), times
               the number of N-row steps in the four layers;
    hessians_v / hessians_qk: the Table 1 sums of ONE (sequence, query head) pair (A_h, Y = A_h X_s, Y^T Y and the deviation
               term), times n_seqs * Hq; X_s^T X_s and dX_s^T X_s of one sequence, times n_seqs;
    hessian_out_proj: A_h V_h of one (sequence, head) pair on both paths, times n_seqs * Hq, and O_s^T O_s, dO_s^T O_s of one
               sequence, times n_seqs."""
    import numpy as np
    from oracle import turboboa_ref as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    dh, N, d = cfg.head_dim, min(cfg.block, cfg.head_dim), cfg.d_model
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    Hin = f(hessians["Hin_qk"]); Hout = f(hessians["Hout_q"][:1, :N, :N])
    R = f(hessians["R_qk"]) if hessians["R_qk"] is not None else None
    t = time.perf_counter()
    Hd = O.damp_hessian(Hin, 0.01); U = O.chol_inv_upper(Hd)
    if R is not None:
        O.sweep_P(R, U); O.residual_S(R, Hd)
    t_setup = time.perf_counter() - t
    del U, Hd
    t = time.perf_counter()
    O.quantize_layer(f(blk["Wq"][:N]), Hin, Hout, R, 1, bits=cfg.bits, block=N, group=cfg.group)
    t_step = max(time.perf_counter() - t - t_setup, 0.0)
    n_setups = 1 + cfg.n_kv_heads + 1
    n_steps = (cfg.d_q + 2 * cfg.d_kv + d) // N
    quant = n_setups * t_setup + n_steps * t_step
    xs = f(blk["X"][0]) if blk["X"] is not None else f(out["X"][0])
    xf = f(out["X_fp"][0]); wq = f(blk["Wq"][:dh]); wk = f(blk["Wk"][:dh]); wv = f(blk["Wv"][:dh])
    t = time.perf_counter()
    A, _, _ = O.attention_probs(xs, wq, wk)
    Y = A @ xs; Y.T @ Y
    if R is not None:
        Af, _, _ = O.attention_probs(xf, wq, wk)
        (Y - Af @ xf).T @ Y
    t_pair = time.perf_counter() - t
    t = time.perf_counter()
    xs.T @ xs
    if R is not None:
        (xs - xf).T @ xs
    t_seq = time.perf_counter() - t
    t = time.perf_counter()
    A, _, _ = O.attention_probs(xs, wq, wk); A @ (xs @ wv.T)
    if R is not None:
        Af, _, _ = O.attention_probs(xf, wq, wk); Af @ (xf @ wv.T)
    t_opair = time.perf_counter() - t
    Os = np.ascontiguousarray(xs[:, :cfg.d_q]) if cfg.d_q <= d else xs      # a stand-in of the right shape [L, Hq dh] for the Gram timing
    t = time.perf_counter()
    Os.T @ Os
    if R is not None:
        (Os - 0.5 * Os).T @ Os
    t_oseq = time.perf_counter() - t
    pairs = cfg.n_seqs * cfg.n_q_heads
    stages = {"hessians_qk": t_seq * cfg.n_seqs, "hessians_v": t_pair * pairs, "quantize": quant,
              "hessian_out_proj": t_opair * pairs + t_oseq * cfg.n_seqs}
    return {"value": sum(stages.values()), "unit": "s per attention block (extrapolated)", "cores": int(cores), "kind": "oracle",
            "stage_seconds": stages,
            "sample": "oracle set-up of one in-channel Hessian (U, P, S; d = %d): %.1f s, x %d distinct H_in; oracle quantize_layer on one step of "
                      "%d out-channels of W_Q minus that set-up: %.1f s, x %d steps in W_Q, W_K, W_V, W_O; Table 1 sums of one (sequence, head) "
                      "pair: %.2f s, x %d pairs; of one sequence for H_in, R: %.2f s, x %d; attention output of one pair: %.2f s, x %d; "
                      "O^T O, dO^T O of one sequence: %.2f s, x %d" % (d, t_setup, n_setups, N, t_step, n_steps, t_pair, pairs, t_seq, cfg.n_seqs,
                                                                        t_opair, pairs, t_oseq, cfg.n_seqs)}


def roofline_probe(ctx, cfg, torch, tag, zero=False, reps=0, persistent=False, seqs=8, bf16=False):
    """The command the HBM-traffic counter runs are made with: one plain copy of 1 GiB (a kernel of known traffic, to scale
    the counters), then ONE launch of the benchmark's dominant kernel in its launch shape, for all KV heads over a chunk of `seqs` (8)
    sequences, accumulating into fp32, operands in 16 x 32 blocks at the benchmark's row pitch (random values; IEEE half, as the
    build has them when the activations fit half, or bf16: the same kernel instantiated for the other MFMA):
      rv:      R_v[g] += alpha Z_g^T X  -- A = Z^T per KV head [d, 8 L], B = X^T [d, 8 L] shared by the heads, full product;
      hv_syrk: H_in^V[g] += T1_g^T X    -- the same operands, lower tiles only.
    zero: all-zero operands instead of random ones (same launch, same addresses: what the operand values alone do to the
    rate).  reps > 0: that many further launches, timed with events on the context's stream, their median printed."""
    import paper_2602_04929_amd as tb
    G = seqs
    K = G * cfg.seq_len
    n, Hkv = cfg.d_model, cfg.n_kv_heads
    g = torch.Generator(device="cuda"); g.manual_seed(1)
    src = torch.randn(1 << 28, generator=g, device="cuda")                    # 1 GiB
    dst = torch.empty_like(src)
    dt = torch.bfloat16 if bf16 else torch.float16
    ZT = torch.empty(Hkv, n, K + 256, dtype=dt, device="cuda")
    for h in range(Hkv):
        ZT[h] = torch.randn(n, K + 256, generator=g, device="cuda").to(dt)
    XT = torch.randn(n, K + 256, generator=g, device="cuda").to(torch.bfloat16).to(dt)      # the input: bf16 values in either type
    if zero:
        ZT.zero_(); XT.zero_()
    C = torch.zeros(Hkv, n, n, device="cuda")
    torch.cuda.synchronize()
    torch.mul(src, 1.0, out=dst)                                              # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    A = ZT[:, :, :K]; B = XT[None, :, :K].expand(Hkv, n, K)
    flags = tb.GEMM_A_TILED | tb.GEMM_B_TILED | (tb.GEMM_LOWER if tag == "hv_syrk" else 0) | (tb.GEMM_PERSISTENT if persistent else 0)
    ctx.gemm_bf16_nt(A, B, C_out=C, accumulate=True, flags=flags)
    torch.cuda.synchronize()
    cells = n * (n + 1) // 2 if tag == "hv_syrk" else n * n
    alg = Hkv * n * K * 2 + n * K * 2 + Hkv * 2 * 4 * cells                   # A read once, B read once, C read + written
    rec = {"probe": "copy 1 GiB, then gemm_bf16_nt accumulate (%s, %s operands), blocked operands, B shared by the batch" % (tag, "bf16" if bf16 else "half"),
           "copy_bytes_read": src.numel() * 4,
           "copy_bytes_written": src.numel() * 4, "gemm_batch": Hkv, "gemm_M": n, "gemm_K": K,
           "gemm_algorithmic_bytes": alg, "operands": "zero" if zero else "random"}
    if reps > 0:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]    # the context runs on torch's current stream
        ev[0].record()
        for i in range(reps):
            ctx.gemm_bf16_nt(A, B, C_out=C, accumulate=True, flags=flags)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
        flops = 2.0 * Hkv * cells * K
        rec.update({"reps": reps, "median_launch_ms": ms[reps // 2], "min_launch_ms": ms[0],
                    "median_tflops": flops / (ms[reps // 2] * 1e-3) / 1e12})
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="llama2-70b")
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
    ap.add_argument("--probe-tag", default="rv", choices=("rv", "hv_syrk"), help="with --roofline-probe: which launch")
    ap.add_argument("--probe-zero", action="store_true", help="with --roofline-probe: all-zero operands (same launch otherwise)")
    ap.add_argument("--probe-reps", type=int, default=0, help="with --roofline-probe: time this many further launches of the kernel")
    ap.add_argument("--probe-seqs", type=int, default=8, help="with --roofline-probe: sequences per launch (the contraction is seqs x seq_len deep)")
    ap.add_argument("--probe-bf16", action="store_true", help="with --roofline-probe: bf16 operands (what the build takes when an activation exceeds the range of half)")
    ap.add_argument("--probe-persistent", action="store_true", help="with --roofline-probe: the persistent form of the kernel (one resident workgroup per CU)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (heads would shard across GPUs; that is not built); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_04929_amd as tb
    from paper_2602_04929_amd import synth
    from paper_2602_04929_amd.pipeline import make_side_contexts, quantize_attention_block, reserve_workspaces

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(2)
    cfg = synth.CONFIGS[args.config]
    if args.n_seqs:
        cfg = synth.scaled(cfg, n_seqs=args.n_seqs)
    torch.cuda.set_device(0)
    if args.roofline_probe:
        ctx = tb.Context()
        roofline_probe(ctx, cfg, torch, args.probe_tag, zero=args.probe_zero, reps=args.probe_reps, persistent=args.probe_persistent, seqs=args.probe_seqs, bf16=args.probe_bf16)
        ctx.close()
        return
    note = lambda msg: print("bench.py: " + msg, file=sys.stderr, flush=True)      # progress on stderr; stdout carries the one JSON line
    note("building the %s block" % cfg.name)
    blk = synth.make_block(cfg, seed=0, device="cuda:0")
    if args.correlated:
        synth.apply_mix(blk, synth.correlated_mix(cfg.d_model, seed=0, device="cuda:0"))
    ctx = tb.Context()
    use_R = not args.no_R
    side = None if args.serial_layers else make_side_contexts(2)
    reserved = reserve_workspaces(ctx, cfg, side, seq_chunk=args.seq_chunk)      # sized by the library's queries: no call allocates afterwards

    def step(timings=None):
        return quantize_attention_block(ctx, blk, cfg, alpha=0.25, use_R=use_R, timings=timings, side_contexts=side, seq_chunk=args.seq_chunk)

    note("%d warm-up step(s)" % args.warmup)
    for _ in range(args.warmup):
        out = step()
    torch.cuda.synchronize()
    note("%d timed step(s)" % args.steps)
    ctxs = [ctx] + list(side or [])
    for c in ctxs:
        c.profile(True)
    stages = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(stages)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sec_per_block = dt / args.steps

    prof = {}
    for k in ctx.PROF_TAGS:
        recs = [c.profile_read(k) for c in ctxs]
        prof[k] = {f: sum(r[f] for r in recs) for f in ("ms", "launches", "flops")}
    for c in ctxs:
        c.profile(False)
    rate = lambda v: (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["ms"] > 0 else 0.0
    # the dominant kernel is taken among the launches of the Hessian builds, which have the GPU to themselves; the grid search's
    # product runs beside other layers' kernels on other streams, so its event times overstate it
    dom = max((k for k in BF16_TAGS if k != "grid"), key=lambda k: prof[k]["ms"])
    achieved = rate(prof[dom])
    roofline = {"bound": "mfma", "kernel": KERNEL_OF[dom], "tag": dom, "achieved": achieved,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": prof[dom]["ms"] / max(1, prof[dom]["launches"]), "launches": prof[dom]["launches"],
                "ms_per_step": prof[dom]["ms"] / args.steps,
                "traffic": measured_traffic(cfg.name if not args.n_seqs else "", dom),
                "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy)"}
    # the fp64 matrix-core GEMMs of quantize_layer (compensation, sweep updates, P, scale refinement): the largest tag with counted flops
    f64_counted = [k for k in F64_TAGS if prof[k]["flops"] > 0]
    dom64 = max(f64_counted, key=lambda k: prof[k]["ms"]) if f64_counted else None
    roofline_f64 = None
    if dom64:
        tot_ms = sum(prof[k]["ms"] for k in f64_counted); tot_fl = sum(prof[k]["flops"] for k in f64_counted)
        roofline_f64 = {"bound": "mfma", "kernel": "gemm_f64_kernel", "tag": dom64, "achieved": rate(prof[dom64]), "peak": PEAK_F64_TFLOPS,
                        "unit": "TFLOP/s", "frac": rate(prof[dom64]) / PEAK_F64_TFLOPS, "ms_per_step": prof[dom64]["ms"] / args.steps,
                        "all_counted_tags": {"ms_per_step": tot_ms / args.steps, "achieved": tot_fl / (tot_ms * 1e-3) / 1e12 if tot_ms > 0 else 0.0},
                        "note": "tagged launches run beside other layers' kernels on other streams: rates are lower bounds"}
    kernels = {k: {"ms_per_step": v["ms"] / args.steps, "launches_per_step": v["launches"] // args.steps, "tflops": rate(v)} for k, v in prof.items()}
    bf_ms = sum(prof[k]["ms"] for k in BF16_TAGS); bf_fl = sum(prof[k]["flops"] for k in BF16_TAGS)
    util_all = (bf_fl / (bf_ms * 1e-3) / 1e12) / PEAK_BF16_TFLOPS if bf_ms > 0 else 0.0

    rec = {
        "metric": "sec per attention block (Wq,Wk,Wv,Wo) quantized INT%d; MFMA util %%" % cfg.bits,
        "value": sec_per_block, "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_block * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 / fp16 (Hessian contractions, (hi, lo) operand pairs, fp32 accumulate) + f64 (quantization)", "data": "synthetic",
        "config": {"workload": "%s attention block: d_model=%d, %d q-heads / %d kv-heads x %d, %d seqs x %d tokens, INT%d, N=%d, "
                               "group=%d, alpha=0.25, R %s, adaptive grid, 1 CD sweep"
                               % (cfg.name, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n_seqs, cfg.seq_len, cfg.bits,
                                  cfg.block, cfg.group, "on" if use_R else "off") + (", correlated channels" if args.correlated else "")},
        "mfma_util_pct": 100.0 * util_all,
        "mfma_util_note": "all tagged bf16 / fp16 GEMM launches of the step: sum of algorithmic flops / sum of kernel time / 2.5 PFLOP/s",
        "stage_seconds": {k: v / args.steps for k, v in stages.items()},
        "bf16_gemm_seconds_per_step": bf_ms * 1e-3 / args.steps,
        "f64_gemm_seconds_per_step": sum(prof[k]["ms"] for k in F64_TAGS) * 1e-3 / args.steps,
        "kernels": kernels,
        "losses": {k: out[k]["loss"] for k in ("q", "k", "v", "o")},
        "workspace_gib": sum(c.workspace_bytes() for c in ctxs) / 2 ** 30,
        "workspace_reserved_gib": sum(reserved) / 2 ** 30,
        "grid_search": {"two_phase_passes": sum(c.counter(0) for c in ctxs), "layers_rerun_exact": sum(c.counter(1) for c in ctxs)},
        "roofline": roofline,
        "roofline_f64": roofline_f64,
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
        note("timing the oracle on the host cores (bounded sample)")
        rec["cpu_baseline"] = cpu_baseline(blk, cfg, out["hessians"], out)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
