#!/usr/bin/env python3
"""Quantization time of one attention block against the number N of out-channels quantized jointly per step.

The paper's one timing experiment (Table 2: wall time of BoA, N = 1, and of joint quantization with N = 4 .. 64) has the
shape "time falls steeply up to N = 16 and flattens after": the number of sequential out-channel steps per head is
ceil(d_h / N), each of which holds a full in-channel sweep (Algorithm 3).  This script measures the same curve for the HIP
library on one synthetic block: Hessians are built once, then W_Q, W_K, W_V (Algorithm 1) are quantized for every N.
W_O has no out-channel coupling (all rows one step) and is timed once.

    python -m paper_2602_04929_amd.sweep_block [--config llama2-7b] [--blocks 1,4,8,16,32,64] [--n-seqs 128]

Prints one line per setting and a final JSON line."""
import argparse
import json
import time

import torch

import paper_2602_04929_amd as tb
from paper_2602_04929_amd import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="llama2-7b")
    ap.add_argument("--blocks", default="1,4,8,16,32,64")
    ap.add_argument("--n-seqs", type=int, default=0)
    args = ap.parse_args()
    cfg = synth.CONFIGS[args.config]
    if args.n_seqs:
        cfg = synth.scaled(cfg, n_seqs=args.n_seqs)
    blk = synth.make_block(cfg, seed=0, device="cuda:0")
    ctx = tb.Context()
    X_fp = blk["X_fp"] if blk["signs"] is None else ctx.hadamard_rotate(blk["X_fp"], blk["signs"])
    X = blk["X"] if blk["X"] is not None else ctx.act_fakequant(X_fp, cfg.act_bits)
    Hs = ctx.build_hessians(X, X_fp, blk["Wq"], blk["Wk"], blk["Wv"], blk["Wo"], cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, alpha=0.25)
    layers = (("q", "Wq", "Hin_qk", "Hout_q", "R_qk", cfg.n_q_heads), ("k", "Wk", "Hin_qk", "Hout_k", "R_qk", cfg.n_kv_heads),
              ("v", "Wv", "Hin_v", "Hout_v", "R_v", cfg.n_kv_heads))

    def run(N, full):
        """full: R, adaptive grid and one CD sweep (the paper's F1+F2+F3); else plain BoA-style steps (F1 only)."""
        kw = dict(bits=cfg.bits, block=N, group=cfg.group)
        if not full:
            kw.update(adaptive_grid=False, cd_iters=0)
        out = {}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for name, w, hin, hout, r, nh in layers:
            t = time.perf_counter()
            res = ctx.quantize_layer(blk[w], Hs[hin], Hs[hout], Hs[r] if full else None, nh, **kw)
            torch.cuda.synchronize()
            out[name] = time.perf_counter() - t
            out["loss_" + name] = res["loss"]
        out["qkv"] = time.perf_counter() - t0
        return out

    rows = []
    run(cfg.head_dim, True)   # warm-up: workspace, tile tables
    for full in (False, True):
        for N in [int(b) for b in args.blocks.split(",")]:
            r = run(N, full)
            r.update(N=N, setting="R + adaptive grid + CD" if full else "joint steps only", steps_per_head=-(-cfg.head_dim // N))
            rows.append(r)
            print("%-24s N=%-3d steps/head=%-4d  W_Q %.3f s  W_K %.3f s  W_V %.3f s  sum %.3f s" %
                  (r["setting"], N, r["steps_per_head"], r["q"], r["k"], r["v"], r["qkv"]), flush=True)
    print(json.dumps({"config": cfg.name, "n_seqs": cfg.n_seqs, "rows": rows}))
    ctx.close()


if __name__ == "__main__":
    main()
