"""One attention block through the library: the sequence of C-ABI calls of the hot path, nothing else."""
from __future__ import annotations

import threading
import time

import torch


def make_side_contexts(n=2):
    """Contexts on fresh streams (default priority) for layers that may run beside the main context's work."""
    import paper_2602_04929_amd as tb
    return [tb.Context(stream=torch.cuda.Stream()) for _ in range(n)]


def reserve_workspaces(ctx, cfg, side_contexts=None, stack_qk=True, cd_iters=1, adaptive_grid=True, seq_chunk=0):
    """Sizes every context's workspace for one attention block of `cfg` ahead of the calls (tboa_hessian_workspace_bytes,
    tboa_quantize_workspace_bytes, tboa_reserve_workspace), so that no call of quantize_attention_block allocates.  Returns
    the bytes reserved per context."""
    import paper_2602_04929_amd as tb
    dt = {"fp32": torch.float32, "bf16": torch.bfloat16}[cfg.dtype]
    wd = tb.F32 if cfg.dtype == "fp32" else tb.BF16
    Hq, Hkv, dh, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_model

    def layer(d_out, d_in, n_heads, per_head, block, with_H_out=True):
        return ctx.quantize_workspace_bytes(tb.LayerDesc(d_out, d_in, n_heads, int(per_head), cfg.bits, block, cfg.group, wd, cd_iters,
                                                         int(adaptive_grid), 100, 0.8, 0.01, 0.0), with_H_out, True)
    hess = ctx.hessian_workspace_bytes(d, Hq, Hkv, dh, cfg.n_seqs, cfg.seq_len, dt, seq_chunk=seq_chunk)
    o = layer(d, Hq * dh, 1, False, d, with_H_out=False)
    v = layer(Hkv * dh, d, Hkv, True, cfg.block)
    first = [layer((Hq + Hkv) * dh, d, Hq + Hkv, False, cfg.block)] if stack_qk else [layer(Hq * dh, d, Hq, False, cfg.block), layer(Hkv * dh, d, Hkv, False, cfg.block)]
    jobs = first + [v]
    ctxs = [ctx] + list(side_contexts or [])[:len(jobs) - 1]
    need = [0] * len(ctxs)
    for i, b in enumerate(jobs):          # job i runs on context i when there are side contexts, else all on the main one
        need[i if i < len(ctxs) else 0] = max(need[i if i < len(ctxs) else 0], b)
    need[0] = max(need[0], hess, o, *(jobs if len(ctxs) == 1 else []))
    for c, n in zip(ctxs, need):
        c.reserve_workspace(n)
    return need


def _split_stacked(res, rows_q, heads_q):
    """Per-layer views of a result of W_Q and W_K quantized as one stacked layer (heads are independent)."""
    def part(rs, hs):
        lph, terms = res["loss_per_head"][hs], res["loss_per_head_terms"][hs]
        d = {k: res[k][rs] for k in ("codes", "scales", "zeros", "W_deq")}
        d.update(loss_per_head=lph, loss_per_head_terms=terms, loss=float(sum(lph)),
                 loss_quad=float(sum(t[0] for t in terms)), loss_cross=float(sum(t[1] for t in terms)))
        return d
    return part(slice(0, rows_q), slice(0, heads_q)), part(slice(rows_q, None), slice(heads_q, None))


def quantize_attention_block(ctx, blk, cfg, alpha=0.25, use_R=True, with_R_v=True, cd_iters=1, adaptive_grid=True,
                             damp=0.01, seq_chunk=0, timings=None, side_contexts=None, stack_qk=True, hout_k_from_quantized_q=False, kv_bits=0):
    """(rotation, activation fake-quant ->) Hessians -> W_Q, W_K, W_V -> output-projection Hessian -> W_O.

    blk: dict from synth.make_block (device tensors); cfg: synth.BlockConfig.  Returns dict of per-layer results
    and the Hessians.  `timings` (a dict) receives per-stage seconds measured with stream synchronisation.
    side_contexts: more contexts on streams of their own (see make_side_contexts): the layers then run side by side.
    stack_qk: W_Q and W_K share H_in and R (Table 1) and their heads are independent, so [W_Q; W_K] goes through
    tboa_quantize_layer as ONE layer of Hq + Hkv heads with H_out = [H_out^Q; H_out^K]: one factorisation of H_in, one P,
    steps over twice the rows.  out["qk"] is that call's result, out["q"] and out["k"] are views of it (their losses are the sums
    over their heads).
    hout_k_from_quantized_q: the other reading of Algorithm 1 line 4 (Hessians formed inside the loop over the layers): W_Q is
    quantized first and H_out of W_K is sum_h Q_h^T Q_h with Q_h from the DEQUANTIZED W_Q (tboa_build_hout); W_Q and W_K then go
    through tboa_quantize_layer one after the other (no stacking, no side contexts for them).
    kv_bits > 0: the keys are held in a kv_bits-bit cache (Sec. 4.2): H_out of W_Q is built from the fake-quantized keys
    (tboa_build_hout_q_kv_cache)."""
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    X_fp = blk["X_fp"]
    X = blk["X"]

    def stage(name, fn):
        if timings is None:
            return fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        timings[name] = timings.get(name, 0.0) + time.perf_counter() - t
        return out

    if blk.get("signs") is not None:      # randomised Hadamard rotation ahead of everything else (outlier suppression)
        X_fp = stage("hadamard_rotate", lambda: ctx.hadamard_rotate(X_fp, blk["signs"]))
        if X is not None:
            X = ctx.hadamard_rotate(X, blk["signs"])
    if X is None:      # weight-activation setting: the quantized path sees per-token fake-quantized activations
        X = stage("act_fakequant", lambda: ctx.act_fakequant(X_fp, cfg.act_bits))
    Xf = X_fp if use_R else None
    hargs = (X, Xf, blk["Wq"], blk["Wk"], blk["Wv"], blk["Wo"], Hq, Hkv, dh)
    hkw = dict(alpha=alpha, with_R_v=with_R_v, seq_chunk=seq_chunk, keep_fp_projections=True)
    kw = dict(bits=cfg.bits, block=cfg.block, group=cfg.group, cd_iters=cd_iters, adaptive_grid=adaptive_grid, damp=damp)
    out = {"X": X, "X_fp": X_fp}
    Hs = stage("build_hessians", lambda: ctx.build_hessians(*hargs, **hkw))
    if kv_bits:
        Hs["Hout_q"] = stage("build_hout_q_kv_cache", lambda: ctx.build_hout_q_kv_cache(X, blk["Wk"], Hq, Hkv, dh, kv_bits))
    if hout_k_from_quantized_q:
        stack_qk = False
        out["q"] = stage("quantize_q", lambda: ctx.quantize_layer(blk["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq, **kw))
        Hs["Hout_k"] = stage("build_hout_k", lambda: ctx.build_hout(Hs["Hin_qk"], out["q"]["W_deq"], Hkv, Hq // Hkv, dh))
        jobs = (("k", (blk["Wk"], Hs["Hin_qk"], Hs["Hout_k"], Hs["R_qk"], Hkv)), ("v", (blk["Wv"], Hs["Hin_v"], Hs["Hout_v"], Hs["R_v"], Hkv)))
    elif stack_qk:
        Wqk = blk.get("Wqk")
        if Wqk is None:
            Wqk = torch.cat([blk["Wq"], blk["Wk"]], dim=0)
        jobs = (("qk", (Wqk, Hs["Hin_qk"], torch.cat([Hs["Hout_q"], Hs["Hout_k"]], dim=0), Hs["R_qk"], Hq + Hkv)),
                ("v", (blk["Wv"], Hs["Hin_v"], Hs["Hout_v"], Hs["R_v"], Hkv)))
    else:
        jobs = (("q", (blk["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq)), ("k", (blk["Wk"], Hs["Hin_qk"], Hs["Hout_k"], Hs["R_qk"], Hkv)),
                ("v", (blk["Wv"], Hs["Hin_v"], Hs["Hout_v"], Hs["R_v"], Hkv)))
    if side_contexts:
        # W_Q, W_K, W_V are independent given the Hessians: one context (and stream) each, driven from three host threads, so
        # that the latency-bound steps of one layer (factorisation panels, in-channel sweeps) run beside the GEMMs of another.
        # (Starting W_Q and W_K already beside the H_in^V build, which tboa_build_hessians allows, was measured and gains
        # nothing more: that build keeps the matrix cores busy by itself.)
        def run(name, c, args):
            with torch.cuda.stream(c._stream):
                out[name] = c.quantize_layer(*args, **kw)

        def all_three():
            main = torch.cuda.current_stream()
            ctxs = (ctx,) + tuple(side_contexts[:len(jobs) - 1])
            for c in ctxs[1:]:
                c._stream.wait_stream(main)
            threads = [threading.Thread(target=run, args=(name, c, args)) for (name, args), c in zip(jobs, ctxs)]
            for t in threads:
                t.start()
            for t in threads:
                t.join()
            for c in ctxs[1:]:
                main.wait_stream(c._stream)
            for name, _ in jobs[1:]:
                for v in out[name].values():
                    if torch.is_tensor(v):
                        v.record_stream(main)
        stage("quantize_qkv", all_three)
    else:
        for name, args in jobs:
            out[name] = stage("quantize_" + name, lambda a=args: ctx.quantize_layer(*a, **kw))
    if stack_qk:
        out["q"], out["k"] = _split_stacked(out["qk"], Hq * dh, Hq)
    out["hessians"] = Hs
    Ho = stage("build_hessian_out_proj", lambda: ctx.build_hessian_out_proj(
        X, Xf, out["q"]["W_deq"], out["k"]["W_deq"], out["v"]["W_deq"], blk["Wq"], blk["Wk"], blk["Wv"], Hq, Hkv, dh,
        alpha=alpha, seq_chunk=seq_chunk, fp_cache=Hs.get("fp_cache")))
    out["Hin_o"], out["R_o"] = Ho
    kwo = dict(kw, block=cfg.d_model)      # H_out = I: all rows form one step
    out["o"] = stage("quantize_o", lambda: ctx.quantize_layer(blk["Wo"], Ho[0], None, Ho[1], 1, **kwo))
    return out


def quantize_blocks(ctx, blocks, X, X_fp, cfg, alpha=0.25, cd_iters=1, adaptive_grid=True, damp=0.01, side_contexts=None, **attn_kw):
    """Several transformer blocks in a row (attention + gated MLP, residual connections, no normalisation layers), carrying both
    activation streams from block to block: X through the quantized weights, X_fp through the full-precision ones, so that the
    deviation X - X_fp every block sees is the one accumulated through the blocks before it (what Prop. 3.2 corrects).

    blocks: list of dicts with Wq, Wk, Wv, Wo, Wg, Wu, Wd; X, X_fp [S, L, d] (X_fp is X for the first block of a model).
    Per block: quantize_attention_block; Xa = X + attention(X; dequantized) W_O,deq^T (and the same with the full-precision
    weights on X_fp); quantize_mlp on (Xa, Xa_fp); X <- Xa + act W_down,deq^T.  Returns the per-block results and the final
    activations.  Every product runs in the library (tboa_attention_forward, tboa_linear_forward, tboa_swiglu_forward)."""
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    results = []
    for b in blocks:
        blk = dict(Wq=b["Wq"], Wk=b["Wk"], Wv=b["Wv"], Wo=b["Wo"], X=X, X_fp=X_fp, signs=None)
        att = quantize_attention_block(ctx, blk, cfg, alpha=alpha, cd_iters=cd_iters, adaptive_grid=adaptive_grid, damp=damp,
                                       side_contexts=side_contexts, **attn_kw)
        O_q = ctx.attention_forward(X, att["q"]["W_deq"], att["k"]["W_deq"], att["v"]["W_deq"], Hq, Hkv, dh)
        O_f = ctx.attention_forward(X_fp, b["Wq"], b["Wk"], b["Wv"], Hq, Hkv, dh)
        Xa = ctx.linear_forward(O_q, att["o"]["W_deq"], residual=X)
        Xa_fp = ctx.linear_forward(O_f, b["Wo"], residual=X_fp)
        mlp = quantize_mlp(ctx, dict(Wg=b["Wg"], Wu=b["Wu"], Wd=b["Wd"], M=Xa, M_fp=Xa_fp), cfg, alpha=alpha, cd_iters=cd_iters,
                           adaptive_grid=adaptive_grid, damp=damp)
        X = ctx.linear_forward(mlp["act"], mlp["down"]["W_deq"], residual=Xa)
        X_fp = ctx.linear_forward(mlp["act_fp"], b["Wd"], residual=Xa_fp)
        results.append(dict(attention=att, mlp=mlp, X_out=X, X_fp_out=X_fp, X_mid=Xa, X_fp_mid=Xa_fp))
    return results, X, X_fp


def quantize_mlp(ctx, mlp, cfg, alpha=0.25, use_R=True, cd_iters=1, adaptive_grid=True, damp=0.01, timings=None,
                 stack_gate_up=True):
    """The gated MLP of the block: W_gate and W_up share their input (one Hessian), W_down sees silu(gate) * up computed
    from the dequantized W_gate, W_up on the quantized-path input (and from the full-precision weights on the
    full-precision input for its deviation correlation).  Every layer: tboa_quantize_layer with H_out = NULL."""
    def stage(name, fn):
        if timings is None:
            return fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        timings[name] = timings.get(name, 0.0) + time.perf_counter() - t
        return out

    M, M_fp = mlp["M"], mlp["M_fp"]
    Mf = M_fp if use_R else None
    kw = dict(bits=cfg.bits, group=cfg.group, cd_iters=cd_iters, adaptive_grid=adaptive_grid, damp=damp)
    out = {}
    H, R = stage("hessian_gate_up", lambda: ctx.build_hessian_linear(M, Mf, alpha))
    if stack_gate_up:   # same H_in and R, rows decouple (H_out = I): one layer of 2 d_ff rows, one factorisation and one P
        Wgu = torch.cat([mlp["Wg"], mlp["Wu"]], dim=0)
        res = stage("quantize_gate_up", lambda: ctx.quantize_layer(Wgu, H, None, R, 1, block=2 * cfg.d_ff, **kw))
        out["gate_up"] = res
        for name, rs in (("gate", slice(0, cfg.d_ff)), ("up", slice(cfg.d_ff, None))):
            out[name] = {k: res[k][rs] for k in ("codes", "scales", "zeros", "W_deq")}
    else:
        out["gate"] = stage("quantize_gate", lambda: ctx.quantize_layer(mlp["Wg"], H, None, R, 1, block=cfg.d_ff, **kw))
        out["up"] = stage("quantize_up", lambda: ctx.quantize_layer(mlp["Wu"], H, None, R, 1, block=cfg.d_ff, **kw))
    act = stage("swiglu", lambda: ctx.swiglu_forward(M, out["gate"]["W_deq"], out["up"]["W_deq"]))
    act_fp = stage("swiglu", lambda: ctx.swiglu_forward(M_fp, mlp["Wg"], mlp["Wu"])) if use_R else None
    Hd, Rd = stage("hessian_down", lambda: ctx.build_hessian_linear(act, act_fp, alpha))
    out["down"] = stage("quantize_down", lambda: ctx.quantize_layer(mlp["Wd"], Hd, None, Rd, 1, block=cfg.d_model, **kw))
    out["hessians"] = dict(H_gate_up=H, R_gate_up=R, H_down=Hd, R_down=Rd)
    out["act"], out["act_fp"] = act, act_fp
    return out
