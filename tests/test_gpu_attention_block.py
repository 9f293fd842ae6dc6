"""Whole hot path on the tiny configuration, end to end against the oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O
from paper_2602_04929_amd import synth
from tests.parity import compare_layer, stacked

pytestmark = pytest.mark.gpu


def f64(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


def oracle_block(blk, cfg, alpha=0.25, use_R=True):
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    X, Xf = f64(blk["X"]), f64(blk["X_fp"]) if use_R else None
    W = {k: f64(blk[k]) for k in ("Wq", "Wk", "Wv", "Wo")}
    Hs = O.build_hessians(X, Xf, W["Wq"], W["Wk"], W["Wv"], W["Wo"], Hq, Hkv, dh, alpha=alpha)
    kw = dict(bits=cfg.bits, block=cfg.block, group=cfg.group)
    out = {"hessians": Hs}
    out["q"] = O.quantize_layer(W["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq, **kw)
    out["k"] = O.quantize_layer(W["Wk"], Hs["Hin_qk"], Hs["Hout_k"], Hs["R_qk"], Hkv, **kw)
    out["v"] = O.quantize_layer(W["Wv"], Hs["Hin_v"], Hs["Hout_v"], Hs["R_v"], Hkv, **kw)
    Hin_o, R_o = O.build_hessian_out_proj(X, Xf, out["q"]["W_deq"], out["k"]["W_deq"], out["v"]["W_deq"], W["Wq"], W["Wk"], W["Wv"],
                                          Hq, Hkv, dh, alpha=alpha)
    out["o"] = O.quantize_layer(W["Wo"], Hin_o, None, R_o, 1, **dict(kw, block=cfg.d_model))
    return out


@pytest.mark.parametrize("use_R,side,stack", [(True, False, True), (False, False, True), (True, True, True), (True, False, False), (True, True, False)])
def test_tiny_config_end_to_end(lib, use_R, side, stack):
    """Config 1 (d_model 256, 4 heads x 64, 8 x 128 tokens, INT2, N = 4, seed 0): every layer against the oracle,
    each side building its own Hessians from the same X.  stack: W_Q and W_K through tboa_quantize_layer as one layer of
    Hq + Hkv heads (they share H_in and R), which must give what the two separate calls give."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    cfg = synth.CONFIGS["tiny"]
    blk = synth.make_block(cfg, seed=0, device="cuda")
    ctx = lib.Context()
    from paper_2602_04929_amd.pipeline import make_side_contexts
    sc = make_side_contexts(2) if side else None        # W_Q, W_K, W_V on three streams from three host threads
    got = quantize_attention_block(ctx, blk, cfg, use_R=use_R, side_contexts=sc, stack_qk=stack)
    torch.cuda.synchronize()
    for c in sc or []:
        c.close()
    want = oracle_block(blk, cfg, use_R=use_R)
    if stack:
        want["qk"] = stacked(want["q"], want["k"])
        for layer, rows in (("q", slice(0, cfg.n_q_heads * cfg.head_dim)), ("k", slice(cfg.n_q_heads * cfg.head_dim, None))):
            assert torch.equal(got[layer]["codes"], got["qk"]["codes"][rows]) and torch.equal(got[layer]["W_deq"], got["qk"]["W_deq"][rows])
            compare_layer(got[layer], want[layer], label=layer + " (rows of the stacked layer)")
    for layer in ("qk", "v", "o") if stack else ("q", "k", "v", "o"):
        frac = compare_layer(got[layer], want[layer], label=layer)
        print("tiny R=%s layer %s: codes identical %.4f%%" % (use_R, layer, 100 * frac), flush=True)
    ctx.close()


def test_tiny_config_correlated_channels(lib):
    """The tiny configuration with correlated channels (X <- X (I + 0.3 low-rank)): iid channels give a nearly diagonal
    H_in, under which the compensation and the P term of the sweep do little; here they carry weight."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    cfg = synth.CONFIGS["tiny"]
    blk = synth.make_block(cfg, seed=0, device="cuda")
    synth.apply_mix(blk, synth.correlated_mix(cfg.d_model, seed=0, device="cuda"))
    ctx = lib.Context()
    got = quantize_attention_block(ctx, blk, cfg, use_R=True)
    torch.cuda.synchronize()
    want = oracle_block(blk, cfg, use_R=True)
    Hin = want["hessians"]["Hin_qk"]
    dg = np.sqrt(np.diag(Hin))
    off = np.abs(Hin / dg[:, None] / dg[None, :] - np.eye(cfg.d_model)).max()
    assert off > 0.3, "the mix should couple the channels"
    want["qk"] = stacked(want["q"], want["k"])
    for layer in ("qk", "v", "o"):
        frac = compare_layer(got[layer], want[layer], label=layer)
        print("tiny correlated layer %s: codes identical %.4f%%, largest off-diagonal correlation %.2f" % (layer, 100 * frac, off), flush=True)
    ctx.close()


@pytest.mark.parametrize("seed", [1, 2])
def test_tiny_config_other_seeds(lib, seed):
    """The tiny configuration end to end on two more seeds (the parity cases above all use seed 0)."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    cfg = synth.CONFIGS["tiny"]
    blk = synth.make_block(cfg, seed=seed, device="cuda")
    ctx = lib.Context()
    got = quantize_attention_block(ctx, blk, cfg, use_R=True)
    torch.cuda.synchronize()
    want = oracle_block(blk, cfg, use_R=True)
    want["qk"] = stacked(want["q"], want["k"])
    for layer in ("qk", "v", "o"):
        frac = compare_layer(got[layer], want[layer], label=layer)
        print("tiny seed %d layer %s: codes identical %.4f%%" % (seed, layer, 100 * frac), flush=True)
    ctx.close()


BF16_CASES = [
    # name, d_model, q heads, kv heads, head_dim, sequences, tokens per sequence.  16 tokens per channel: a quarter of the
    # ratio of the named configurations (64), whose sums over the tokens average the rounding of the 16-bit operands further
    ("mha-256", 256, 4, 4, 64, 16, 256),
    ("gqa-256", 256, 8, 2, 32, 16, 256),
    ("mha-512", 512, 3, 3, 96, 8, 768),              # odd tile counts: 2 x 2 tiles of d, 3 x 3 of L, head_dim not a power of two
]


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("case", BF16_CASES, ids=[c[0] for c in BF16_CASES])
def test_bf16_block_end_to_end(lib, case, seed):
    """bf16 inputs (the path the benchmark times), each side building its own Hessians from the same X.

    What is compared at the full bar, on every seed: the Hessians (fp32-grade bounds), and every layer with the oracle reading
    the Hessians the library built (so that only the quantizer differs).

    Each side on its OWN Hessians is compared with what the method allows.  The Hessians agree to 1e-7 .. 1e-5, and the
    method takes discrete decisions on them: the grid search an argmin over candidates whose costs near the minimum differ
    by arbitrarily little, the sweep a rounding of w / s.  A decision that falls within that 1e-6 of a tie goes the other way;
    the rows of a head are coupled through H_out, so the compensation and the scale refinement then move the later columns
    and the scales of the whole head by 1e-3, and a handful of rows drift apart.  Both results are outputs of the same
    algorithm on Hessians that agree to fp32 rounding and their losses agree to a fraction of a percent.  Over seeds 0..2 of
    the three cases most layers come out with identical codes (printed); the asserted floor is what the worst case shows.
    W_O is the most sensitive: its H_in = O^T O is built from attention outputs, averages of the values, and is close to
    singular (condition number printed), so U = Chol(H_in^-1)^T moves by cond * eps."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    name, d, hq, hkv, dh, S, L = case
    cfg = synth.scaled(synth.CONFIGS["llama2-7b"], name=name, d_model=d, n_q_heads=hq, n_kv_heads=hkv, head_dim=dh, n_seqs=S, seq_len=L,
                       n_outlier=3, block=8)
    blk = synth.make_block(cfg, seed=seed, device="cuda")
    ctx = lib.Context()
    got = quantize_attention_block(ctx, blk, cfg, use_R=True)
    torch.cuda.synchronize()
    want = oracle_block(blk, cfg, use_R=True)
    want["qk"] = stacked(want["q"], want["k"])
    Hs, Hw = got["hessians"], want["hessians"]
    for k in ("Hin_qk", "R_qk", "Hout_q", "Hout_k", "Hin_v", "R_v", "Hout_v"):
        g, w = f64(Hs[k]), Hw[k]
        e = np.abs(g - w).max() / np.abs(w).max()
        print("  %s seed %d %s: max |err| / max |entry| = %.2e" % (name, seed, k, e), flush=True)
        assert e <= (6e-5 if k.startswith("R_v") else 2e-6), (k, e)
    Xn, Xfn = f64(blk["X"]), f64(blk["X_fp"])
    wq, wk, wv = (f64(got[k]["W_deq"]) for k in ("q", "k", "v"))       # the oracle's Table 1 sums from the library's own W_deq
    Ho_w, Ro_w = O.build_hessian_out_proj(Xn, Xfn, wq, wk, wv, f64(blk["Wq"]), f64(blk["Wk"]), f64(blk["Wv"]), hq, hkv, dh, alpha=0.25)
    for k, g, w in (("Hin_o", got["Hin_o"], Ho_w), ("R_o", got["R_o"], Ro_w)):
        e = np.abs(f64(g) - w).max() / np.abs(w).max()
        print("  %s seed %d %s: max |err| / max |entry| = %.2e" % (name, seed, k, e), flush=True)
        assert e <= (1e-6 if k == "Hin_o" else 1e-5)
    # ---- the quantizer alone: the oracle on the Hessians the library built, at the full bar
    kw = dict(bits=cfg.bits, block=cfg.block, group=cfg.group)
    W = {k: f64(blk[k]) for k in ("Wq", "Wk", "Wv", "Wo")}
    Hl = {k: (f64(v) if v is not None and k != "fp_cache" else None) for k, v in Hs.items()}
    iso = {"q": O.quantize_layer(W["Wq"], Hl["Hin_qk"], Hl["Hout_q"], Hl["R_qk"], hq, **kw),
           "k": O.quantize_layer(W["Wk"], Hl["Hin_qk"], Hl["Hout_k"], Hl["R_qk"], hkv, **kw),
           "v": O.quantize_layer(W["Wv"], Hl["Hin_v"], Hl["Hout_v"], Hl["R_v"], hkv, **kw),
           "o": O.quantize_layer(W["Wo"], f64(got["Hin_o"]), None, f64(got["R_o"]), 1, **dict(kw, block=cfg.d_model))}
    iso["qk"] = stacked(iso["q"], iso["k"])
    for layer in ("qk", "v", "o"):
        frac = compare_layer(got[layer], iso[layer], label="%s seed %d %s (oracle on the library's Hessians)" % (name, seed, layer))
        assert frac == 1.0, (layer, frac)
    # ---- each side on its own Hessians
    cond = {}
    for layer, H in (("v", Hw["Hin_v"][0]), ("o", Ho_w)):
        ev = np.linalg.eigvalsh(O.damp_hessian(H, 0.01)); cond[layer] = ev[-1] / ev[0]
    for layer, min_codes, max_loss in (("qk", 0.95, 5e-3), ("v", 0.95, 5e-3), ("o", 0.90, 1e-1)):
        e2e = (got[layer]["codes"].cpu().numpy() == want[layer]["codes"]).mean()
        rel_loss = abs(got[layer]["loss"] - want[layer]["loss"]) / abs(want[layer]["loss"])
        print("bf16 end to end %s seed %d layer %s: each side its own Hessians: codes identical %.4f%%, loss rel. diff %.1e%s" %
              (name, seed, layer, 100 * e2e, rel_loss, "" if layer == "qk" else "; cond(H_in) %.1e" % cond[layer]), flush=True)
        assert e2e >= min_codes and rel_loss <= max_loss, (layer, e2e, rel_loss)
    ctx.close()
