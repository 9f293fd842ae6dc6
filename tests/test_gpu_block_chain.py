"""The forward entry points, the other reading of Algorithm 1 line 4 (H_out of W_K from the quantized W_Q) and the driver
that carries both activation streams from one transformer block to the next, against the oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O
from paper_2602_04929_amd import synth
from tests.parity import compare_layer, stacked

pytestmark = pytest.mark.gpu


def f64(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context()
    yield c
    c.close()


def test_forward_entry_points_fp32(ctx):
    cfg = synth.scaled(synth.CONFIGS["tiny"], d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, n_seqs=2, seq_len=40, n_outlier=2)
    b = synth.make_block(cfg, seed=3, device="cuda")
    Og = ctx.attention_forward(b["X"], b["Wq"], b["Wk"], b["Wv"], 4, 2, 16)
    want = O.attention_output(f64(b["X"]), f64(b["Wq"]), f64(b["Wk"]), f64(b["Wv"]), 4, 2, 16)
    assert Og.shape == (2, 40, 64) and np.abs(f64(Og) - want).max() <= 1e-6 * np.abs(want).max()
    Y = ctx.linear_forward(Og, b["Wo"], residual=b["X"])
    wantY = f64(Og) @ f64(b["Wo"]).T + f64(b["X"])
    assert np.abs(f64(Y) - wantY).max() <= 1e-6 * np.abs(wantY).max()
    Y0 = ctx.linear_forward(Og, b["Wo"])
    assert np.abs(f64(Y0) - f64(Og) @ f64(b["Wo"]).T).max() <= 1e-6 * np.abs(wantY).max()


@pytest.mark.parametrize("dequantized", [False, True])
def test_forward_entry_points_bf16(ctx, dequantized):
    cfg = synth.scaled(synth.CONFIGS["llama2-7b"], d_model=264, n_q_heads=4, n_kv_heads=2, head_dim=32, n_seqs=3, seq_len=320, n_outlier=3)
    b = synth.make_block(cfg, seed=4, device="cuda")
    Wq, Wk, Wv, Wo = b["Wq"], b["Wk"], b["Wv"], b["Wo"]
    if dequantized:      # fp32 weights that bf16 cannot hold
        g = torch.Generator(device="cuda"); g.manual_seed(1)
        Wq, Wk, Wv, Wo = (w.float() * (1 + 0.05 * torch.randn(w.shape, generator=g, device="cuda")) for w in (Wq, Wk, Wv, Wo))
    Og = ctx.attention_forward(b["X"], Wq, Wk, Wv, 4, 2, 32)
    want = O.attention_output(f64(b["X"]), f64(Wq), f64(Wk), f64(Wv), 4, 2, 32)
    assert Og.dtype == torch.bfloat16
    # the result is stored in bf16: half an ulp of the value
    assert (np.abs(f64(Og) - want) <= 2.0 ** -8 * np.abs(want) + 1e-5 * np.abs(want).max()).all()
    Y = ctx.linear_forward(Og, Wo, residual=b["X"])
    wantY = f64(Og) @ f64(Wo).T + f64(b["X"])
    assert (np.abs(f64(Y) - wantY) <= 2.0 ** -8 * np.abs(wantY) + 1e-5 * np.abs(wantY).max()).all()


@pytest.mark.parametrize("name", ["tiny", "llama2-7b"])
def test_build_hout(ctx, name):
    cfg = synth.scaled(synth.CONFIGS[name], d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=32, n_seqs=2, seq_len=64, n_outlier=2)
    b = synth.make_block(cfg, seed=5, device="cuda")
    Hs = ctx.build_hessians(b["X"], None, b["Wq"], b["Wk"], b["Wv"], b["Wo"], 4, 2, 32)
    # from the weights of the block itself: the same matrices tboa_build_hessians returns
    hk = ctx.build_hout(Hs["Hin_qk"], b["Wq"], 2, 2, 32)
    hq = ctx.build_hout(Hs["Hin_qk"], b["Wk"], 2, 1, 32)
    assert np.allclose(f64(hk), f64(Hs["Hout_k"]), rtol=1e-5) and np.allclose(f64(hq), f64(Hs["Hout_q"][::2]), rtol=1e-5)
    # from other (dequantized, fp32) query weights: against the oracle's Table 1 sums with those weights
    Wq2 = (torch.round(b["Wq"].float() * 64) / 64 * 1.003)
    want = O.build_hessians(f64(b["X"]), None, f64(Wq2), f64(b["Wk"]), f64(b["Wv"]), f64(b["Wo"]), 4, 2, 32)["Hout_k"]
    got = f64(ctx.build_hout(Hs["Hin_qk"], Wq2, 2, 2, 32))
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


def test_tiny_config_hout_k_from_quantized_q(lib):
    """Tiny configuration with the Hessians of W_K formed after W_Q has been quantized (Algorithm 1 line 4 read as inside the
    loop): both sides follow the same order."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    cfg = synth.CONFIGS["tiny"]
    blk = synth.make_block(cfg, seed=0, device="cuda")
    ctx = lib.Context()
    got = quantize_attention_block(ctx, blk, cfg, hout_k_from_quantized_q=True)
    base = quantize_attention_block(ctx, blk, cfg, stack_qk=False)
    torch.cuda.synchronize()
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    X, Xf = f64(blk["X"]), f64(blk["X_fp"])
    W = {k: f64(blk[k]) for k in ("Wq", "Wk", "Wv", "Wo")}
    Hs = O.build_hessians(X, Xf, W["Wq"], W["Wk"], W["Wv"], W["Wo"], Hq, Hkv, dh, alpha=0.25)
    kw = dict(bits=cfg.bits, block=cfg.block)
    wq = O.quantize_layer(W["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq, **kw)
    Hk2 = O.build_hessians(X, Xf, wq["W_deq"], W["Wk"], W["Wv"], W["Wo"], Hq, Hkv, dh, alpha=0.25)["Hout_k"]
    wk = O.quantize_layer(W["Wk"], Hs["Hin_qk"], Hk2, Hs["R_qk"], Hkv, **kw)
    compare_layer(got["q"], wq, label="q")
    frac = compare_layer(got["k"], wk, label="k (H_out from the quantized W_Q)")
    changed = (got["k"]["codes"] != base["k"]["codes"]).float().mean().item()
    print("H_out of W_K from the quantized W_Q: codes identical to the oracle %.4f%%; %.2f%% of W_K's codes differ from the default reading"
          % (100 * frac, 100 * changed), flush=True)
    assert changed > 0 and torch.equal(got["q"]["codes"], base["q"]["codes"])
    ctx.close()


def oracle_chain(blocks, X, Xf, cfg, alpha=0.25):
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    kw = dict(bits=cfg.bits, group=cfg.group)
    outs = []
    for b in blocks:
        W = {k: f64(v) for k, v in b.items()}
        Hs = O.build_hessians(X, Xf, W["Wq"], W["Wk"], W["Wv"], W["Wo"], Hq, Hkv, dh, alpha=alpha)
        q = O.quantize_layer(W["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq, block=cfg.block, **kw)
        k = O.quantize_layer(W["Wk"], Hs["Hin_qk"], Hs["Hout_k"], Hs["R_qk"], Hkv, block=cfg.block, **kw)
        v = O.quantize_layer(W["Wv"], Hs["Hin_v"], Hs["Hout_v"], Hs["R_v"], Hkv, block=cfg.block, **kw)
        Hin_o, R_o = O.build_hessian_out_proj(X, Xf, q["W_deq"], k["W_deq"], v["W_deq"], W["Wq"], W["Wk"], W["Wv"], Hq, Hkv, dh, alpha=alpha)
        o = O.quantize_layer(W["Wo"], Hin_o, None, R_o, 1, block=cfg.d_model, **kw)
        Xa = X + O.attention_output(X, q["W_deq"], k["W_deq"], v["W_deq"], Hq, Hkv, dh) @ o["W_deq"].T
        Xaf = Xf + O.attention_output(Xf, W["Wq"], W["Wk"], W["Wv"], Hq, Hkv, dh) @ W["Wo"].T
        H, R = O.build_hessian_linear(Xa, Xaf, alpha)
        gate = O.quantize_layer(W["Wg"], H, None, R, 1, block=cfg.d_ff, **kw)
        up = O.quantize_layer(W["Wu"], H, None, R, 1, block=cfg.d_ff, **kw)
        act = O.swiglu(Xa, gate["W_deq"], up["W_deq"]); actf = O.swiglu(Xaf, W["Wg"], W["Wu"])
        Hd, Rd = O.build_hessian_linear(act, actf, alpha)
        down = O.quantize_layer(W["Wd"], Hd, None, Rd, 1, block=cfg.d_model, **kw)
        X = Xa + act @ down["W_deq"].T
        Xf = Xaf + actf @ W["Wd"].T
        outs.append(dict(qk=stacked(q, k), v=v, o=o, gate_up=stacked(gate, up, concat_heads=False), down=down, X=X, Xf=Xf))
    return outs


def test_two_tiny_blocks_in_a_row(lib):
    """Two tiny transformer blocks: block 2 sees the activations that block 1's quantized weights produce, and the deviation
    from the full-precision stream that has accumulated through block 1 (for block 1 the two streams are the calibration
    input itself and a perturbed copy).  Every layer of both blocks, and the activations handed on, against the oracle."""
    from paper_2602_04929_amd.pipeline import quantize_blocks
    cfg = synth.scaled(synth.CONFIGS["tiny"], d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=32, n_seqs=6, seq_len=96, n_outlier=2, d_ff=192)
    blocks = []
    for i in range(2):
        a = synth.make_block(cfg, seed=10 + i, device="cuda"); m = synth.make_mlp(cfg, seed=10 + i, device="cuda")
        blocks.append(dict(Wq=a["Wq"], Wk=a["Wk"], Wv=a["Wv"], Wo=a["Wo"], Wg=m["Wg"], Wu=m["Wu"], Wd=m["Wd"]))
        if i == 0:
            X, Xf = a["X"], a["X_fp"]
    ctx = lib.Context()
    res, Xo, Xfo = quantize_blocks(ctx, blocks, X, Xf, cfg)
    torch.cuda.synchronize()
    want = oracle_chain(blocks, f64(X), f64(Xf), cfg)
    for i, (r, w) in enumerate(zip(res, want)):
        for name, got in (("qk", r["attention"]["qk"]), ("v", r["attention"]["v"]), ("o", r["attention"]["o"]),
                          ("gate_up", r["mlp"]["gate_up"]), ("down", r["mlp"]["down"])):
            frac = compare_layer(got, w[name], label="block %d %s" % (i, name))
            print("block %d layer %s: codes identical %.4f%%" % (i, name, 100 * frac), flush=True)
        for got, ref, nm in ((r["X_out"], w["X"], "X"), (r["X_fp_out"], w["Xf"], "X_fp")):
            e = np.abs(f64(got) - ref).max() / np.abs(ref).max()
            print("block %d %s handed on: max rel err %.2e" % (i, nm, e), flush=True)
            assert e <= 1e-5
    dev0 = float((X.double() - Xf.double()).norm() / Xf.double().norm()); dev1 = float((res[0]["X_out"].double() - res[0]["X_fp_out"].double()).norm() / res[0]["X_fp_out"].double().norm())
    print("relative deviation of the two streams: %.3f entering block 1, %.3f entering block 2" % (dev0, dev1), flush=True)
    ctx.close()


@pytest.mark.parametrize("name,kv_bits", [("tiny", 4), ("tiny", 2), ("llama2-7b", 4)])
def test_hout_q_from_a_quantized_kv_cache(ctx, name, kv_bits):
    """tboa_build_hout_q_kv_cache against the oracle: H_out of W_Q from per-token fake-quantized keys (Sec. 4.2, KV cache).
    The levels are decided on fp64 keys by the oracle and on keys accumulated in fp32 (bf16 inputs) or fp64 (fp32 inputs) by
    the library, so single levels can differ at ties: the sums over all tokens agree to 1e-5 (fp32 inputs: 1e-6)."""
    cfg = synth.scaled(synth.CONFIGS[name], d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=32, n_seqs=3, seq_len=200, n_outlier=2)
    b = synth.make_block(cfg, seed=6, device="cuda")
    got = f64(ctx.build_hout_q_kv_cache(b["X"], b["Wk"], 4, 2, 32, kv_bits))
    want = O.hout_q_kv_cache(f64(b["X"]), f64(b["Wk"]), 4, 2, 32, kv_bits)
    plain = O.build_hessians(f64(b["X"]), None, f64(b["Wq"]), f64(b["Wk"]), f64(b["Wv"]), f64(b["Wo"]), 4, 2, 32)["Hout_q"]
    err = np.abs(got - want).max() / np.abs(want).max()
    print("H_out^Q from a %d-bit key cache (%s inputs): max |err| / max |entry| = %.2e" % (kv_bits, name, err), flush=True)
    assert got.shape == (4, 32, 32) and err <= (1e-6 if name == "tiny" else 1e-5)
    assert np.array_equal(got[0], got[1]) and np.array_equal(got[2], got[3]) and not np.array_equal(got[0], got[2])
    assert np.abs(want[0] - plain[0]).max() > 1e-3 * np.abs(want).max(), "the cache should matter at this width"


def test_tiny_block_with_kv_cache_end_to_end(ctx):
    """The tiny configuration with H_out of W_Q from a 4-bit key cache, end to end against the oracle."""
    from paper_2602_04929_amd.pipeline import quantize_attention_block
    cfg = synth.CONFIGS["tiny"]
    blk = synth.make_block(cfg, seed=0, device="cuda")
    got = quantize_attention_block(ctx, blk, cfg, use_R=True, stack_qk=False, kv_bits=4)
    torch.cuda.synchronize()
    X, Xf = f64(blk["X"]), f64(blk["X_fp"])
    W = {k: f64(blk[k]) for k in ("Wq", "Wk", "Wv", "Wo")}
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    Hs = O.build_hessians(X, Xf, W["Wq"], W["Wk"], W["Wv"], W["Wo"], Hq, Hkv, dh, alpha=0.25)
    Hs["Hout_q"] = O.hout_q_kv_cache(X, W["Wk"], Hq, Hkv, dh, 4)
    want = O.quantize_layer(W["Wq"], Hs["Hin_qk"], Hs["Hout_q"], Hs["R_qk"], Hq, bits=cfg.bits, block=cfg.block, group=cfg.group)
    frac = compare_layer(got["q"], want, label="W_Q with a 4-bit key cache")
    print("tiny, 4-bit key cache, W_Q: codes identical %.4f%%" % (100 * frac), flush=True)
