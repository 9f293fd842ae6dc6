"""Parity at the full size of the benchmark workload (Llama-2-7B-shaped block, 128 x 2048 tokens), in the launch
configuration bench.py times, on sampled outputs the oracle can compute one by one (GPU).

Hessians: sampled entries recomputed in fp64 from X.  quantize_layer: sampled heads (heads are independent) with the
oracle consuming the GPU-built, spot-checked Hessians."""
import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O
from paper_2602_04929_amd import synth
from tests.parity import check_returned_loss, compare_layer, head_of, rows_of

pytestmark = pytest.mark.gpu

CFG = synth.CONFIGS["llama2-7b"]
ALPHA = 0.25


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def full(lib):
    print("building the 7B-shaped block and its Hessians", flush=True)
    blk = synth.make_block(CFG, seed=0, device="cuda")
    ctx = lib.Context()
    Hs = ctx.build_hessians(blk["X"], blk["X_fp"], blk["Wq"], blk["Wk"], blk["Wv"], blk["Wo"], CFG.n_q_heads, CFG.n_kv_heads,
                            CFG.head_dim, alpha=ALPHA)
    torch.cuda.synchronize()
    yield dict(blk=blk, ctx=ctx, Hs=Hs)
    ctx.close()


def sampled_channels(d, seed, n=6):
    r = np.random.default_rng(seed)
    return np.sort(r.choice(d, n, replace=False))


def test_hessian_entries_qk(full):
    blk, Hs = full["blk"], full["Hs"]
    d, dh = CFG.d_model, CFG.head_dim
    ch = sampled_channels(d, 1, 8)
    X = blk["X"].reshape(-1, d); Xf = blk["X_fp"].reshape(-1, d)
    Xc = f64(X[:, ch]); dXc = Xc - f64(Xf[:, ch])
    want = Xc.T @ Xc
    got = f64(Hs["Hin_qk"][ch][:, ch])
    scale = np.sqrt(np.outer(np.diag(want), np.diag(want)))
    print("Hin_qk sampled rel err %.2e" % (np.abs(got - want) / scale).max(), flush=True)
    assert (np.abs(got - want) / scale).max() <= 1e-5          # exact bf16 products, fp32 accumulation in 16 chunks
    wantR = ALPHA * dXc.T @ Xc
    gotR = f64(Hs["R_qk"][ch][:, ch])
    scaleR = ALPHA * np.sqrt(np.outer(np.diag(dXc.T @ dXc), np.diag(want)))
    print("R_qk sampled rel err %.2e" % (np.abs(gotR - wantR) / scaleR).max(), flush=True)
    assert (np.abs(gotR - wantR) / scaleR).max() <= 1e-4
    # H_out of W_Q head 3 and W_K head 3: a few entries from explicit K, Q columns
    h, cols = 3, [0, 17, 127]
    Kc = np.zeros((X.shape[0], len(cols))); Qc = np.zeros_like(Kc)
    wk = f64(blk["Wk"][h * dh:(h + 1) * dh][cols]); wq = f64(blk["Wq"][h * dh:(h + 1) * dh][cols])
    for s in range(CFG.n_seqs):
        xs = f64(blk["X"][s]); sl = slice(s * CFG.seq_len, (s + 1) * CFG.seq_len)
        Kc[sl] = xs @ wk.T; Qc[sl] = xs @ wq.T
    for name, M, G in (("Hout_q", Hs["Hout_q"], Kc), ("Hout_k", Hs["Hout_k"], Qc)):
        want = G.T @ G; got = f64(M[h][cols][:, cols])
        e = (np.abs(got - want) / np.sqrt(np.outer(np.diag(want), np.diag(want)))).max()
        print(name, "sampled rel err %.2e" % e, flush=True)
        assert e <= 1e-5
    Wo_h = f64(blk["Wo"][:, h * dh:(h + 1) * dh])
    assert np.allclose(f64(Hs["Hout_v"][h]), Wo_h.T @ Wo_h, rtol=1e-6, atol=1e-9)


def test_hessian_entries_v(full):
    """H_in and R of W_V for one head on sampled channels: sum over all 128 sequences of (A_h X_s)^T (A_h X_s)."""
    blk, Hs = full["blk"], full["Hs"]
    d, dh, h = CFG.d_model, CFG.head_dim, 5
    ch = sampled_channels(d, 2, 6)
    wq = f64(blk["Wq"][h * dh:(h + 1) * dh]); wk = f64(blk["Wk"][h * dh:(h + 1) * dh])
    Hv = np.zeros((len(ch), len(ch))); Rv = np.zeros_like(Hv); dYY = np.zeros_like(Hv)
    for s in range(CFG.n_seqs):
        xs, xf = f64(blk["X"][s]), f64(blk["X_fp"][s])
        A, _, _ = O.attention_probs(xs, wq, wk)
        Af, _, _ = O.attention_probs(xf, wq, wk)
        Y = A @ xs[:, ch]; dY = Y - Af @ xf[:, ch]
        Hv += Y.T @ Y; Rv += ALPHA * dY.T @ Y; dYY += dY.T @ dY
        if s % 32 == 0:
            print("  oracle V-Hessian sample: sequence", s, flush=True)
    got = f64(Hs["Hin_v"][h][ch][:, ch]); gotR = f64(Hs["R_v"][h][ch][:, ch])
    e = (np.abs(got - Hv) / np.sqrt(np.outer(np.diag(Hv), np.diag(Hv)))).max()
    eR = (np.abs(gotR - Rv) / (ALPHA * np.sqrt(np.outer(np.diag(dYY), np.diag(Hv))))).max()
    print("Hin_v sampled rel err %.2e, R_v %.2e" % (e, eR), flush=True)
    # every intermediate of the W_V build is an exact-to-twice-the-mantissa (hi, lo) pair; X - X~ alone is a single half-precision value
    assert e <= 5e-6 and eR <= 3e-5


LAYERS = [("q", "Wq", "Hin_qk", "Hout_q", "R_qk", False), ("k", "Wk", "Hin_qk", "Hout_k", "R_qk", False),
          ("v", "Wv", "Hin_v", "Hout_v", "R_v", True)]


@pytest.mark.parametrize("layer", LAYERS, ids=[l[0] for l in LAYERS])
def test_quantize_layer_sampled_heads(full, layer):
    name, wkey, hin, hout, rkey, per_head = layer
    blk, Hs, ctx = full["blk"], full["Hs"], full["ctx"]
    dh, nh = CFG.head_dim, CFG.n_q_heads
    print("full-size quantize_layer", name, flush=True)
    got = ctx.quantize_layer(blk[wkey], Hs[hin], Hs[hout], Hs[rkey], nh, bits=CFG.bits, block=CFG.block)
    check_returned_loss(got, blk[wkey], Hs[hin], Hs[hout], Hs[rkey], nh, label=name)
    for h in (7, 30):
        rows = slice(h * dh, (h + 1) * dh)
        Hi = f64(Hs[hin][h:h + 1]) if per_head else f64(Hs[hin])
        Rr = f64(Hs[rkey][h:h + 1]) if per_head else f64(Hs[rkey])
        want = O.quantize_layer(f64(blk[wkey][rows]), Hi, f64(Hs[hout][h:h + 1]), Rr, 1, bits=CFG.bits, block=CFG.block)
        sub = head_of(got, h, dh)
        frac = compare_layer(sub, want, label="%s head %d" % (name, h))
        print("  %s head %d: codes identical %.4f%%, loss %.6g vs %.6g" % (name, h, 100 * frac, sub["loss"], want["loss"]), flush=True)
    full[name] = got
    print("  grid-search passes %d, fully exact passes %d, fully exact rows %d" % (ctx.counter(0), ctx.counter(1), ctx.counter(2)), flush=True)


def test_quantize_out_proj_sampled_rows(full):
    blk, ctx = full["blk"], full["ctx"]
    if not all(k in full for k in ("q", "k", "v")):
        pytest.skip("needs the three quantized projections of the previous tests")
    Hin_o, R_o = ctx.build_hessian_out_proj(blk["X"], blk["X_fp"], full["q"]["W_deq"], full["k"]["W_deq"], full["v"]["W_deq"],
                                            blk["Wq"], blk["Wk"], blk["Wv"], CFG.n_q_heads, CFG.n_kv_heads, CFG.head_dim, alpha=ALPHA)
    got = ctx.quantize_layer(blk["Wo"], Hin_o, None, R_o, 1, bits=CFG.bits, block=CFG.d_model)
    rows = np.sort(np.random.default_rng(3).choice(CFG.d_model, 48, replace=False))
    ridx = torch.tensor(rows, device="cuda")
    want = O.quantize_layer(f64(blk["Wo"][ridx]), f64(Hin_o), None, f64(R_o), 1, bits=CFG.bits, block=len(rows))
    sub = rows_of(got, ridx, f64(blk["Wo"][ridx]), O.damp_hessian(f64(Hin_o), 0.01), f64(R_o), O.layer_loss)
    check_returned_loss(got, blk["Wo"], Hin_o, None, R_o, 1, label="o")
    frac = compare_layer(sub, want, label="o rows")
    print("  W_O sampled rows: codes identical %.4f%%" % (100 * frac), flush=True)
    assert np.isfinite(got["loss"])


def test_quantize_layer_coupled_channels_full_width(lib):
    """d_in = 4096 with strongly coupled channels (X <- X (I + 0.3 low-rank), built here rather than through the attention
    block): the two-phase grid search over 16 tile columns where the cost is a small difference of large terms."""
    d, dh, nh, T = CFG.d_model, CFG.head_dim, 2, 16384
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    M = synth.correlated_mix(d, seed=3, device="cuda")
    X = torch.randn(T, d, generator=g, device="cuda") @ M
    dX = 0.05 * torch.randn(T, d, generator=g, device="cuda")
    Hin = (X.double().T @ X.double()).float()
    R = (0.25 * (dX.double().T @ X.double())).float()
    Gq = torch.randn(nh, T, dh, generator=g, device="cuda").double()
    Hout = (Gq.transpose(1, 2) @ Gq).float()
    W = (0.02 * torch.randn(nh * dh, d, generator=g, device="cuda")).to(torch.bfloat16)
    ctx = lib.Context()
    got = ctx.quantize_layer(W, Hin, Hout, R, nh, bits=CFG.bits, block=CFG.block)
    print("  passes %d, fully exact passes %d, fully exact rows %d" % (ctx.counter(0), ctx.counter(1), ctx.counter(2)), flush=True)
    want = O.quantize_layer(f64(W), f64(Hin), f64(Hout), f64(R), nh, bits=CFG.bits, block=CFG.block)
    frac = compare_layer(got, want, label="coupled full width")
    print("  coupled channels, d_in 4096: codes identical %.4f%%" % (100 * frac), flush=True)
    ctx.close()
