"""The gated MLP of the block: layer-wise Hessians, SwiGLU activation and the three quantized projections against the
oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O
from paper_2602_04929_amd import synth
from tests.parity import compare_layer, rows_of, stacked

pytestmark = pytest.mark.gpu


def f64(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context()
    yield c
    c.close()


def rel(got, want):
    return np.abs(got - want).max() / np.abs(want).max()


def test_linear_hessian_and_swiglu_fp32(ctx):
    cfg = synth.scaled(synth.CONFIGS["tiny"], d_model=72, n_seqs=3, seq_len=50, n_outlier=2, d_ff=100)
    m = synth.make_mlp(cfg, seed=1, device="cuda")
    H, R = ctx.build_hessian_linear(m["M"], m["M_fp"], 0.25)
    wH, wR = O.build_hessian_linear(f64(m["M"]), f64(m["M_fp"]), 0.25)
    assert rel(f64(H), wH) <= 1e-6 and rel(f64(R), wR) <= 1e-6
    H0, R0 = ctx.build_hessian_linear(m["M"])
    assert R0 is None and torch.equal(H0, H)
    act = ctx.swiglu_forward(m["M"], m["Wg"], m["Wu"])
    want = O.swiglu(f64(m["M"]), f64(m["Wg"]), f64(m["Wu"]))
    assert act.shape == (3, 50, 100) and rel(f64(act), want) <= 1e-6


@pytest.mark.parametrize("dequantized", [False, True, "grid"])
def test_linear_hessian_and_swiglu_bf16(ctx, dequantized):
    """bf16 path at sizes that span several 256-tiles with ragged edges (T = 960, d = 264, d_ff = 392)."""
    cfg = synth.scaled(synth.CONFIGS["llama2-7b"], d_model=264, n_seqs=3, seq_len=320, n_outlier=3, d_ff=392)
    m = synth.make_mlp(cfg, seed=2, device="cuda")
    H, R = ctx.build_hessian_linear(m["M"], m["M_fp"], 0.25)
    wH, wR = O.build_hessian_linear(f64(m["M"]), f64(m["M_fp"]), 0.25)
    print("H %.2e R %.2e" % (rel(f64(H), wH), rel(f64(R), wR)), flush=True)
    assert rel(f64(H), wH) <= 1e-5 and rel(f64(R), wR) <= 1e-4
    assert torch.equal(H, H.T)
    Wg, Wu = m["Wg"], m["Wu"]
    n_int, n_split = ctx.counter(4), ctx.counter(5)
    if dequantized == "grid":     # fp32 weights on a per-row uniform INT3 grid: taken as exact small integers times a step per row
        g = torch.Generator(device="cuda"); g.manual_seed(3)
        def on_grid(w):
            lo, hi = w.min(dim=1, keepdim=True).values.clamp(max=0), w.max(dim=1, keepdim=True).values.clamp(min=0)
            s = (hi - lo) / 7 * (0.7 + 0.3 * torch.rand(lo.shape, generator=g, device="cuda"))
            z = torch.round(-lo / s)
            return (s * (torch.clamp(torch.round(w / s) + z, 0, 7) - z)).float()
        Wg, Wu = on_grid(Wg.float()), on_grid(Wu.float())
    elif dequantized:      # fp32 weights that are not representable in bf16: the (hi, lo) split must carry them
        g = torch.Generator(device="cuda"); g.manual_seed(3)
        Wg = Wg.float() * (1 + 0.01 * torch.randn(Wg.shape, generator=g, device="cuda"))
        Wu = Wu.float() * (1 + 0.01 * torch.randn(Wu.shape, generator=g, device="cuda"))
    act = ctx.swiglu_forward(m["M"], Wg, Wu)
    assert (ctx.counter(4) - n_int, ctx.counter(5) - n_split) == {False: (0, 0), True: (0, 2), "grid": (2, 0)}[dequantized]
    want = O.swiglu(f64(m["M"]), f64(Wg), f64(Wu))
    err = np.abs(f64(act) - want)
    # the result is stored in bf16: half an ulp of the value, plus the fp32 arithmetic before it
    assert (err <= 2.0 ** -8 * np.abs(want) + 1e-6 * np.abs(want).max()).all()


@pytest.mark.parametrize("use_R,stack", [(True, True), (False, True), (True, False)])
def test_tiny_mlp_end_to_end(lib, use_R, stack):
    """Tiny configuration (d 256, d_ff 512, 8 x 128 tokens, INT2): gate, up and down projections against the oracle, each
    side computing its own Hessians and activations from the same inputs.  stack: gate and up (same H_in and R, rows
    decouple) through tboa_quantize_layer as one layer of 2 d_ff rows."""
    from paper_2602_04929_amd.pipeline import quantize_mlp
    cfg = synth.CONFIGS["tiny"]
    m = synth.make_mlp(cfg, seed=0, device="cuda")
    c = lib.Context()
    got = quantize_mlp(c, m, cfg, use_R=use_R, stack_gate_up=stack)
    M, Mf = f64(m["M"]), f64(m["M_fp"]) if use_R else None
    W = {k: f64(m[k]) for k in ("Wg", "Wu", "Wd")}
    kw = dict(bits=cfg.bits, group=cfg.group)
    H, R = O.build_hessian_linear(M, Mf, 0.25)
    want = {"gate": O.quantize_layer(W["Wg"], H, None, R, 1, block=cfg.d_ff, **kw),
            "up": O.quantize_layer(W["Wu"], H, None, R, 1, block=cfg.d_ff, **kw)}
    act = O.swiglu(M, want["gate"]["W_deq"], want["up"]["W_deq"])
    act_fp = O.swiglu(Mf, W["Wg"], W["Wu"]) if use_R else None
    Hd, Rd = O.build_hessian_linear(act, act_fp, 0.25)
    want["down"] = O.quantize_layer(W["Wd"], Hd, None, Rd, 1, block=cfg.d_model, **kw)
    if stack:
        want["gate_up"] = stacked(want["gate"], want["up"], concat_heads=False)
        assert torch.equal(got["gate"]["codes"], got["gate_up"]["codes"][:cfg.d_ff]) and torch.equal(got["up"]["W_deq"], got["gate_up"]["W_deq"][cfg.d_ff:])
    for layer in ("gate_up", "down") if stack else ("gate", "up", "down"):
        frac = compare_layer(got[layer], want[layer], label=layer)
        print("tiny MLP R=%s layer %s: codes identical %.4f%%" % (use_R, layer, 100 * frac), flush=True)
    c.close()


def test_llama2_7b_shape_mlp_sampled(lib):
    """Real widths (d 4096, d_ff 11008, bf16), 16 calibration sequences: sampled Hessian entries, sampled activations and
    sampled rows of the gate and down projections (rows decouple when H_out = I) against the oracle, which consumes the
    GPU-built, spot-checked Hessians."""
    from paper_2602_04929_amd.pipeline import quantize_mlp
    cfg = synth.scaled(synth.CONFIGS["llama2-7b"], n_seqs=16)
    d, dff = cfg.d_model, cfg.d_ff
    print("building the MLP inputs (16 sequences) and quantizing on the GPU", flush=True)
    m = synth.make_mlp(cfg, seed=0, device="cuda")
    c = lib.Context()
    got = quantize_mlp(c, m, cfg)
    r = np.random.default_rng(5)
    # Hessian of gate / up: sampled channels
    ch = np.sort(r.choice(d, 8, replace=False))
    Mc = f64(m["M"].reshape(-1, d)[:, ch]); dMc = Mc - f64(m["M_fp"].reshape(-1, d)[:, ch])
    want = Mc.T @ Mc
    e = (np.abs(f64(got["hessians"]["H_gate_up"][ch][:, ch]) - want) / np.sqrt(np.outer(np.diag(want), np.diag(want)))).max()
    eR = (np.abs(f64(got["hessians"]["R_gate_up"][ch][:, ch]) - 0.25 * dMc.T @ Mc) / (0.25 * np.sqrt(np.outer(np.diag(dMc.T @ dMc), np.diag(want))))).max()
    print("  H_gate_up sampled rel err %.2e, R %.2e" % (e, eR), flush=True)
    assert e <= 1e-5 and eR <= 1e-4
    # activations: sampled tokens x sampled hidden units, from the dequantized gate / up weights
    tok = torch.tensor(np.sort(r.choice(cfg.n_tokens, 32, replace=False)), device="cuda")
    hid = torch.tensor(np.sort(r.choice(dff, 64, replace=False)), device="cuda")
    want_a = O.swiglu(f64(m["M"].reshape(-1, d)[tok]), f64(got["gate"]["W_deq"][hid]), f64(got["up"]["W_deq"][hid]))
    got_a = f64(got["act"].reshape(-1, dff)[tok][:, hid])
    assert (np.abs(got_a - want_a) <= 2.0 ** -8 * np.abs(want_a) + 1e-6 * np.abs(want_a).max()).all()
    # Hessian of down: sampled hidden units, from the GPU's own activations
    hc = np.sort(r.choice(dff, 8, replace=False))
    Ac = f64(got["act"].reshape(-1, dff)[:, hc]); dAc = Ac - f64(got["act_fp"].reshape(-1, dff)[:, hc])
    want = Ac.T @ Ac
    e = (np.abs(f64(got["hessians"]["H_down"][hc][:, hc]) - want) / np.sqrt(np.outer(np.diag(want), np.diag(want)))).max()
    eR = (np.abs(f64(got["hessians"]["R_down"][hc][:, hc]) - 0.25 * dAc.T @ Ac) / (0.25 * np.sqrt(np.outer(np.diag(dAc.T @ dAc), np.diag(want))))).max()
    print("  H_down sampled rel err %.2e, R %.2e" % (e, eR), flush=True)
    assert e <= 1e-5 and eR <= 1e-4
    for layer, wkey, hk, rk, nrows in (("gate", "Wg", "H_gate_up", "R_gate_up", 48), ("down", "Wd", "H_down", "R_down", 16)):
        rows = np.sort(r.choice(m[wkey].shape[0], nrows, replace=False)); ridx = torch.tensor(rows, device="cuda")
        print("  oracle quantize_layer on %d sampled rows of %s" % (nrows, layer), flush=True)
        want = O.quantize_layer(f64(m[wkey][ridx]), f64(got["hessians"][hk]), None, f64(got["hessians"][rk]), 1, bits=cfg.bits, block=nrows)
        g = got[layer]
        sub = rows_of(g, ridx, f64(m[wkey][ridx]), O.damp_hessian(f64(got["hessians"][hk]), 0.01), f64(got["hessians"][rk]), O.layer_loss)
        frac = compare_layer(sub, want, label=layer + " rows")
        print("  %s sampled rows: codes identical %.4f%%" % (layer, 100 * frac), flush=True)
    c.close()


def test_mlp_entry_points_reject_bad_arguments(ctx, lib):
    X = torch.zeros(4, 10, 72, device="cuda")
    with pytest.raises(lib.TurboBoAError) as e:          # bf16 inputs need multiples of 8
        ctx.build_hessian_linear(torch.zeros(3, 9, 20, device="cuda", dtype=torch.bfloat16))
    assert e.value.code == -1
    with pytest.raises(lib.TurboBoAError) as e:          # weights neither fp32 nor of the activations' type
        ctx.swiglu_forward(X, torch.zeros(16, 72, device="cuda", dtype=torch.bfloat16), torch.zeros(16, 72, device="cuda", dtype=torch.bfloat16))
    assert e.value.code == -1
    H, R = ctx.build_hessian_linear(X)                     # all-zero activations: a zero Hessian, and quantize_layer reports it
    assert R is None and float(H.abs().max()) == 0.0
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.quantize_layer(torch.ones(8, 72, device="cuda"), H, None, None, 1, bits=2, block=8)
    assert e.value.code == -2
