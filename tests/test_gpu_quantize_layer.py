"""tboa_quantize_layer against the fp64 oracle on the same seeded inputs (GPU)."""
import zlib

import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O
from tests.parity import compare_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context()
    yield c
    c.close()


def make_case(seed, n_heads, dh, n, T, per_head_in=False, corr=0.5, mix=0.0):
    r = np.random.default_rng(seed)
    M = np.eye(n) + mix * (r.standard_normal((n, 8)) @ r.standard_normal((8, n))) / np.sqrt(8.0) if mix else None
    def acts():
        X = r.standard_normal((T, n)) + corr * r.standard_normal((T, 1))
        X[:, r.integers(0, n, 3)] *= 10
        return X @ M if mix else X
    W = (r.standard_normal((n_heads * dh, n)) * 0.02).astype(np.float32)
    if per_head_in:
        Xs = [acts() for _ in range(n_heads)]
        Hin = np.stack([x.T @ x for x in Xs]).astype(np.float32)
        R = np.stack([0.25 * (0.1 * r.standard_normal((T, n))).T @ x for x in Xs]).astype(np.float32)
    else:
        X = acts()
        Hin = (X.T @ X).astype(np.float32)
        R = (0.25 * (0.1 * r.standard_normal((T, n))).T @ X).astype(np.float32)
    G = [r.standard_normal((T, dh)) + 0.7 * r.standard_normal((T, 1)) for _ in range(n_heads)]
    Hout = np.stack([g.T @ g for g in G]).astype(np.float32)
    return W, Hin, Hout, R


def run_both(ctx, W, Hin, Hout, R, n_heads, **kw):
    dev = lambda a: None if a is None else torch.tensor(a, device="cuda")
    got = ctx.quantize_layer(dev(W), dev(Hin), dev(Hout), dev(R), n_heads, **kw)
    f64 = lambda a: None if a is None else a.astype(np.float64)
    want = O.quantize_layer(f64(W), f64(Hin), f64(Hout), f64(R), n_heads, **kw)
    return got, want


CASES = [
    # name, n_heads, dh, n, per_head_in, use_Hout, use_R, kwargs
    ("q-like", 3, 40, 200, False, True, True, dict(bits=2, block=16)),
    ("q-like-noR", 2, 64, 256, False, True, False, dict(bits=2, block=4)),
    ("v-like", 3, 32, 136, True, True, True, dict(bits=2, block=8)),
    ("o-like", 1, 96, 192, False, False, True, dict(bits=2, block=96)),
    ("boa", 2, 24, 128, False, True, False, dict(bits=2, block=1, adaptive_grid=False, cd_iters=0)),
    ("int3", 2, 32, 160, False, True, True, dict(bits=3, block=32)),
    ("int4-cd2", 2, 32, 130, False, True, True, dict(bits=4, block=12, cd_iters=2)),
    ("nodamp", 2, 16, 96, False, True, True, dict(bits=2, block=8, damp=0.0)),
    # group-wise grids: (scale, zero) per (row, group), found when the sweep enters the group; refinement per (row, group)
    ("group-sweep-only", 2, 32, 256, False, True, True, dict(bits=3, block=8, group=64, cd_iters=0)),
    ("group-q", 2, 32, 256, False, True, True, dict(bits=3, block=8, group=64)),
    ("group-q-noR-cd2", 3, 24, 192, False, True, False, dict(bits=3, block=24, group=64, cd_iters=2)),
    ("group-v", 2, 16, 128, True, True, True, dict(bits=3, block=8, group=64)),
    ("group-o", 1, 48, 256, False, False, True, dict(bits=3, block=48, group=128, cd_iters=2)),
    ("group-32", 2, 16, 96, False, True, True, dict(bits=4, block=4, group=32)),
    ("group-fixed-grid", 2, 16, 128, False, True, False, dict(bits=3, block=4, group=64, adaptive_grid=False)),
    # the two-phase grid search (d_in >= 256) over two tile columns, with strongly coupled input channels (X <- X (I + 0.3
    # low-rank)): the cost delta H delta^T is then a small difference of large terms
    ("coupled-q-512", 2, 32, 512, False, True, True, dict(bits=2, block=16)),
    ("coupled-v-512", 2, 16, 512, True, True, True, dict(bits=2, block=8)),
    ("coupled-o-384-int4", 1, 64, 384, False, False, True, dict(bits=4, block=64)),
    # d_in not a multiple of 32: row-major operands, the register-staged GEMM kernel with the causal limit per segment
    ("coupled-q-264", 2, 16, 264, False, True, True, dict(bits=2, block=8)),
    ("coupled-v-328", 2, 16, 328, True, True, True, dict(bits=3, block=16)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_quantize_layer_matches_oracle(ctx, case):
    name, nh, dh, n, ph, use_ho, use_r, kw = case
    print("quantize_layer case", name, flush=True)
    W, Hin, Hout, R = make_case(zlib.crc32(name.encode()) % 1000, nh, dh, n, T=4 * n, per_head_in=ph,
                                mix=0.3 if name.startswith("coupled") else 0.0)
    fallbacks = ctx.counter(1)
    got, want = run_both(ctx, W, Hin, Hout if use_ho else None, R if use_r else None, nh, **kw)
    # a pass of the two-phase grid search that distrusts its approximate costs repeats itself exactly: that must not be
    # what makes these cases agree
    assert ctx.counter(1) == fallbacks, "a grid-search pass fell back to exact costs"
    frac = compare_layer(got, want, label=name)
    print("codes identical: %.4f%%" % (100 * frac), flush=True)
    codes = got["codes"].cpu().numpy()
    assert codes.max() <= 2 ** kw["bits"] - 1
    gsz = kw.get("group", 0) or n
    s = np.repeat(got["scales"].cpu().numpy(), gsz, axis=1); z = np.repeat(got["zeros"].cpu().numpy(), gsz, axis=1)
    assert np.allclose(got["W_deq"].cpu().numpy(), s * (codes.astype(np.float32) - z), rtol=1e-6)


def test_bf16_weights_and_determinism(ctx):
    W, Hin, Hout, R = make_case(7, 2, 32, 128, T=512)
    Wb = torch.tensor(W, device="cuda").to(torch.bfloat16)
    args = (torch.tensor(Hin, device="cuda"), torch.tensor(Hout, device="cuda"), torch.tensor(R, device="cuda"), 2)
    a = ctx.quantize_layer(Wb, *args, bits=2, block=8)
    b = ctx.quantize_layer(Wb, *args, bits=2, block=8)
    assert torch.equal(a["codes"], b["codes"]) and torch.equal(a["scales"], b["scales"]) and a["loss"] == b["loss"]
    want = O.quantize_layer(Wb.float().cpu().numpy().astype(np.float64), Hin.astype(np.float64), Hout.astype(np.float64),
                            R.astype(np.float64), 2, bits=2, block=8)
    compare_layer(a, want, label="bf16")


def test_error_paths(ctx, lib):
    W, Hin, Hout, R = make_case(8, 2, 16, 64, T=256)
    t = lambda a: torch.tensor(a, device="cuda")
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.quantize_layer(t(W), t(Hin), t(Hout), None, 2, bits=5, block=4)
    assert e.value.code == -1
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.quantize_layer(t(W), t(Hin), t(Hout), None, 2, bits=2, block=4, group=48)
    assert e.value.code == -1
    Hbad = Hin.copy(); Hbad[:, 5] = 0; Hbad[5, :] = 0      # a dead input channel, no damping: not SPD
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.quantize_layer(t(W), t(Hbad), t(Hout), None, 2, bits=2, block=4, damp=0.0)
    assert e.value.code == -2
    ok = ctx.quantize_layer(t(W), t(Hbad), t(Hout), None, 2, bits=2, block=4, damp=0.01)   # damping repairs it
    assert np.isfinite(ok["loss"])
    Hobad = Hout.copy(); Hobad[1, 3, :] = 0; Hobad[1, :, 3] = 0     # the same for H_out of head 1 (its own status words)
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.quantize_layer(t(W), t(Hin), t(Hobad), None, 2, bits=2, block=4, damp=0.0)
    assert e.value.code == -2 and "Hessian 1" in str(e.value)
    ok = ctx.quantize_layer(t(W), t(Hin), t(Hout), None, 2, bits=2, block=4)                # the context is usable afterwards
    assert np.isfinite(ok["loss"])


@pytest.mark.parametrize("bits,group", [(2, 0), (3, 0), (3, 64), (4, 32), (8, 0)])
def test_packed_codes_and_dequant_gemv(ctx, bits, group):
    """Packing is bit-exact against the oracle's bit stream (ragged row lengths); the packed form reproduces W_deq x."""
    r = np.random.default_rng(100 + bits)
    for d_out, d_in in ((37, 200), (64, 136), (5, 4096)):
        if group and d_in % group:
            continue
        codes = r.integers(0, 2 ** bits, size=(d_out, d_in)).astype(np.uint8)
        packed = ctx.pack_codes(torch.tensor(codes, device="cuda"), bits)
        want = O.pack_codes(codes, bits)
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), want), (bits, d_out, d_in)
        ng = d_in // group if group else 1
        scales = (r.random((d_out, ng)) * 0.01 + 0.001).astype(np.float32); zeros = r.integers(0, 2 ** bits, size=(d_out, ng)).astype(np.float32)
        x = r.standard_normal(d_in).astype(np.float32)
        y = ctx.dequant_gemv(packed, torch.tensor(scales, device="cuda"), torch.tensor(zeros, device="cuda"), torch.tensor(x, device="cuda"),
                             d_in, bits, group)
        ref = O.dequant_matvec(codes, scales, zeros, x, group)
        assert np.allclose(y.cpu().numpy(), ref, rtol=1e-6, atol=1e-6 * np.abs(ref).max())


def test_packed_layer_carries_the_quantized_weights(ctx):
    """quantize_layer -> pack -> GEMV from the packed form equals W_deq x."""
    W, Hin, Hout, R = make_case(11, 2, 32, 256, T=1024)
    t = lambda a: torch.tensor(a, device="cuda")
    got = ctx.quantize_layer(t(W), t(Hin), t(Hout), t(R), 2, bits=3, block=8, group=64)
    packed = ctx.pack_codes(got["codes"], 3)
    x = torch.randn(256, device="cuda")
    y = ctx.dequant_gemv(packed, got["scales"], got["zeros"], x, 256, 3, 64)
    ref = got["W_deq"].double() @ x.double()
    assert torch.allclose(y.double(), ref, rtol=1e-5, atol=1e-6 * ref.abs().max().item())


def test_grid_search_guard_takes_the_exact_path(ctx):
    """The two-phase search compares every exact re-evaluation with its approximation, and a call in which one strays by
    more than grid_guard * tau is run again with exact costs for every candidate.  With a vanishing grid_guard every call
    that re-evaluated anything takes that path; the result must be the oracle's all the same, and equal to what asking for
    exact costs from the start (negative grid_guard) gives."""
    W, Hin, Hout, R = make_case(77, 2, 32, 256, T=1024, mix=0.3)
    dev = lambda a: torch.tensor(a, device="cuda")
    before, passes = ctx.counter(1), ctx.counter(0)
    got = ctx.quantize_layer(dev(W), dev(Hin), dev(Hout), dev(R), 2, bits=2, block=16, grid_guard=1e-300)
    assert ctx.counter(1) == before + 1, "the call was not run again with exact costs"
    assert ctx.counter(0) > passes
    want = O.quantize_layer(W.astype(np.float64), Hin.astype(np.float64), Hout.astype(np.float64), R.astype(np.float64), 2, bits=2, block=16)
    frac = compare_layer(got, want, label="guard")
    print("guarded call: codes identical %.4f%%" % (100 * frac), flush=True)
    passes = ctx.counter(0)
    exact = ctx.quantize_layer(dev(W), dev(Hin), dev(Hout), dev(R), 2, bits=2, block=16, grid_guard=-1.0)
    assert ctx.counter(0) == passes and ctx.counter(1) == before + 1          # no two-phase pass at all
    assert torch.equal(exact["codes"], got["codes"]) and torch.equal(exact["scales"], got["scales"])


def test_workspace_queries(ctx, lib):
    """tboa_quantize_workspace_bytes bounds what a call takes; a context that reserved it does not grow."""
    W, Hin, Hout, R = make_case(5, 2, 32, 256, T=1024)
    t = lambda a: torch.tensor(a, device="cuda")
    c2 = lib.Context()
    try:
        desc = c2.layer_desc(t(W), t(Hin), 2, bits=2, block=8)
        need = c2.quantize_workspace_bytes(desc)
        assert need > 0 and c2.workspace_bytes() == 0
        c2.reserve_workspace(need)
        assert c2.workspace_bytes() == need
        a = c2.quantize_layer(t(W), t(Hin), t(Hout), t(R), 2, bits=2, block=8)
        assert c2.workspace_bytes() == need                      # with H_out and R: exactly the bound
        c2.quantize_layer(t(W), t(Hin), None, None, 2, bits=2, block=8)
        assert c2.workspace_bytes() == need                      # without them: less
        assert 0 < c2.quantize_workspace_bytes(desc, with_H_out=False, with_R=False) <= need
        b = ctx.quantize_layer(t(W), t(Hin), t(Hout), t(R), 2, bits=2, block=8)
        assert torch.equal(a["codes"], b["codes"]) and a["loss"] == b["loss"]
        bad = c2.layer_desc(t(W), t(Hin), 2, bits=5, block=8)
        assert c2.quantize_workspace_bytes(bad) == 0
    finally:
        c2.close()
