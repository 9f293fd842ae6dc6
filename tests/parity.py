"""Shared comparison of a HIP quantize_layer result with the oracle's (spec tolerances)."""
import numpy as np


def compare_layer(got, want, min_code_match=0.999, rtol=1e-4, label=""):
    """got: dict of torch tensors / floats from the binding; want: dict from the oracle."""
    codes = got["codes"].cpu().numpy()
    match = (codes == want["codes"])
    frac = match.mean()
    assert frac >= min_code_match, "%s codes identical: %.5f%%" % (label, 100 * frac)
    # rows whose codes all agree took the same (scale, zero) decisions up to rounding
    same_rows = match.all(axis=1)
    s_got = got["scales"].cpu().numpy().astype(np.float64); z_got = got["zeros"].cpu().numpy().astype(np.float64)
    assert np.allclose(s_got[same_rows], want["scales"][same_rows], rtol=rtol, atol=0), label + " scales"
    assert np.array_equal(z_got[same_rows], want["zeros"][same_rows]), label + " zeros"
    # dequantized weights: element-wise where the codes agree (scale / zero parity)
    wd = got["W_deq"].cpu().numpy().astype(np.float64)
    ref = want["W_deq"]
    scale_el = np.abs(ref).max(axis=1, keepdims=True) + 1e-300
    err = np.abs(wd - ref) / scale_el
    assert err[match].max() <= rtol, "%s W_deq rel err %.3e" % (label, err[match].max())
    for k in ("loss_quad", "loss_cross", "loss"):
        ref_v = want[k]; tol = rtol * max(abs(want["loss_quad"]), abs(ref_v))
        assert abs(got[k] - ref_v) <= tol, "%s %s: %r vs %r" % (label, k, got[k], ref_v)
    lph = np.asarray(got["loss_per_head"])
    assert np.allclose(lph, want["loss_per_head"], rtol=10 * rtol, atol=rtol * abs(want["loss"])), label + " loss_per_head"
    return frac


def stacked(a, b, concat_heads=True):
    """Oracle results of two layers that share H_in and R as the result of the one stacked layer [W_a; W_b]: rows
    concatenated, loss terms summed; loss_per_head concatenated (the layers' heads stay heads) or, for layers without
    out-channel coupling that are quantized as ONE head, summed."""
    out = {k: np.concatenate([a[k], b[k]], axis=0) for k in ("codes", "scales", "zeros", "W_deq")}
    out.update({k: a[k] + b[k] for k in ("loss_quad", "loss_cross", "loss")})
    la, lb = np.asarray(a["loss_per_head"]), np.asarray(b["loss_per_head"])
    out["loss_per_head"] = np.concatenate([la, lb]) if concat_heads else la + lb
    return out
