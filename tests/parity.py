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
    # dequantized weights: element by element, relative to the element itself, in the rows whose codes all agree (a flipped
    # code moves the refined scale of its row, so the other elements of that row follow it)
    wd = got["W_deq"].cpu().numpy().astype(np.float64)[same_rows]
    ref = want["W_deq"][same_rows]
    err = np.abs(wd - ref)
    assert np.all(err <= rtol * np.abs(ref)), "%s W_deq rel err %.3e" % (label, (err / (np.abs(ref) + 1e-300)).max())
    # every loss term against itself
    for k in ("loss_quad", "loss_cross", "loss"):
        ref_v = want[k]
        assert abs(got[k] - ref_v) <= rtol * abs(ref_v), "%s %s: %r vs %r" % (label, k, got[k], ref_v)
    lph = np.asarray(got["loss_per_head"])
    assert np.allclose(lph, want["loss_per_head"], rtol=rtol, atol=0), label + " loss_per_head"
    if "loss_per_head_terms" in got and "loss_per_head_terms" in want:
        assert np.allclose(np.asarray(got["loss_per_head_terms"]), want["loss_per_head_terms"], rtol=rtol, atol=0), label + " loss terms per head"
    return frac


def stacked(a, b, concat_heads=True):
    """Oracle results of two layers that share H_in and R as the result of the one stacked layer [W_a; W_b]: rows
    concatenated, loss terms summed; per-head losses concatenated (the layers' heads stay heads) or, for layers without
    out-channel coupling that are quantized as ONE head, summed."""
    out = {k: np.concatenate([a[k], b[k]], axis=0) for k in ("codes", "scales", "zeros", "W_deq")}
    out.update({k: a[k] + b[k] for k in ("loss_quad", "loss_cross", "loss")})
    for k in ("loss_per_head", "loss_per_head_terms"):
        la, lb = np.asarray(a[k]), np.asarray(b[k])
        out[k] = np.concatenate([la, lb]) if concat_heads else la + lb
    return out


def head_of(got, h, d_h):
    """The rows and the losses of head h of a quantize_layer result from the binding, as a result of its own."""
    rows = slice(h * d_h, (h + 1) * d_h)
    q, c = got["loss_per_head_terms"][h]
    return dict(codes=got["codes"][rows], scales=got["scales"][rows], zeros=got["zeros"][rows], W_deq=got["W_deq"][rows],
                loss_per_head=[got["loss_per_head"][h]], loss_per_head_terms=[(q, c)], loss=q + c, loss_quad=q, loss_cross=c)


def rows_of(got, ridx, W_rows, H_in, R, layer_loss):
    """Sampled rows of a layer without out-channel coupling (H_out = I: every row is a problem of its own), as a result of
    their own.  The library returns no per-row loss, so the two terms are evaluated (fp64, host) on the rows it returned:
    what is compared with the oracle is then the library's codes, scales and dequantized values, in the loss's own metric."""
    wd = got["W_deq"][ridx].double().cpu().numpy()
    q, c = layer_loss(W_rows, wd, H_in, None, R)
    return dict(codes=got["codes"][ridx], scales=got["scales"][ridx], zeros=got["zeros"][ridx], W_deq=got["W_deq"][ridx],
                loss=q + c, loss_quad=q, loss_cross=c, loss_per_head=[q + c])


def check_returned_loss(got, W, H_in, H_out, R, n_heads, damp=0.01, rtol=1e-6, label=""):
    """The losses a quantize_layer call returned against tr(H_out D H_in D^T) and 2 tr(H_out W R D^T) evaluated from the
    W_deq it returned (torch fp64 on the device: the test's own arithmetic, at any size), head by head."""
    import torch
    Wd = W.double(); D = got["W_deq"].double() - Wd
    d_h = W.shape[0] // n_heads
    def damped(H):
        H = H.double().clone()
        H.diagonal().add_(damp * H.diagonal().mean())
        return H
    Hi_shared = damped(H_in) if H_in.dim() == 2 else None
    for h in range(n_heads):
        rows = slice(h * d_h, (h + 1) * d_h)
        Hi = Hi_shared if Hi_shared is not None else damped(H_in[h])
        Ho = torch.eye(d_h, dtype=torch.float64, device=W.device) if H_out is None else damped(H_out[h])
        quad = float(torch.sum((Ho @ D[rows] @ Hi) * D[rows]))
        cross = 0.0
        if R is not None:
            Rh = (R if R.dim() == 2 else R[h]).double()
            cross = 2.0 * float(torch.sum((Ho @ Wd[rows] @ Rh) * D[rows]))
        gq, gc = got["loss_per_head_terms"][h]
        assert abs(gq - quad) <= rtol * abs(quad) and abs(gc - cross) <= rtol * max(abs(cross), 1e-300), \
            "%s head %d: returned (%r, %r), evaluated (%r, %r)" % (label, h, gq, gc, quad, cross)
    assert abs(got["loss_quad"] - sum(t[0] for t in got["loss_per_head_terms"])) <= 1e-9 * abs(got["loss_quad"])
