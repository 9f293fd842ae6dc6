"""fp64 CPU oracle for the TurboBoA quantization path.  TEST INFRASTRUCTURE ONLY.

This file is a plain, slow, step-by-step restatement of what the paper's method
computes for one attention block, in numpy float64.  It shares no code with the
HIP library and must never be imported by the product path: only tests, the
smoke check and the CPU-baseline leg of the benchmark may call it.

Notation follows the paper.  Activations are stored token-major, ``Xr[t, :]`` is
one token (the paper's ``X`` is ``Xr.T``), so ``H_in = X X^T = Xr^T Xr``.
The paper's N (out-channels quantized jointly) is ``block`` here.

Pins (see tests/test_oracle_pins.py): trace/Kronecker identities for the Hessians,
textbook properties of U = Chol(H^-1)^T, brute-force constrained least squares
for Prop. 3.1 and Prop. 3.2, an independently written row-at-a-time BoA for
block=1, textbook OBS elimination for the in-channel sweep with R = 0, every step
of the sweep with R != 0 as the least-squares problem it solves (explicit X and
X - X~, no factor of H), Algorithm 1 with R != 0 and per-head Hessians rebuilt from
those pieces, the explicit quadratic in s for Prop. 3.3, exhaustive evaluation for
the grid search, hand-computed rows for the activation quantizer, a hand-computed
Gram matrix for the keys of a quantized cache.

parity unpinned:
  * the candidate list of the grid search (ranges, number and spacing of the
    candidates) is a reading of ours, the paper gives only the objective; the search
    over that list is checked against an exhaustive loop.
The group-wise (row, group) extension is ours as well; it is checked against the
per-row algorithm it extends (Hessians that couple no two groups) and against a
step-wise least-squares sweep with exhaustive grids at group entry.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Table 1: attention-aware Kronecker-factored Hessians
# --------------------------------------------------------------------------

def softmax_rows(S):
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=-1, keepdims=True)


def attention_probs(Xs, Wq_h, Wk_g, causal=True):
    """A_h for one sequence: softmax_rows(Q_h K_g^T / sqrt(d_h) + mask)  (Table 1, W_V row).

    Xs [L, d]; Wq_h, Wk_g [d_h, d].  Returns A [L, L], Q_h [L, d_h], K_g [L, d_h]."""
    Q = Xs @ Wq_h.T
    K = Xs @ Wk_g.T
    S = (Q @ K.T) / np.sqrt(F64(Wq_h.shape[0]))
    if causal:
        L = S.shape[0]
        S = np.where(np.tril(np.ones((L, L), dtype=bool)), S, -np.inf)
    return softmax_rows(S), Q, K


def build_hessians(X, X_fp, Wq, Wk, Wv, Wo, n_q_heads, n_kv_heads, head_dim,
                   alpha=0.0, causal=True):
    """Hessian factors of Table 1 for W_Q,h / W_K,g / W_V,g, plus R = alpha*dX X^T
    (Algorithm 1, line 5).  Literal sums over all tokens of all sequences.

    X, X_fp: [S, L, d] (X_fp may be None -> every R is None).
    Wq [Hq*dh, d], Wk, Wv [Hkv*dh, d], Wo [d, Hq*dh].
    GQA reading: query head h uses KV group g = h // (Hq/Hkv); the K and V layers sum
    their Hessian factors over the query heads of the group.
    """
    X = np.asarray(X, F64)
    S_, L, d = X.shape
    Hq, Hkv, dh = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    Wq = np.asarray(Wq, F64); Wk = np.asarray(Wk, F64)
    Wv = np.asarray(Wv, F64); Wo = np.asarray(Wo, F64)
    have_fp = X_fp is not None
    if have_fp:
        X_fp = np.asarray(X_fp, F64)

    Hin_qk = np.zeros((d, d), F64)
    R_qk = np.zeros((d, d), F64) if have_fp else None
    Hout_q = np.zeros((Hq, dh, dh), F64)
    Hout_k = np.zeros((Hkv, dh, dh), F64)
    Hin_v = np.zeros((Hkv, d, d), F64)
    R_v = np.zeros((Hkv, d, d), F64) if have_fp else None
    Hout_v = np.zeros((Hkv, dh, dh), F64)

    for s in range(S_):
        Xs = X[s]
        Hin_qk += Xs.T @ Xs
        if have_fp:
            R_qk += alpha * (Xs - X_fp[s]).T @ Xs          # R = dX X^T: rows index dX
        for h in range(Hq):
            g = h // rep
            A, Q, K = attention_probs(Xs, Wq[h*dh:(h+1)*dh], Wk[g*dh:(g+1)*dh], causal)
            Hout_q[h] += K.T @ K                           # G = K_h for W_Q,h
            Hout_k[g] += Q.T @ Q                           # G = Q_h for W_K,h
            Y = A @ Xs                                     # effective input of W_V,h is X A_h^T
            Hin_v[g] += Y.T @ Y
            if have_fp:
                A_fp, _, _ = attention_probs(X_fp[s], Wq[h*dh:(h+1)*dh], Wk[g*dh:(g+1)*dh], causal)
                Y_fp = A_fp @ X_fp[s]
                R_v[g] += alpha * (Y - Y_fp).T @ Y
    for h in range(Hq):
        Wout_h = Wo[:, h*dh:(h+1)*dh]                       # d x d_h
        Hout_v[h // rep] += Wout_h.T @ Wout_h
    return dict(Hin_qk=Hin_qk, R_qk=R_qk, Hout_q=Hout_q, Hout_k=Hout_k,
                Hin_v=Hin_v, R_v=R_v, Hout_v=Hout_v)


def attention_output(X, Wq, Wk, Wv, n_q_heads, n_kv_heads, head_dim, causal=True):
    """Input of the output projection: concat_h(A_h V_g(h)) per sequence.  [S, L, Hq*dh]."""
    X = np.asarray(X, F64)
    S_, L, d = X.shape
    Hq, Hkv, dh = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    O = np.zeros((S_, L, Hq * dh), F64)
    for s in range(S_):
        for h in range(Hq):
            g = h // rep
            A, _, _ = attention_probs(X[s], np.asarray(Wq, F64)[h*dh:(h+1)*dh],
                                      np.asarray(Wk, F64)[g*dh:(g+1)*dh], causal)
            V = X[s] @ np.asarray(Wv, F64)[g*dh:(g+1)*dh].T
            O[s, :, h*dh:(h+1)*dh] = A @ V
    return O


def build_hessian_out_proj(X, X_fp, Wq_deq, Wk_deq, Wv_deq, Wq, Wk, Wv,
                           n_q_heads, n_kv_heads, head_dim, alpha=0.0, causal=True):
    """Layer-wise Hessian X_o X_o^T (GPTQ row of Table 1) for the output projection, with
    X_o computed from the dequantized Q/K/V weights on X; R_o = alpha (X_o - X~_o) X_o^T with
    X~_o from the FP weights on X_fp."""
    O = attention_output(X, Wq_deq, Wk_deq, Wv_deq, n_q_heads, n_kv_heads, head_dim, causal)
    O2 = O.reshape(-1, O.shape[-1])
    Hin_o = O2.T @ O2
    R_o = None
    if X_fp is not None:
        Of = attention_output(X_fp, Wq, Wk, Wv, n_q_heads, n_kv_heads, head_dim, causal)
        R_o = alpha * (O2 - Of.reshape(O2.shape)).T @ O2
    return Hin_o, R_o


def build_hessian_linear(X, X_fp=None, alpha=0.0):
    """Layer-wise row of Table 1 for a plain linear layer (the MLP projections): H_in = sum_t x_t x_t^T and, with the
    full-precision input given, R = alpha sum_t (x_t - x~_t) x_t^T (Algorithm 1, line 5).  X [.., d_in]."""
    X2 = np.asarray(X, F64).reshape(-1, np.shape(X)[-1])
    H = X2.T @ X2
    if X_fp is None:
        return H, None
    Xf2 = np.asarray(X_fp, F64).reshape(X2.shape)
    return H, alpha * (X2 - Xf2).T @ X2


def swiglu(X, Wg, Wu):
    """Input of the down projection of a gated MLP: silu(X Wg^T) * (X Wu^T), silu(g) = g / (1 + exp(-g))."""
    G = np.asarray(X, F64) @ np.asarray(Wg, F64).T
    U = np.asarray(X, F64) @ np.asarray(Wu, F64).T
    return G / (1.0 + np.exp(-G)) * U


def act_fakequant_per_token(X, bits):
    """Min-Max dynamic per-token activation quantizer (asymmetric), returned dequantized.
    One (scale, zero) per token from that token's own min and max."""
    X = np.asarray(X, F64)
    maxq = F64(2 ** bits - 1)
    lo = np.minimum(X.min(axis=-1, keepdims=True), 0.0)
    hi = np.maximum(X.max(axis=-1, keepdims=True), 0.0)
    same = (lo == hi)
    lo = np.where(same, -1.0, lo); hi = np.where(same, 1.0, hi)
    s = (hi - lo) / maxq
    z = np.rint(-lo / s)
    q = np.clip(np.rint(X / s) + z, 0.0, maxq)
    return s * (q - z)


def hout_q_kv_cache(X, Wk, n_q_heads, n_kv_heads, head_dim, kv_bits):
    """H_out of W_Q,h when the keys are held in a kv_bits-bit cache (the KV4 setting of Sec. 4.2):
    G = K^_g in the W_Q row of Table 1, K^_g the per-token Min-Max fake-quant of the head vectors
    k_{g,t} = W_K,g x_t (one scale and zero per token and KV head), g = h // (Hq/Hkv).
    Returns [Hq, dh, dh] = K^_g^T K^_g summed over all tokens."""
    X = np.asarray(X, F64); Wk = np.asarray(Wk, F64)
    X2 = X.reshape(-1, X.shape[-1])
    Hq, Hkv, dh = n_q_heads, n_kv_heads, head_dim
    rep = Hq // Hkv
    out = np.zeros((Hq, dh, dh), F64)
    for g in range(Hkv):
        K = X2 @ Wk[g*dh:(g+1)*dh].T                      # [T, dh]
        Kq = act_fakequant_per_token(K, kv_bits)
        G = Kq.T @ Kq
        for r in range(rep):
            out[g * rep + r] = G
    return out


def hadamard_matrix(d):
    """Sylvester-Hadamard matrix of order d = 2^k: H_1 = [1], H_2n = [[H_n, H_n], [H_n, -H_n]]."""
    H = np.ones((1, 1), F64)
    while H.shape[0] < d:
        H = np.block([[H, H], [H, -H]])
    assert H.shape[0] == d, "d must be a power of two"
    return H


def hadamard_rotate(X, signs=None):
    """Randomised Hadamard rotation of activation rows (the fixed transform of App. B used in the weight-activation
    setting): (X * signs) H_d / sqrt(d).  X [..., d], signs [d] of +-1 or None."""
    X = np.asarray(X, F64)
    d = X.shape[-1]
    if signs is not None:
        X = X * np.asarray(signs, F64)
    return X @ hadamard_matrix(d) / np.sqrt(F64(d))


# --------------------------------------------------------------------------
# eq. 3: U = Chol(H^-1)^T
# --------------------------------------------------------------------------

def damp_hessian(H, damp):
    """H + damp * mean(diag H) * I  (no damping in the paper; damp = 0 recovers it)."""
    H = np.array(H, F64, copy=True)
    if damp:
        H[np.diag_indices_from(H)] += F64(damp) * np.mean(np.diag(H))
    return H


def chol_inv_upper(H):
    """U upper triangular with H^-1 = U^T U (eq. 3): invert, then factor."""
    Hinv = np.linalg.inv(np.asarray(H, F64))
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv).T


# --------------------------------------------------------------------------
# quantization grid
# --------------------------------------------------------------------------

def quantize_codes(w, s, z, maxq):
    """q = clamp(round_half_even(w / s) + z, 0, 2^b - 1)  (Algorithm 3, quantize step,
    with an integer zero-point added so the grid can be asymmetric)."""
    return np.clip(np.rint(w / s) + z, 0.0, maxq)


def grid_search(Wrows, H, bits, grid_points=100, max_shrink=0.8):
    """Algorithm 1 line 9: per row, (s, z) minimising delta H delta^T over a list of shrunken
    min-max grids.  Wrows [r, n], H [n, n].  Returns s [r], z [r].

    Candidate k = 0 .. ceil(max_shrink*grid_points)-1 uses p = 1 - k/grid_points,
    s = (p*hi - p*lo)/(2^b-1), z = round(-p*lo/s); the lowest k among equal minima wins."""
    Wrows = np.asarray(Wrows, F64)
    r, n = Wrows.shape
    if r > 64:                                   # rows are independent: bound the temporaries
        parts = [grid_search(Wrows[i:i + 64], H, bits, grid_points, max_shrink) for i in range(0, r, 64)]
        return np.concatenate([a for a, _ in parts]), np.concatenate([b for _, b in parts])
    maxq = F64(2 ** bits - 1)
    n_cand = int(np.ceil(max_shrink * grid_points))
    lo = np.minimum(Wrows.min(axis=1), 0.0)
    hi = np.maximum(Wrows.max(axis=1), 0.0)
    flat = (lo == hi)
    lo = np.where(flat, -1.0, lo); hi = np.where(flat, 1.0, hi)
    p = 1.0 - np.arange(n_cand, dtype=F64) / F64(grid_points)            # [c]
    s = (p[None, :] * hi[:, None] - p[None, :] * lo[:, None]) / maxq       # [r, c]
    z = np.rint(-(p[None, :] * lo[:, None]) / s)                           # [r, c]
    w = Wrows[:, None, :]
    delta = s[:, :, None] * (quantize_codes(w, s[:, :, None], z[:, :, None], maxq) - z[:, :, None]) - w
    d2 = delta.reshape(r * n_cand, n)
    cost = ((d2 @ H) * d2).sum(axis=1).reshape(r, n_cand)                  # delta H delta^T
    k = np.argmin(cost, axis=1)                                            # first minimum
    rr = np.arange(r)
    return s[rr, k], z[rr, k]


# --------------------------------------------------------------------------
# Algorithm 3: in-channel sweep
# --------------------------------------------------------------------------

def sweep_P(R, U):
    """P = ((R U^T) * M_U) U with M_U the strictly-upper mask (Algorithm 3, line 2)."""
    return np.triu(np.asarray(R, F64) @ U.T, k=1) @ U


def gptaq_sweep(Wb, U, P, s, z, bits, group=0, H_in=None, adaptive=True,
                grid_points=100, max_shrink=0.8):
    """Algorithm 3 on the rows Wb [r, n] (modified in a private copy).

    s, z: [r, n_groups] arrays; with group > 0 and adaptive, the (s, z) of a group are
    recomputed when the sweep enters it, from the current columns of that group and
    H_in[G, G] (they are written into s, z in place).
    Returns Q [r, n] (dequantized) and codes [r, n]."""
    Wk = np.array(Wb, F64, copy=True)
    r, n = Wk.shape
    maxq = F64(2 ** bits - 1)
    Q = np.zeros((r, n), F64); codes = np.zeros((r, n), F64)
    for j in range(n):
        gi = j // group if group else 0
        if group and adaptive and j % group == 0:
            G = slice(j, j + group)
            s[:, gi], z[:, gi] = grid_search(Wk[:, G], H_in[G, G], bits, grid_points, max_shrink)
        wj = Wk[:, j].copy()
        q = quantize_codes(wj, s[:, gi], z[:, gi], maxq)
        Qj = s[:, gi] * (q - z[:, gi])
        codes[:, j] = q; Q[:, j] = Qj
        e = (wj - Qj) / U[j, j]
        Wk[:, j:] -= np.outer(e, U[j, j:])
        if P is not None:
            Wk[:, j:] -= np.outer(wj, P[j, j:])
    return Q, codes


# --------------------------------------------------------------------------
# Prop. 3.1 / 3.2: compensation of the remaining out-channels
# --------------------------------------------------------------------------

def block_schedule(d_h, block):
    """Index ranges [i0, i1) of the sequential out-channel steps i = 0, N, 2N, ... (Algorithm 1,
    line 7); the last block is ragged when N does not divide d_h."""
    return [(i0, min(i0 + block, d_h)) for i0 in range(0, d_h, block)]


def compensation_matrix(U_out, i0, i1):
    """T = [U_out^T]_{i1:, B} [U_out^T]_{B, B}^{-1},  B = {i0 .. i1-1}  (Prop. 3.1)."""
    Lo = U_out.T
    return Lo[i1:, i0:i1] @ np.linalg.inv(Lo[i0:i1, i0:i1])


def residual_S(R, H_in):
    """S = R H_in^{-1}, the factor of the upstream-error term of Prop. 3.2."""
    return np.asarray(R, F64) @ np.linalg.inv(np.asarray(H_in, F64))


def compensation_update(U_out, i0, i1, Wb, Qb, S=None):
    """[Delta W]_{i1:, :} = -T ((W_B - Q_B) - W_B R H_in^{-1})  (Prop. 3.2; Prop. 3.1 when S is None).
    Wb are the rows of the block as they were when its quantization began."""
    E = Wb - Qb
    if S is not None:
        E = E - Wb @ S
    return -compensation_matrix(U_out, i0, i1) @ E


# --------------------------------------------------------------------------
# Prop. 3.3 / Algorithm 2: coordinate-descent scale refinement
# --------------------------------------------------------------------------

def cd_refine(W, Wbar_int, s, H_in, H_out, R, n_iter, group=0):
    """Algorithm 2 for one head.  W [r, n] original FP weights, Wbar_int = codes - z [r, n],
    s [r, n_groups] refined in place, H_out [r, r] (identity if None), R [n, n] or None.

    Per-row (group = 0): s_j += [Wbar (H_in (W-Q)^T - R^T W^T) H_out]_jj
                                / ([Wbar H_in Wbar^T]_jj [H_out]_jj)      (Prop. 3.3)
    evaluated with the current Q, in order j = 0 .. r-1.
    Group-wise: the coordinate is (j, G); Wbar is masked to the columns of G in the leading
    factor of the numerator and in the denominator."""
    W = np.asarray(W, F64)
    r, n = W.shape
    Ho = np.eye(r) if H_out is None else np.asarray(H_out, F64)
    ng = s.shape[1]
    gsz = group if group else n
    WR = (W @ R) if R is not None else np.zeros((r, n), F64)   # (R^T W^T)^T
    Q = np.repeat(s, gsz, axis=1) * Wbar_int
    for _ in range(n_iter):
        for j in range(r):
            for gi in range(ng):
                G = slice(gi * gsz, (gi + 1) * gsz)
                wb = Wbar_int[j, G]
                a = wb @ H_in[G, :]                             # row j of Wbar(masked to G) H_in
                # row j of Wbar (H_in (W-Q)^T - R^T W^T), with the current Q:
                m = (W - Q) @ a - WR[:, G] @ wb
                num = m @ Ho[:, j]
                den = (a[G] @ wb) * Ho[j, j]
                if den > 0.0:
                    s[j, gi] = s[j, gi] + num / den
                Q[j, G] = s[j, gi] * Wbar_int[j, G]
    return s


# --------------------------------------------------------------------------
# packed form of the codes
# --------------------------------------------------------------------------

def pack_codes(codes, bits):
    """Row-wise little-endian bit stream: code c occupies bits [bits*c, bits*c + bits); stored as uint32 words
    (bit i of the stream is bit i % 32 of word i // 32), each row padded with zero bits to whole words."""
    codes = np.asarray(codes)
    d_out, d_in = codes.shape
    wpr = (d_in * bits + 31) // 32
    stream = np.zeros((d_out, wpr * 32), np.uint8)
    for b in range(bits):
        stream[:, b:d_in * bits:bits] = (codes >> b) & 1
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (stream.reshape(d_out, wpr, 32).astype(np.uint64) * weights).sum(axis=2).astype(np.uint32)


def dequant_matvec(codes, scales, zeros, x, group=0):
    """y = W_deq x with W_deq = scales (codes - zeros), (scale, zero) per row and group of in-channels."""
    codes = np.asarray(codes, F64)
    gsz = group if group else codes.shape[1]
    Wd = np.repeat(np.asarray(scales, F64), gsz, axis=1) * (codes - np.repeat(np.asarray(zeros, F64), gsz, axis=1))
    return Wd @ np.asarray(x, F64)


# --------------------------------------------------------------------------
# losses
# --------------------------------------------------------------------------

def layer_loss(W, Q, H_in, H_out, R):
    """(quad, cross) with quad = tr(H_out D H_in D^T), cross = 2 tr(H_out W R D^T), D = Q - W:
    the D-dependent part of ||G D X + G W dX||_F^2 (App. D, first display)."""
    D = Q - W
    Ho = np.eye(W.shape[0]) if H_out is None else H_out
    quad = np.trace(Ho @ D @ H_in @ D.T)
    cross = 2.0 * np.trace(Ho @ W @ R @ D.T) if R is not None else 0.0
    return quad, cross


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------

def quantize_layer(W, H_in, H_out, R, n_heads, bits, block, group=0, cd_iters=1,
                   adaptive_grid=True, grid_points=100, max_shrink=0.8, damp=0.01):
    """Algorithm 1 for one projection weight.

    W [d_out, d_in], d_out = n_heads * d_h; H_in [d_in, d_in] or [n_heads, d_in, d_in];
    H_out [n_heads, d_h, d_h] or None (identity: no out-channel coupling, the output-projection /
    GPTQ case); R like H_in (already alpha-scaled) or None.
    Returns dict(codes, scales, zeros, W_deq, loss, loss_quad, loss_cross, loss_per_head [n_heads],
    loss_per_head_terms [n_heads, 2] = (quad, cross) of every head).
    Every Hessian is damped once at entry and the damped matrices are used throughout."""
    W = np.asarray(W, F64)
    d_out, n = W.shape
    dh = d_out // n_heads
    ng = n // group if group else 1
    per_head_in = (np.ndim(H_in) == 3)
    codes = np.zeros((d_out, n), F64)
    scales = np.zeros((d_out, ng), F64); zeros = np.zeros((d_out, ng), F64)
    Qfull = np.zeros((d_out, n), F64)
    loss_per_head = np.zeros((n_heads, 2), F64)

    shared = None
    for h in range(n_heads):
        rows = slice(h * dh, (h + 1) * dh)
        if per_head_in or shared is None:
            Hi = damp_hessian(H_in[h] if per_head_in else H_in, damp)
            Rh = None if R is None else np.asarray(R[h] if per_head_in else R, F64)
            U_in = chol_inv_upper(Hi)
            P = sweep_P(Rh, U_in) if Rh is not None else None
            S = residual_S(Rh, Hi) if Rh is not None else None
            shared = (Hi, Rh, U_in, P, S)
        Hi, Rh, U_in, P, S = shared
        Ho = None if H_out is None else damp_hessian(H_out[h], damp)
        U_out = None if Ho is None else chol_inv_upper(Ho)

        Wh = W[rows]
        Wt = Wh.copy()                                        # W~ <- W
        s = scales[rows]; z = zeros[rows]
        if not adaptive_grid:                                 # BoA: one grid from the original weights
            if group:
                for gi in range(ng):
                    G = slice(gi * group, (gi + 1) * group)
                    s[:, gi], z[:, gi] = grid_search(Wh[:, G], Hi[G, G], bits, grid_points, max_shrink)
            else:
                s[:, 0], z[:, 0] = grid_search(Wh, Hi, bits, grid_points, max_shrink)
        for i0, i1 in block_schedule(dh, block):
            Wb = Wt[i0:i1].copy()                             # W^(i): rows as they are when the block starts
            sb = s[i0:i1]; zb = z[i0:i1]
            if adaptive_grid and not group:
                sb[:, 0], zb[:, 0] = grid_search(Wb, Hi, bits, grid_points, max_shrink)
            Qb, cb = gptaq_sweep(Wb, U_in, P, sb, zb, bits, group, Hi, adaptive_grid,
                                 grid_points, max_shrink)
            Qfull[rows][i0:i1] = Qb; codes[rows][i0:i1] = cb
            if U_out is not None and i1 < dh:
                Wt[i1:] += compensation_update(U_out, i0, i1, Wb, Qb, S)
        if cd_iters > 0:
            gsz = group if group else n
            Wbar = codes[rows] - np.repeat(z, gsz, axis=1)
            cd_refine(Wh, Wbar, s, Hi, Ho, Rh, cd_iters, group)
            Qfull[rows] = np.repeat(s, gsz, axis=1) * Wbar
        loss_per_head[h] = layer_loss(Wh, Qfull[rows], Hi, Ho, Rh)

    quad = loss_per_head[:, 0].sum(); cross = loss_per_head[:, 1].sum()
    return dict(codes=codes.astype(np.uint8), scales=scales, zeros=zeros, W_deq=Qfull,
                loss=quad + cross, loss_quad=quad, loss_cross=cross,
                loss_per_head=loss_per_head.sum(axis=1), loss_per_head_terms=loss_per_head)
