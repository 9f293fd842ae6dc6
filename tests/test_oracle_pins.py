"""Pins of the fp64 oracle against what the paper and plain mathematics fix.

Every expected value here is computed by a route that does not go through the oracle's own
formula for the same quantity: brute-force constrained least squares, direct Frobenius norms
with explicit G, X, dX, textbook elimination on H^-1, exhaustive loops.
"""
import os

import numpy as np
import pytest

from oracle import turboboa_ref as O

rng = np.random.default_rng


def spd(n, seed, cond=30.0):
    A = rng(seed).standard_normal((n, 3 * n))
    H = A @ A.T
    return H + (np.trace(H) / n / cond) * np.eye(n)


def direct_softmax_causal(S):
    L = S.shape[0]
    A = np.zeros_like(S)
    for t in range(L):
        row = S[t, :t + 1]
        e = np.exp(row - row.max())
        A[t, :t + 1] = e / e.sum()
    return A


# ---------------------------------------------------------------- structure (Sec. 3.1 examples)

def test_block_schedule_matches_printed_counts():
    path = os.path.join(os.path.dirname(__file__), "golden", "sequential_steps.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for d_h, n, steps, comp_rows in rows:
        sched = O.block_schedule(int(d_h), int(n))
        assert len(sched) == int(steps)
        assert int(d_h) - sched[0][1] == int(comp_rows)      # rows that absorb the first block's error
    assert O.block_schedule(10, 4) == [(0, 4), (4, 8), (8, 10)]


# ---------------------------------------------------------------- Table 1

@pytest.fixture(scope="module")
def small_block():
    r = rng(1)
    S, L, d, Hq, Hkv, dh = 3, 7, 12, 4, 2, 3
    X = r.standard_normal((S, L, d))
    Xf = X - 0.1 * r.standard_normal((S, L, d))
    Wq = r.standard_normal((Hq * dh, d)) * 0.4
    Wk = r.standard_normal((Hkv * dh, d)) * 0.4
    Wv = r.standard_normal((Hkv * dh, d)) * 0.4
    Wo = r.standard_normal((d, Hq * dh)) * 0.4
    Hs = O.build_hessians(X, Xf, Wq, Wk, Wv, Wo, Hq, Hkv, dh, alpha=1.0)
    return dict(S=S, L=L, d=d, Hq=Hq, Hkv=Hkv, dh=dh, X=X, Xf=Xf, Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, Hs=Hs)


def test_hessian_qk_trace_identity_and_kron(small_block):
    b = small_block
    d, dh, rep = b["d"], b["dh"], b["Hq"] // b["Hkv"]
    Xall = b["X"].reshape(-1, d)                       # tokens x d ; the paper's X is Xall.T
    dXall = (b["X"] - b["Xf"]).reshape(-1, d)
    r = rng(2)
    for h in range(b["Hq"]):
        g = h // rep
        K = Xall @ b["Wk"][g * dh:(g + 1) * dh].T      # G = K_h for W_Q,h
        D = r.standard_normal((dh, d)); W = r.standard_normal((dh, d))
        direct = np.linalg.norm(K @ D @ Xall.T) ** 2
        Hin, Hout = b["Hs"]["Hin_qk"], b["Hs"]["Hout_q"][h]
        assert np.isclose(np.trace(Hout @ D @ Hin @ D.T), direct, rtol=1e-10)
        v = D.reshape(-1, order="F")                   # column-stacking vec
        assert np.isclose(v @ np.kron(Hin, Hout) @ v, direct, rtol=1e-10)
        # cross term pins the orientation of R = dX X^T
        cross = 2.0 * np.sum((K @ D @ Xall.T) * (K @ W @ dXall.T))
        assert np.isclose(2.0 * np.trace(Hout @ W @ b["Hs"]["R_qk"] @ D.T), cross, rtol=1e-9)
        q, c = O.layer_loss(W, W + D, Hin, Hout, b["Hs"]["R_qk"])
        full = np.linalg.norm(K @ D @ Xall.T + K @ W @ dXall.T) ** 2 - np.linalg.norm(K @ W @ dXall.T) ** 2
        assert np.isclose(q + c, full, rtol=1e-9)


def test_hessian_k_layer_sums_query_heads_of_group(small_block):
    b = small_block
    d, dh, rep = b["d"], b["dh"], b["Hq"] // b["Hkv"]
    Xall = b["X"].reshape(-1, d)
    D = rng(3).standard_normal((dh, d))
    for g in range(b["Hkv"]):
        direct = 0.0
        for h in range(g * rep, (g + 1) * rep):        # sum_h ||Q_h dW_K,g X||^2
            Q = Xall @ b["Wq"][h * dh:(h + 1) * dh].T
            direct += np.linalg.norm(Q @ D @ Xall.T) ** 2
        assert np.isclose(np.trace(b["Hs"]["Hout_k"][g] @ D @ b["Hs"]["Hin_qk"] @ D.T), direct, rtol=1e-10)


def test_hout_q_closed_form(small_block):
    b = small_block
    dh, rep = b["dh"], b["Hq"] // b["Hkv"]
    for h in range(b["Hq"]):
        Wk_g = b["Wk"][(h // rep) * dh:(h // rep + 1) * dh]
        assert np.allclose(b["Hs"]["Hout_q"][h], Wk_g @ b["Hs"]["Hin_qk"] @ Wk_g.T, rtol=1e-10)


def test_hessian_v_direct(small_block):
    """sum_{h in g} sum_s ||W_out,h dW X_s A_h^T||_F^2 with A built by an explicit per-row softmax."""
    b = small_block
    d, dh, rep, L = b["d"], b["dh"], b["Hq"] // b["Hkv"], b["L"]
    r = rng(4)
    for g in range(b["Hkv"]):
        D = r.standard_normal((dh, d)); W = r.standard_normal((dh, d))
        quad = 0.0; cross = 0.0; kron_sum = np.zeros((d * dh, d * dh))
        for h in range(g * rep, (g + 1) * rep):
            Wout = b["Wo"][:, h * dh:(h + 1) * dh]
            for s in range(b["S"]):
                def eff_input(X):
                    Q = X[s] @ b["Wq"][h * dh:(h + 1) * dh].T
                    K = X[s] @ b["Wk"][g * dh:(g + 1) * dh].T
                    A = direct_softmax_causal(Q @ K.T / np.sqrt(dh))
                    return X[s].T @ A.T                 # d x L : the paper's X A_h^T
                Z = eff_input(b["X"]); Zf = eff_input(b["Xf"])
                quad += np.linalg.norm(Wout @ D @ Z) ** 2
                cross += 2.0 * np.sum((Wout @ D @ Z) * (Wout @ W @ (Z - Zf)))
                kron_sum += np.kron(Z @ Z.T, Wout.T @ Wout)
        Hin, Hout, R = b["Hs"]["Hin_v"][g], b["Hs"]["Hout_v"][g], b["Hs"]["R_v"][g]
        if rep == 1:
            assert np.isclose(np.trace(Hout @ D @ Hin @ D.T), quad, rtol=1e-10)
        # with several query heads per KV head the true Hessian is a sum of Kronecker products;
        # the factors are the sums over the group (documented approximation): check the factors.
        Hin_direct = np.zeros((d, d)); Hout_direct = np.zeros((dh, dh))
        for h in range(g * rep, (g + 1) * rep):
            Wout = b["Wo"][:, h * dh:(h + 1) * dh]
            Hout_direct += Wout.T @ Wout
            for s in range(b["S"]):
                Q = b["X"][s] @ b["Wq"][h * dh:(h + 1) * dh].T
                K = b["X"][s] @ b["Wk"][g * dh:(g + 1) * dh].T
                Y = direct_softmax_causal(Q @ K.T / np.sqrt(dh)) @ b["X"][s]
                Hin_direct += Y.T @ Y
        assert np.allclose(Hin, Hin_direct, rtol=1e-10) and np.allclose(Hout, Hout_direct, rtol=1e-10)
        assert np.allclose(Hin, Hin.T) and np.all(np.linalg.eigvalsh(Hin) > -1e-9)
        assert R.shape == (d, d)


def test_hessian_v_single_kv_group_is_exact_kronecker():
    r = rng(5)
    S, L, d, H, dh = 2, 6, 8, 2, 3
    X = r.standard_normal((S, L, d)); Xf = X + 0.1 * r.standard_normal((S, L, d))
    Wq, Wk, Wv = (r.standard_normal((H * dh, d)) * 0.5 for _ in range(3))
    Wo = r.standard_normal((d, H * dh))
    Hs = O.build_hessians(X, Xf, Wq, Wk, Wv, Wo, H, H, dh, alpha=0.5)
    for h in range(H):
        D = r.standard_normal((dh, d)); W = r.standard_normal((dh, d))
        Wout = Wo[:, h * dh:(h + 1) * dh]
        quad = cross = 0.0
        for s in range(S):
            def Z_of(Xa):
                A = direct_softmax_causal((Xa[s] @ Wq[h*dh:(h+1)*dh].T) @ (Xa[s] @ Wk[h*dh:(h+1)*dh].T).T / np.sqrt(dh))
                return Xa[s].T @ A.T
            Z, Zf = Z_of(X), Z_of(Xf)
            quad += np.linalg.norm(Wout @ D @ Z) ** 2
            cross += 2.0 * np.sum((Wout @ D @ Z) * (Wout @ W @ (Z - Zf)))
        q, c = O.layer_loss(W, W + D, Hs["Hin_v"][h], Hs["Hout_v"][h], Hs["R_v"][h])
        assert np.isclose(q, quad, rtol=1e-10)
        assert np.isclose(c, 0.5 * cross, rtol=1e-9)          # alpha = 0.5 scales R


def test_attention_special_cases():
    r = rng(6)
    d, dh = 6, 2
    X = r.standard_normal((4, 1, d))                     # L = 1: A = [1] so H_in^V = H_in
    W = r.standard_normal((dh, d))
    Hs = O.build_hessians(X, None, W, W, W, r.standard_normal((d, dh)), 1, 1, dh)
    assert np.allclose(Hs["Hin_v"][0], Hs["Hin_qk"])
    assert Hs["R_qk"] is None and Hs["R_v"] is None
    Xs = r.standard_normal((9, d))
    A, _, _ = O.attention_probs(Xs, W, W, causal=True)
    assert np.allclose(A.sum(1), 1.0) and np.allclose(np.triu(A, 1), 0.0)
    assert np.allclose((A @ Xs)[0], Xs[0])               # first token attends to itself only
    assert np.allclose(A, direct_softmax_causal((Xs @ W.T) @ (Xs @ W.T).T / np.sqrt(dh)))
    A2, _, _ = O.attention_probs(Xs, W, W, causal=False)
    assert np.all(A2 > 0) and np.allclose(A2.sum(1), 1.0)


def test_out_proj_hessian(small_block):
    b = small_block
    args = (b["Hq"], b["Hkv"], b["dh"])
    Wq2, Wk2, Wv2 = b["Wq"] * 0.9, b["Wk"] * 1.1, b["Wv"] * 0.95
    Hin_o, R_o = O.build_hessian_out_proj(b["X"], b["Xf"], Wq2, Wk2, Wv2, b["Wq"], b["Wk"], b["Wv"], *args, alpha=1.0)
    dq = b["Hq"] * b["dh"]; d, dh, rep = b["d"], b["dh"], b["Hq"] // b["Hkv"]

    def attn_out(X, Wq, Wk, Wv):
        rows = []
        for s in range(b["S"]):
            heads = []
            for h in range(b["Hq"]):
                g = h // rep
                A = direct_softmax_causal((X[s] @ Wq[h*dh:(h+1)*dh].T) @ (X[s] @ Wk[g*dh:(g+1)*dh].T).T / np.sqrt(dh))
                heads.append(A @ (X[s] @ Wv[g*dh:(g+1)*dh].T))
            rows.append(np.concatenate(heads, axis=1))
        return np.concatenate(rows, axis=0)              # tokens x dq
    Oq = attn_out(b["X"], Wq2, Wk2, Wv2); Of = attn_out(b["Xf"], b["Wq"], b["Wk"], b["Wv"])
    D = rng(7).standard_normal((d, dq)); W = rng(8).standard_normal((d, dq))
    q, c = O.layer_loss(W, W + D, Hin_o, None, R_o)
    direct = np.linalg.norm(D @ Oq.T + W @ (Oq - Of).T) ** 2 - np.linalg.norm(W @ (Oq - Of).T) ** 2
    assert np.isclose(q + c, direct, rtol=1e-9)


def test_act_fakequant():
    X = rng(9).standard_normal((5, 40)) * np.array([[1], [3], [0.2], [10], [1]])
    Y = O.act_fakequant_per_token(X, 4)
    for t in range(5):
        assert len(np.unique(Y[t])) <= 16
        step = (X[t].max() - X[t].min()) / 15
        assert np.max(np.abs(Y[t] - X[t])) <= step / 2 + 1e-12
        lv = np.unique(Y[t]); assert np.allclose(np.diff(lv) / step, np.rint(np.diff(lv) / step))
    assert np.allclose(O.act_fakequant_per_token(np.zeros((2, 8)), 4), 0.0)


def test_hadamard_rotation_is_the_sylvester_transform():
    """Pins of the rotation: entries (-1)^popcount(i & j), orthogonality, a brute-force butterfly, one-hot inputs."""
    d = 64
    H = O.hadamard_matrix(d)
    pc = np.array([[bin(i & j).count("1") for j in range(d)] for i in range(d)])
    assert np.array_equal(H, (-1.0) ** pc)
    assert np.array_equal(H @ H.T, d * np.eye(d))
    X = rng(21).standard_normal((7, d)); sg = np.where(rng(22).random(d) < 0.5, -1.0, 1.0)
    Y = O.hadamard_rotate(X, sg)
    assert np.allclose(np.linalg.norm(Y, axis=1), np.linalg.norm(X, axis=1), rtol=1e-12)          # orthogonal: norms kept
    assert np.allclose(O.hadamard_rotate(Y) * sg, X, atol=1e-12)                                   # H / sqrt(d) is an involution
    # textbook in-place butterfly network written out on plain lists
    def fwht(v):
        v = list(v); h = 1
        while h < len(v):
            for i in range(0, len(v), 2 * h):
                for j in range(i, i + h):
                    v[j], v[j + h] = v[j] + v[j + h], v[j] - v[j + h]
            h *= 2
        return np.array(v) / np.sqrt(len(v))
    for t in range(3):
        assert np.allclose(Y[t], fwht(X[t] * sg), atol=1e-12)
    e = np.zeros(d); e[5] = 1.0
    assert np.allclose(O.hadamard_rotate(e[None])[0], H[5] / 8.0)
    # outlier channels are spread: the largest |entry| of a row with one dominant channel drops by about sqrt(d)
    Xo = rng(23).standard_normal((4, d)); Xo[:, 3] *= 100
    assert np.abs(O.hadamard_rotate(Xo)).max() < np.abs(Xo).max() / 4


def test_mlp_pieces():
    """Layer-wise Hessian of a plain linear layer and the SwiGLU activation."""
    from scipy.special import expit
    X = rng(40).standard_normal((3, 20, 12)); Xf = X + 0.1 * rng(41).standard_normal(X.shape)
    H, R = O.build_hessian_linear(X, Xf, 0.25)
    X2, Xf2 = X.reshape(-1, 12), Xf.reshape(-1, 12)
    D = rng(42).standard_normal((5, 12)); W = rng(43).standard_normal((5, 12))
    # ||D X + W dX||^2 - ||W dX||^2 = tr(D H D^T) + 2 tr(W (R / alpha) D^T)   (App. D, first display, G = I)
    direct = np.linalg.norm(D @ X2.T + W @ (X2 - Xf2).T) ** 2 - np.linalg.norm(W @ (X2 - Xf2).T) ** 2
    assert np.isclose(np.trace(D @ H @ D.T) + 2 * np.trace(W @ (R / 0.25) @ D.T), direct, rtol=1e-10)
    # the same sums as the attention block's H_in, R for W_Q / W_K
    Wz = np.zeros((8, 12))
    Hs = O.build_hessians(X, Xf, Wz, Wz, Wz, np.zeros((12, 8)), 2, 2, 4, alpha=0.25)
    assert np.allclose(H, Hs["Hin_qk"]) and np.allclose(R, Hs["R_qk"])
    Wg = rng(44).standard_normal((7, 12)); Wu = rng(45).standard_normal((7, 12))
    A = O.swiglu(X, Wg, Wu)
    G, U = X @ Wg.T, X @ Wu.T
    assert np.allclose(A, G * expit(G) * U, rtol=1e-12)                     # silu(g) = g sigmoid(g), library sigmoid
    assert np.allclose(O.swiglu(X, 0 * Wg, Wu), 0.0)                          # silu(0) = 0
    big = O.swiglu(np.array([[40.0]]), np.array([[1.0]]), np.array([[2.0]]))
    assert np.isclose(big[0, 0], 40.0 * 80.0, rtol=1e-12)                     # silu(g) -> g for large g


def test_pack_codes_bit_stream():
    """Hand-computed words, and an independent unpacking through Python integers."""
    assert O.pack_codes(np.array([[1, 2, 3, 0]]), 2).tolist() == [[1 | 2 << 2 | 3 << 4]]
    assert O.pack_codes(np.array([[7, 0, 5]]), 3).tolist() == [[7 | 5 << 6]]
    assert O.pack_codes(np.array([[0xAB, 0xCD, 0xEF, 0x01, 0x23]]), 8).tolist() == [[0x01EFCDAB, 0x23]]
    # eleven 3-bit codes: the eleventh (bits 30..32) straddles the word boundary
    c = np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 5, 3]])
    big = sum(int(v) << (3 * i) for i, v in enumerate(c[0]))
    assert O.pack_codes(c, 3).tolist() == [[big & 0xFFFFFFFF, big >> 32]]
    for bits in (2, 3, 4, 8):
        codes = rng(30 + bits).integers(0, 2 ** bits, size=(5, 77))
        P = O.pack_codes(codes, bits)
        assert P.shape == (5, (77 * bits + 31) // 32) and P.dtype == np.uint32
        for r in range(5):
            big = sum(int(w) << (32 * i) for i, w in enumerate(P[r]))
            assert [(big >> (bits * k)) & (2 ** bits - 1) for k in range(77)] == codes[r].tolist()
            assert big >> (bits * 77) == 0                      # padding bits are zero


# ---------------------------------------------------------------- eq. 3

def test_chol_inv_upper_textbook():
    H = spd(9, 10)
    U = O.chol_inv_upper(H)
    assert np.allclose(np.tril(U, -1), 0.0) and np.all(np.diag(U) > 0)
    assert np.allclose(U.T @ U @ H, np.eye(9), atol=1e-9)
    J = np.eye(9)[::-1]
    V = J @ np.linalg.cholesky(J @ H @ J) @ J              # upper, H = V V^T
    assert np.allclose(np.linalg.inv(V), U, rtol=1e-8, atol=1e-12)
    Hd = O.damp_hessian(H, 0.01)
    assert np.allclose(Hd - H, 0.01 * np.mean(np.diag(H)) * np.eye(9))
    assert O.damp_hessian(H, 0.0) is not H and np.array_equal(O.damp_hessian(H, 0.0), H)


# ---------------------------------------------------------------- Prop. 3.1 / 3.2

def brute_force_remaining_rows(Hin, Hout, dW_B, lin=None):
    """argmin over the free rows of tr(Hout dW Hin dW^T) + 2 tr(lin dW^T) with the first
    N rows of dW fixed to dW_B: dense KKT solve on the column-stacked Kronecker system."""
    do, di = Hout.shape[0], Hin.shape[0]
    N = dW_B.shape[0]
    K = np.kron(Hin, Hout)
    idx = np.arange(do * di).reshape(di, do).T           # idx[i, j] = position of dW[i, j] in vec
    fixed = idx[:N].reshape(-1); free = idx[N:].reshape(-1)
    xc = dW_B.reshape(-1)
    rhs = -K[np.ix_(free, fixed)] @ xc
    if lin is not None:
        rhs = rhs - lin[N:].reshape(-1)
    xf = np.linalg.solve(K[np.ix_(free, free)], rhs)
    return xf.reshape(do - N, di)


@pytest.mark.parametrize("N", [1, 2, 3])
def test_prop31_equals_brute_force(N):
    do, di = 6, 5
    Hin, Hout = spd(di, 11), spd(do, 12)
    r = rng(13 + N)
    W = r.standard_normal((do, di)); QB = np.rint(W[:N] * 2) / 2
    U = O.chol_inv_upper(Hout)
    got = O.compensation_update(U, 0, N, W[:N], QB)
    want = brute_force_remaining_rows(Hin, Hout, QB - W[:N])
    assert np.allclose(got, want, rtol=1e-8, atol=1e-10)
    Hi = np.linalg.inv(Hout)                              # the H_out^-1 form of App. C
    assert np.allclose(got, -Hi[N:, :N] @ np.linalg.inv(Hi[:N, :N]) @ (W[:N] - QB), rtol=1e-8, atol=1e-10)
    assert np.allclose(got, np.linalg.solve(Hout[N:, N:], Hout[N:, :N] @ (W[:N] - QB)), rtol=1e-8, atol=1e-10)
    got2 = O.compensation_update(U, 0, N, W[:N], QB)      # independent of H_in
    assert np.array_equal(got, got2)
    if N == 1:                                            # eq. 3 applied along out-channels
        assert np.allclose(got, -np.outer(U.T[1:, 0] / U[0, 0], W[0] - QB[0]))


def test_prop31_interior_block_is_subproblem_of_trailing_hessian():
    do, di, i0, i1 = 7, 4, 2, 5
    Hin, Hout = spd(di, 21), spd(do, 22)
    r = rng(23)
    Wb = r.standard_normal((i1 - i0, di)); Qb = np.rint(Wb)
    got = O.compensation_update(O.chol_inv_upper(Hout), i0, i1, Wb, Qb)
    want = brute_force_remaining_rows(Hin, Hout[i0:, i0:], Qb - Wb)
    assert np.allclose(got, want, rtol=1e-8, atol=1e-10)


def test_prop31_identity_hout_gives_zero():
    U = O.chol_inv_upper(np.eye(5) * 3.0)
    got = O.compensation_update(U, 1, 3, np.ones((2, 4)), np.zeros((2, 4)))
    assert np.array_equal(got, np.zeros((2, 4)))


@pytest.mark.parametrize("N", [1, 3])
def test_prop32_equals_brute_force_least_squares(N):
    do, di, m, L = 6, 4, 9, 11
    r = rng(31 + N)
    G = r.standard_normal((m, do)); X = r.standard_normal((di, L)); dX = 0.3 * r.standard_normal((di, L))
    W = r.standard_normal((do, di)); QB = np.rint(W[:N] * 2) / 2
    # min || G dW X + G[:, B] W_B dX ||_F^2, rows B of dW fixed: ordinary least squares on vec(dW)
    A = np.kron(X.T, G)
    idx = np.arange(do * di).reshape(di, do).T
    fixed = idx[:N].reshape(-1); free = idx[N:].reshape(-1)
    target = -(G[:, :N] @ W[:N] @ dX).reshape(-1, order="F") - A[:, fixed] @ (QB - W[:N]).reshape(-1)
    xf = np.linalg.lstsq(A[:, free], target, rcond=None)[0].reshape(do - N, di)
    Hin, Hout, R = X @ X.T, G.T @ G, dX @ X.T
    got = O.compensation_update(O.chol_inv_upper(Hout), 0, N, W[:N], QB, O.residual_S(R, Hin))
    assert np.allclose(got, xf, rtol=1e-7, atol=1e-9)
    # the same through the equivalent quadratic (App. D): extra linear term [H_out]_{:,B} W_B R
    want2 = brute_force_remaining_rows(Hin, Hout, QB - W[:N], lin=Hout[:, :N] @ W[:N] @ R)
    assert np.allclose(got, want2, rtol=1e-7, atol=1e-9)


# ---------------------------------------------------------------- grid search

def exhaustive_grid(w, H, bits, grid_points=100, max_shrink=0.8):
    maxq = 2 ** bits - 1
    lo, hi = min(w.min(), 0.0), max(w.max(), 0.0)
    if lo == hi:
        lo, hi = -1.0, 1.0
    best = (np.inf, None, None)
    k = 0
    while k < int(np.ceil(max_shrink * grid_points)):
        p = 1.0 - k / grid_points
        s = (p * hi - p * lo) / maxq
        z = np.rint(-(p * lo) / s)
        dq = np.array([s * (min(max(np.rint(x / s) + z, 0), maxq) - z) for x in w])
        c = (dq - w) @ H @ (dq - w)
        if c < best[0]:
            best = (c, s, z)
        k += 1
    return best


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_grid_search_equals_exhaustive(bits):
    n = 24
    H = spd(n, 40)
    Wr = rng(41).standard_normal((7, n)) * 0.02
    Wr[3] = 0.0; Wr[4] = np.abs(Wr[4])
    s, z = O.grid_search(Wr, H, bits)
    for i in range(7):
        c, s_e, z_e = exhaustive_grid(Wr[i], H, bits)
        assert s[i] == s_e and z[i] == z_e
        q = O.quantize_codes(Wr[i], s[i], z[i], 2 ** bits - 1)
        assert q.min() >= 0 and q.max() <= 2 ** bits - 1 and np.array_equal(q, np.rint(q))
        d0 = (Wr[i].max() - min(Wr[i].min(), 0.0)) / (2 ** bits - 1) if Wr[i].max() > 0 else None
        # never worse than the plain min-max grid (candidate k = 0)
        p0 = exhaustive_grid(Wr[i], H, bits, grid_points=100, max_shrink=0.01)[0]
        assert c <= p0
    assert s[3] == 2.0 / (2 ** bits - 1)                  # all-zero row: lo, hi -> -1, +1


# ---------------------------------------------------------------- Algorithm 3

def textbook_obs_row(w, H, s, z, maxq):
    """GPTQ/OBS on one row with explicit H^-1 and Gaussian elimination of the quantized coordinate."""
    w = w.copy(); n = len(w)
    Hinv = np.linalg.inv(H)
    codes = np.zeros(n)
    for j in range(n):
        q = min(max(np.rint(w[j] / s) + z, 0), maxq)
        codes[j] = q
        err = (w[j] - s * (q - z)) / Hinv[j, j]
        w[j + 1:] -= err * Hinv[j, j + 1:]
        Hinv[j + 1:, j + 1:] -= np.outer(Hinv[j + 1:, j], Hinv[j, j + 1:]) / Hinv[j, j]
    return codes


def test_sweep_without_R_is_textbook_obs():
    n, r_ = 20, 6
    H = spd(n, 50, cond=10)
    Wr = rng(51).standard_normal((r_, n))
    s, z = O.grid_search(Wr, H, 3)
    U = O.chol_inv_upper(H)
    Q, codes = O.gptaq_sweep(Wr, U, None, s[:, None].copy(), z[:, None].copy(), 3)
    for i in range(r_):
        assert np.array_equal(codes[i], textbook_obs_row(Wr[i], H, s[i], z[i], 7))
    assert np.array_equal(Q, s[:, None] * (codes - z[:, None]))
    # reduces the objective relative to plain rounding to the same grid
    rtn = s[:, None] * (O.quantize_codes(Wr, s[:, None], z[:, None], 7) - z[:, None])
    assert np.trace((Q - Wr) @ H @ (Q - Wr).T) < np.trace((rtn - Wr) @ H @ (rtn - Wr).T)


def test_sweep_with_R_structure():
    n, r_ = 16, 4
    r = rng(60)
    X = r.standard_normal((n, 80)); dX = 0.2 * r.standard_normal((n, 80))
    H, R = X @ X.T, dX @ X.T
    U = O.chol_inv_upper(H)
    P = O.sweep_P(R, U)
    assert np.allclose(np.tril(P), 0.0)                    # strictly upper
    # explicit double loop for P
    RU = R @ U.T
    P2 = np.zeros((n, n))
    for j in range(n):
        for k in range(n):
            P2[j, k] = sum(RU[j, m] * U[m, k] for m in range(j + 1, n))
    assert np.allclose(P, P2)
    Wr = r.standard_normal((r_, n))
    # an (almost) lossless grid: nothing to compensate, the sweep reduces to Q (I + P) = W
    s = np.full((r_, 1), 2.0 ** -40); z = np.full((r_, 1), 2.0 ** 45)
    Q, _ = O.gptaq_sweep(Wr, U, P, s, z, bits=47)
    assert np.allclose(Q @ (np.eye(n) + P), Wr, atol=1e-9)
    # with a real grid every column ends on its grid and codes are in range
    s, z = O.grid_search(Wr, H, 2)
    Q, codes = O.gptaq_sweep(Wr, U, P, s[:, None].copy(), z[:, None].copy(), 2)
    assert codes.min() >= 0 and codes.max() <= 3
    assert np.array_equal(Q, s[:, None] * (codes - z[:, None]))


# ---------------------------------------------------------------- Prop. 3.3 / Algorithm 2

def cd_problem(seed, r_=5, n=7, m=8, L=30, diag_out=False):
    r = rng(seed)
    G = np.diag(r.uniform(0.5, 2, r_)) if diag_out else r.standard_normal((m, r_))
    X = r.standard_normal((n, L)); dX = 0.2 * r.standard_normal((n, L))
    W = r.standard_normal((r_, n)) * 0.5
    z = np.full((r_, 1), 2.0)
    s0 = np.full((r_, 1), 0.4)
    Wbar = O.quantize_codes(W, s0, z, 3) - z
    def loss(s):
        Q = s.reshape(-1, 1) * Wbar
        return np.linalg.norm(G @ (Q - W) @ X + G @ W @ dX) ** 2
    return G, X, dX, W, Wbar, s0, loss


def test_cd_is_exact_coordinate_minimisation():
    G, X, dX, W, Wbar, s0, loss = cd_problem(70)
    Hin, Hout, R = X @ X.T, G.T @ G, dX @ X.T
    s = s0.copy()
    O.cd_refine(W, Wbar, s, Hin, Hout, R, n_iter=1)
    # independent Gauss-Seidel: minimise the directly evaluated loss along each coordinate
    # (a parabola through three evaluations)
    t = s0[:, 0].copy(); prev = loss(t)
    for j in range(len(t)):
        def f(x):
            u = t.copy(); u[j] = x; return loss(u)
        a, b_, c = f(t[j] - 1.0), f(t[j]), f(t[j] + 1.0)
        t[j] = t[j] - 0.5 * (c - a) / (c - 2 * b_ + a)
        cur = loss(t); assert cur <= prev + 1e-9; prev = cur
    assert np.allclose(s[:, 0], t, rtol=1e-7)
    # monotone over sweeps, converging to the dense solve of the quadratic (App. E)
    C = Wbar @ Hin @ Wbar.T
    M = C * Hout
    bvec = np.diag(Wbar @ (Hin - R).T @ W.T @ Hout)
    s_star = np.linalg.solve(M, bvec)
    losses = [loss(s0[:, 0])]
    s = s0.copy()
    for _ in range(200):
        O.cd_refine(W, Wbar, s, Hin, Hout, R, n_iter=1)
        losses.append(loss(s[:, 0]))
    assert all(b <= a + 1e-9 for a, b in zip(losses, losses[1:]))
    assert np.allclose(s[:, 0], s_star, rtol=1e-5)
    assert losses[0] - losses[1] > 10 * (losses[1] - losses[2]) or losses[1] - losses[2] < 1e-6 * losses[0]
    # n_iter = k equals k single sweeps
    s2 = s0.copy(); O.cd_refine(W, Wbar, s2, Hin, Hout, R, n_iter=3)
    s3 = s0.copy()
    for _ in range(3):
        O.cd_refine(W, Wbar, s3, Hin, Hout, R, n_iter=1)
    assert np.allclose(s2, s3, rtol=1e-12)


def test_cd_first_and_last_form_of_the_step_agree():
    G, X, dX, W, Wbar, s0, _ = cd_problem(71)
    Hin, Hout, R = X @ X.T, G.T @ G, dX @ X.T
    C = Wbar @ Hin @ Wbar.T
    bvec = np.diag(Wbar @ (Hin - R).T @ W.T @ Hout)
    t = s0[:, 0].copy()
    for j in range(len(t)):                                # first line of the derivation
        off = sum(C[j, k] * Hout[k, j] * t[k] for k in range(len(t)) if k != j)
        t[j] = (bvec[j] - off) / (C[j, j] * Hout[j, j])
    s = s0.copy(); O.cd_refine(W, Wbar, s, Hin, Hout, R, n_iter=1)
    assert np.allclose(s[:, 0], t, rtol=1e-9)


def test_cd_diagonal_hout_one_sweep_is_exact_and_none_is_identity():
    G, X, dX, W, Wbar, s0, loss = cd_problem(72, diag_out=True)
    Hin, Hout, R = X @ X.T, G.T @ G, dX @ X.T
    s = s0.copy(); O.cd_refine(W, Wbar, s, Hin, Hout, R, n_iter=1)
    bvec = np.diag(Wbar @ (Hin - R).T @ W.T)
    assert np.allclose(s[:, 0], bvec / np.diag(Wbar @ Hin @ Wbar.T), rtol=1e-9)
    s_id = s0.copy(); O.cd_refine(W, Wbar, s_id, Hin, None, R, n_iter=1)
    assert np.allclose(s_id, s, rtol=1e-9)                 # rows decouple: the diagonal drops out


def test_cd_groupwise_is_coordinate_minimisation_of_the_same_loss():
    r = rng(73)
    r_, n, g = 3, 8, 4
    G = r.standard_normal((6, r_)); X = r.standard_normal((n, 40)); dX = 0.1 * r.standard_normal((n, 40))
    W = r.standard_normal((r_, n)) * 0.5
    z = np.full((r_, 2), 2.0); s0 = np.full((r_, 2), 0.35)
    Wbar = O.quantize_codes(W, np.repeat(s0, g, 1), np.repeat(z, g, 1), 3) - np.repeat(z, g, 1)
    def loss(S):
        return np.linalg.norm(G @ (np.repeat(S, g, 1) * Wbar - W) @ X + G @ W @ dX) ** 2
    t = s0.copy()
    for j in range(r_):
        for gi in range(2):
            def f(x):
                u = t.copy(); u[j, gi] = x; return loss(u)
            a, b_, c = f(t[j, gi] - 1), f(t[j, gi]), f(t[j, gi] + 1)
            t[j, gi] -= 0.5 * (c - a) / (c - 2 * b_ + a)
    s = s0.copy(); O.cd_refine(W, Wbar, s, X @ X.T, G.T @ G, dX @ X.T, n_iter=1, group=g)
    assert np.allclose(s, t, rtol=1e-7)


# ---------------------------------------------------------------- Algorithm 1 as a whole

def independent_boa(W, Hin, Hout, n_heads, bits, damp):
    """Row-at-a-time BoA: fixed grid from the original weights, R = 0, no refinement; explicit
    H_out^-1 with rank-one downdating in place of Cholesky rows, textbook OBS inside a row."""
    d_out, n = W.shape
    dh = d_out // n_heads
    maxq = 2 ** bits - 1
    Hi = Hin + damp * np.mean(np.diag(Hin)) * np.eye(n)
    codes = np.zeros((d_out, n))
    for h in range(n_heads):
        Wh = W[h * dh:(h + 1) * dh].copy()
        Ho = Hout[h] + damp * np.mean(np.diag(Hout[h])) * np.eye(dh)
        Hoinv = np.linalg.inv(Ho)
        grids = [exhaustive_grid(Wh[i], Hi, bits)[1:] for i in range(dh)]
        for i in range(dh):
            s, z = grids[i]
            c = textbook_obs_row(Wh[i], Hi, s, z, maxq)
            codes[h * dh + i] = c
            err = Wh[i] - s * (c - z)
            Wh[i + 1:] -= np.outer(Hoinv[i + 1:, i] / Hoinv[i, i], err)
            Hoinv[i + 1:, i + 1:] -= np.outer(Hoinv[i + 1:, i], Hoinv[i, i + 1:]) / Hoinv[i, i]
    return codes


@pytest.fixture(scope="module")
def layer_case():
    r = rng(80)
    n_heads, dh, n, T = 2, 8, 24, 96
    X = r.standard_normal((T, n)); X[:, 3] *= 8
    dX = 0.1 * r.standard_normal((T, n))
    W = r.standard_normal((n_heads * dh, n)) * 0.02
    G = [r.standard_normal((T, dh)) + 0.7 * r.standard_normal((T, 1)) for _ in range(n_heads)]
    Hin = X.T @ X
    Hout = np.stack([g.T @ g for g in G])
    R = 0.25 * dX.T @ X
    return dict(W=W, Hin=Hin, Hout=Hout, R=R, n_heads=n_heads, dh=dh, n=n)


def test_block_one_reproduces_sequential_boa(layer_case):
    c = layer_case
    out = O.quantize_layer(c["W"], c["Hin"], c["Hout"], None, c["n_heads"], bits=2, block=1,
                           cd_iters=0, adaptive_grid=False, damp=0.01)
    want = independent_boa(c["W"], c["Hin"], c["Hout"], c["n_heads"], 2, 0.01)
    assert np.array_equal(out["codes"], want.astype(np.uint8))


@pytest.mark.parametrize("block", [1, 3, 4, 8])
@pytest.mark.parametrize("with_R", [False, True])
def test_pipeline_invariants(layer_case, block, with_R):
    c = layer_case
    R = c["R"] if with_R else None
    kw = dict(n_heads=c["n_heads"], bits=2, block=block, damp=0.01)
    out0 = O.quantize_layer(c["W"], c["Hin"], c["Hout"], R, cd_iters=0, **kw)
    out1 = O.quantize_layer(c["W"], c["Hin"], c["Hout"], R, cd_iters=1, **kw)
    out2 = O.quantize_layer(c["W"], c["Hin"], c["Hout"], R, cd_iters=2, **kw)
    for o in (out0, out1, out2):
        assert o["codes"].max() <= 3
        assert np.array_equal(o["W_deq"], o["scales"] * (o["codes"].astype(float) - o["zeros"]))
        assert np.array_equal(o["zeros"], np.rint(o["zeros"]))
        assert np.isclose(o["loss"], o["loss_per_head"].sum())
    assert np.array_equal(out0["codes"], out1["codes"])      # refinement freezes the integers
    assert out2["loss"] <= out1["loss"] <= out0["loss"]      # Table 9's shape
    assert out0["loss"] - out1["loss"] >= out1["loss"] - out2["loss"]
    again = O.quantize_layer(c["W"], c["Hin"], c["Hout"], R, cd_iters=1, **kw)
    assert np.array_equal(again["codes"], out1["codes"]) and np.array_equal(again["scales"], out1["scales"])
    # loss is what it claims to be, on the damped Hessians
    Hi = O.damp_hessian(c["Hin"], 0.01)
    tot = 0.0
    for h in range(c["n_heads"]):
        rows = slice(h * c["dh"], (h + 1) * c["dh"])
        D = out1["W_deq"][rows] - c["W"][rows]
        Ho = O.damp_hessian(c["Hout"][h], 0.01)
        v = D.reshape(-1, order="F")
        tot += v @ np.kron(Hi, Ho) @ v
        if with_R:
            tot += 2 * np.trace(Ho @ c["W"][rows] @ R @ D.T)
    assert np.isclose(out1["loss"], tot, rtol=1e-9)


def test_compensation_helps_and_beats_rtn(layer_case):
    c = layer_case
    kw = dict(n_heads=c["n_heads"], bits=2, cd_iters=0, damp=0.01)
    full = O.quantize_layer(c["W"], c["Hin"], c["Hout"], None, block=2, **kw)
    Hi = O.damp_hessian(c["Hin"], 0.01)
    s, z = O.grid_search(c["W"], Hi, 2)
    rtn = s[:, None] * (O.quantize_codes(c["W"], s[:, None], z[:, None], 3) - z[:, None])
    rtn_loss = sum(O.layer_loss(c["W"][h*8:(h+1)*8], rtn[h*8:(h+1)*8], Hi, O.damp_hessian(c["Hout"][h], 0.01), None)[0]
                   for h in range(2))
    assert full["loss"] < rtn_loss


def test_block_equal_head_dim_and_identity_hout_reduce_to_gptq(layer_case):
    c = layer_case
    kw = dict(bits=2, cd_iters=0, damp=0.01)
    gptq = O.quantize_layer(c["W"], c["Hin"], None, None, n_heads=1, block=16, **kw)
    whole = O.quantize_layer(c["W"], c["Hin"], c["Hout"], None, n_heads=c["n_heads"], block=c["dh"], **kw)
    assert np.array_equal(gptq["codes"], whole["codes"]) and np.array_equal(gptq["scales"], whole["scales"])
    eye = np.stack([np.eye(c["dh"])] * c["n_heads"])
    for blk in (1, 3):
        o = O.quantize_layer(c["W"], c["Hin"], eye, None, n_heads=c["n_heads"], block=blk, **kw)
        assert np.array_equal(gptq["codes"], o["codes"])
    # and with the upstream-error term: H_out = I is GPTAQ, rows decouple
    a = O.quantize_layer(c["W"], c["Hin"], None, c["R"], n_heads=1, block=16, **kw)
    b = O.quantize_layer(c["W"], c["Hin"], eye, c["R"], n_heads=c["n_heads"], block=2, **kw)
    assert np.array_equal(a["codes"], b["codes"])


def test_per_head_hin_and_groupwise(layer_case):
    c = layer_case
    Hin2 = np.stack([c["Hin"], c["Hin"] * 1.0])
    R2 = np.stack([c["R"], c["R"]])
    a = O.quantize_layer(c["W"], c["Hin"], c["Hout"], c["R"], c["n_heads"], bits=3, block=4)
    b = O.quantize_layer(c["W"], Hin2, c["Hout"], R2, c["n_heads"], bits=3, block=4)
    assert np.array_equal(a["codes"], b["codes"]) and np.allclose(a["scales"], b["scales"])
    g = O.quantize_layer(c["W"], c["Hin"], c["Hout"], c["R"], c["n_heads"], bits=3, block=4, group=8)
    assert g["scales"].shape == (16, 3) and g["codes"].max() <= 7
    assert np.array_equal(g["W_deq"], np.repeat(g["scales"], 8, 1) * (g["codes"].astype(float) - np.repeat(g["zeros"], 8, 1)))
    g0 = O.quantize_layer(c["W"], c["Hin"], c["Hout"], c["R"], c["n_heads"], bits=3, block=4, group=8, cd_iters=0)
    assert g["loss"] <= g0["loss"]
    # group = d_in is the per-row path
    gfull = O.quantize_layer(c["W"], c["Hin"], c["Hout"], c["R"], c["n_heads"], bits=3, block=4, group=24)
    assert np.array_equal(gfull["codes"], a["codes"]) and np.allclose(gfull["scales"], a["scales"], rtol=1e-12)


# ---------------------------------------------------------------- Algorithm 3 with R != 0, and Algorithm 1 around it,
# re-derived from explicit activations by least squares (no Cholesky factor, no P, no S anywhere on this route)

def lstsq_sweep_row(w, X, dX, s, z, maxq):
    """One row through the in-channel sweep, every step solved as the least-squares problem it stands for.

    X, dX [n, L] are the paper's X and X - X~ (channels x tokens).  Entering step j the row holds w; channel j is
    rounded to Q_j, and the channels after j move by the delta_F that minimises
        || (Q_j - w_j) x_j + delta_F X_F + w_j dx_j ||^2
    (x_j, dx_j: rows j of X and dX; F = the channels after j): the rounding error of channel j and the deviation that
    channel j carries (its value on entry to the step times dx_j) are absorbed by the channels not yet fixed.  Solving
    the normal equations with H_FF^-1 = U_FF^T U_FF gives the update line of Algorithm 3, e_j U[j, F] + w_j P[j, F]."""
    w = np.array(w, float); n = len(w)
    codes = np.zeros(n); Q = np.zeros(n)
    for j in range(n):
        wj = w[j]
        q = min(max(np.rint(wj / s) + z, 0.0), maxq)
        codes[j] = q; Q[j] = s * (q - z)
        if j + 1 < n:
            target = -((Q[j] - wj) * X[j] + wj * dX[j])
            w[j + 1:] += np.linalg.lstsq(X[j + 1:].T, target, rcond=None)[0]
    return codes, Q


def test_sweep_with_R_is_stepwise_least_squares():
    n, r_, L = 9, 5, 40
    r = rng(61)
    X = r.standard_normal((n, L)); X[2] *= 4.0
    dX = 0.3 * r.standard_normal((n, L)) + 0.2 * X          # deviations correlated with the input: a sizeable R
    H, R = X @ X.T, dX @ X.T
    U = O.chol_inv_upper(H)
    P = O.sweep_P(R, U)
    Wr = r.standard_normal((r_, n))
    for bits in (2, 4):
        maxq = 2 ** bits - 1
        s, z = O.grid_search(Wr, H, bits)
        Q, codes = O.gptaq_sweep(Wr, U, P, s[:, None].copy(), z[:, None].copy(), bits)
        flips_without_P = 0
        for i in range(r_):
            c_ls, Q_ls = lstsq_sweep_row(Wr[i], X, dX, s[i], z[i], maxq)
            assert np.array_equal(codes[i], c_ls), (bits, i)
            assert np.allclose(Q[i], Q_ls, rtol=1e-12)
            flips_without_P += int(np.sum(lstsq_sweep_row(Wr[i], X, 0 * dX, s[i], z[i], maxq)[0] != c_ls))
        assert flips_without_P > 0          # the deviation term matters on this case: the comparison above can see it


def independent_turboboa(W, Xs, dXs, Gs, n_heads, bits, block):
    """Algorithm 1 (no damping, no scale refinement) from explicit G_h, X_h, dX_h: the grid of a step by an exhaustive
    loop, the in-channel sweep as step-wise least squares, the compensation of the remaining out-channels as the dense
    constrained minimiser of || G dW X + G[:, B] W_B dX ||_F^2 (eq. 7) over the rows that are still free."""
    d_out, n = W.shape
    dh = d_out // n_heads
    maxq = 2 ** bits - 1
    codes = np.zeros((d_out, n)); scales = np.zeros(d_out)
    for h in range(n_heads):
        X, dX, G = Xs[h], dXs[h], Gs[h]
        Hin, Hout, R = X @ X.T, G.T @ G, dX @ X.T
        Wt = W[h * dh:(h + 1) * dh].copy()
        for i0 in range(0, dh, block):
            i1 = min(i0 + block, dh)
            Wb = Wt[i0:i1].copy(); Qb = np.zeros_like(Wb)
            for a in range(i1 - i0):
                _, s, z = exhaustive_grid(Wb[a], Hin, bits)
                codes[h * dh + i0 + a], Qb[a] = lstsq_sweep_row(Wb[a], X, dX, s, z, maxq)
                scales[h * dh + i0 + a] = s
            if i1 < dh:
                Ht = Hout[i0:, i0:]                         # rows before i0 are fixed and already accounted for
                Wt[i1:] += brute_force_remaining_rows(Hin, Ht, Qb - Wb, lin=Ht[:, :i1 - i0] @ Wb @ R)
    return codes, scales


@pytest.fixture(scope="module")
def explicit_case():
    r = rng(90)
    n_heads, dh, n, L, m = 2, 6, 5, 30, 9
    Xs = [r.standard_normal((n, L)) * np.array([[1.0], [3.0], [1.0], [0.5], [1.0]]) for _ in range(n_heads)]
    dXs = [0.25 * r.standard_normal((n, L)) + 0.15 * X for X in Xs]
    Gs = [r.standard_normal((m, dh)) + 0.8 * r.standard_normal((m, 1)) for _ in range(n_heads)]
    W = r.standard_normal((n_heads * dh, n))
    return dict(W=W, Xs=Xs, dXs=dXs, Gs=Gs, n_heads=n_heads, dh=dh, n=n)


@pytest.mark.parametrize("block", [1, 2, 4])
def test_algorithm1_with_R_equals_least_squares_reconstruction(explicit_case, block):
    """The deviation term of Prop. 3.2 inside the loop of Algorithm 1 (and the per-head H_in, R of the W_V row of
    Table 1): every head has activations of its own here."""
    c = explicit_case
    Hin = np.stack([X @ X.T for X in c["Xs"]]); R = np.stack([dX @ X.T for dX, X in zip(c["dXs"], c["Xs"])])
    Hout = np.stack([G.T @ G for G in c["Gs"]])
    for bits in (3, 4):
        out = O.quantize_layer(c["W"], Hin, Hout, R, c["n_heads"], bits=bits, block=block, cd_iters=0, damp=0.0)
        codes, scales = independent_turboboa(c["W"], c["Xs"], c["dXs"], c["Gs"], c["n_heads"], bits, block)
        assert np.array_equal(out["codes"], codes.astype(np.uint8)), (bits, block)
        assert np.allclose(out["scales"][:, 0], scales, rtol=1e-12)
    # the case can tell the terms apart: without the deviation the codes of the later steps differ
    zero = [0 * dX for dX in c["dXs"]]
    other, _ = independent_turboboa(c["W"], c["Xs"], zero, c["Gs"], c["n_heads"], 4, block)
    assert np.any(other != codes)


def test_per_head_hessians_are_taken_per_head(explicit_case):
    c = explicit_case
    Hin = np.stack([X @ X.T for X in c["Xs"]]); R = np.stack([dX @ X.T for dX, X in zip(c["dXs"], c["Xs"])])
    Hout = np.stack([G.T @ G for G in c["Gs"]])
    dh = c["dh"]
    both = O.quantize_layer(c["W"], Hin, Hout, R, 2, bits=3, block=2)
    for h in range(2):
        one = O.quantize_layer(c["W"][h * dh:(h + 1) * dh], Hin[h], Hout[h:h + 1], R[h], 1, bits=3, block=2)
        rows = slice(h * dh, (h + 1) * dh)
        assert np.array_equal(both["codes"][rows], one["codes"])
        assert np.array_equal(both["scales"][rows], one["scales"]) and np.array_equal(both["W_deq"][rows], one["W_deq"])
        assert np.isclose(both["loss_per_head"][h], one["loss"], rtol=1e-12)
        assert np.allclose(both["loss_per_head_terms"][h], [one["loss_quad"], one["loss_cross"]], rtol=1e-12)
    # the two heads' Hessians differ enough to matter: swapping them changes the result
    swapped = O.quantize_layer(c["W"], Hin[::-1], Hout, R[::-1], 2, bits=3, block=2)
    assert np.any(swapped["codes"] != both["codes"])


def test_act_fakequant_hand_computed_rows():
    """The per-token range always contains zero.  Rows worked out by hand, 2 bits (levels 0..3):
    [1, 2, 3, 4]: range [0, 4], s = 4/3, z = 0, levels rint(0.75, 1.5, 2.25, 3) = 1, 2, 2, 3 (1.5 rounds to even);
    [-4, -3, -2, -1]: range [-4, 0], s = 4/3, z = 3, levels rint(-3, -2.25, -1.5, -0.75) + 3 = 0, 1, 1, 2;
    [-1, 0, 1, 2]: range [-1, 2], s = 1, z = 1, exact."""
    Y = O.act_fakequant_per_token(np.array([[1.0, 2.0, 3.0, 4.0], [-4.0, -3.0, -2.0, -1.0], [-1.0, 0.0, 1.0, 2.0]]), 2)
    t = 4.0 / 3.0
    assert np.allclose(Y[0], [t, 2 * t, 2 * t, 3 * t], rtol=1e-15)
    assert np.allclose(Y[1], [-3 * t, -2 * t, -2 * t, -t], rtol=1e-15)
    assert np.array_equal(Y[2], [-1.0, 0.0, 1.0, 2.0])


def test_hout_k_closed_form_and_from_other_query_weights(small_block):
    """H_out of W_K,g = sum over the query heads of the group of W_Q,h H_in W_Q,h^T (no positional rotation), whatever query
    weights are put in: the reading of Algorithm 1 that forms the Hessians inside the loop over the layers takes the
    dequantized W_Q there."""
    b = small_block
    d, dh, rep = b["d"], b["dh"], b["Hq"] // b["Hkv"]
    Wq2 = np.rint(b["Wq"] * 4) / 4                               # stands in for a dequantized W_Q
    Hs2 = O.build_hessians(b["X"], b["Xf"], Wq2, b["Wk"], b["Wv"], b["Wo"], b["Hq"], b["Hkv"], dh, alpha=1.0)
    for Wq, Hs in ((b["Wq"], b["Hs"]), (Wq2, Hs2)):
        for g in range(b["Hkv"]):
            want = sum(Wq[h * dh:(h + 1) * dh] @ Hs["Hin_qk"] @ Wq[h * dh:(h + 1) * dh].T for h in range(g * rep, (g + 1) * rep))
            assert np.allclose(Hs["Hout_k"][g], want, rtol=1e-10)
    assert np.array_equal(Hs2["Hin_qk"], b["Hs"]["Hin_qk"]) and np.array_equal(Hs2["Hout_q"], b["Hs"]["Hout_q"])
    assert not np.allclose(Hs2["Hout_k"], b["Hs"]["Hout_k"], rtol=1e-3)


def test_hout_q_kv_cache_hand_computed():
    """H_out of W_Q from the keys of a 2-bit cache (Sec. 4.2, KV setting), rows worked out by hand: with W_K = I the keys
    are the tokens.  [0, 3]: range [0, 3], step 1, zero 0 -> stays.  [-1, 2]: range [-1, 2], step 1, zero 1 -> stays.
    [0.5, 2]: range [0, 2], step 2/3, zero 0, levels round(0.75) = 1 and 3 -> [2/3, 2].  Gram of the three rows."""
    X = np.array([[[0.0, 3.0], [-1.0, 2.0], [0.5, 2.0]]])
    H = O.hout_q_kv_cache(X, np.eye(2), 1, 1, 2, kv_bits=2)
    want = np.array([[0.0 + 1.0 + 4.0 / 9.0, 0.0 - 2.0 + 4.0 / 3.0], [0.0 - 2.0 + 4.0 / 3.0, 9.0 + 4.0 + 4.0]])
    np.testing.assert_allclose(H[0], want, rtol=1e-14)
    # two query heads on one KV head read the same cache; a second KV head is quantized on its own (its own range per token)
    Wk = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 0.0], [0.0, -1.0]])          # head 0: identity; head 1: (2 x0, -x1)
    H2 = O.hout_q_kv_cache(X, Wk, 4, 2, 2, kv_bits=2)
    np.testing.assert_allclose(H2[0], want, rtol=1e-14); np.testing.assert_allclose(H2[1], want, rtol=1e-14)
    # head 1 keys: [0, -3] -> stays; [-2, -2] -> range [-2, 0], step 2/3, zero 3 -> stays; [1, -2] -> range [-2, 1], step 1, zero 2 -> stays
    K1 = np.array([[0.0, -3.0], [-2.0, -2.0], [1.0, -2.0]])
    np.testing.assert_allclose(H2[2], K1.T @ K1, rtol=1e-14); np.testing.assert_allclose(H2[3], K1.T @ K1, rtol=1e-14)
    # keys that already lie on the grid of an 8-bit cache are kept, and the result is then the W_Q row of Table 1
    rng = np.random.default_rng(5)
    Xi = rng.integers(-100, 100, size=(2, 6, 4)).astype(np.float64)
    Xi[:, :, 0] = -100.0; Xi[:, :, 1] = 155.0          # every token spans exactly 255 steps of 1
    Hs = O.build_hessians(Xi, None, np.eye(4), np.eye(4), np.eye(4), np.eye(4), 1, 1, 4)
    np.testing.assert_allclose(O.hout_q_kv_cache(Xi, np.eye(4), 1, 1, 4, kv_bits=8)[0], Hs["Hout_q"][0], rtol=1e-13)


@pytest.mark.parametrize("with_R", [False, True])
def test_groupwise_layer_with_block_diagonal_hin_is_the_per_row_layer_on_every_group(with_R):
    """The (row, group) extension against the per-row algorithm it extends.  When H_in (and R) couple no two groups of
    in-channels, nothing of Algorithm 1 crosses a group boundary: U and P are block diagonal, so the sweep inside one group
    leaves the others alone; the grid of a group, searched when the sweep enters it, sees the columns as the step found
    them; the compensation of the remaining rows acts column by column; the refinement's objective is a sum over the
    groups.  The group-wise layer is then the per-row layer run on each group's columns by itself."""
    r = rng(91)
    n_heads, dh, g, ng, T = 2, 8, 8, 3, 64
    n = g * ng
    W = r.standard_normal((n_heads * dh, n)) * 0.02
    Hin = np.zeros((n, n)); R = np.zeros((n, n))
    for gi in range(ng):
        Xg = r.standard_normal((T, g)); Xg[:, 1] *= 4
        Hin[gi*g:(gi+1)*g, gi*g:(gi+1)*g] = Xg.T @ Xg
        R[gi*g:(gi+1)*g, gi*g:(gi+1)*g] = 0.25 * (0.1 * r.standard_normal((T, g))).T @ Xg
    G = [r.standard_normal((T, dh)) + 0.7 * r.standard_normal((T, 1)) for _ in range(n_heads)]
    Hout = np.stack([x.T @ x for x in G])
    Rq = R if with_R else None
    kw = dict(bits=3, block=4, damp=0.0)
    whole = O.quantize_layer(W, Hin, Hout, Rq, n_heads, group=g, **kw)
    loss = 0.0
    for gi in range(ng):
        sl = slice(gi * g, (gi + 1) * g)
        part = O.quantize_layer(W[:, sl], Hin[sl, sl], Hout, None if Rq is None else R[sl, sl], n_heads, **kw)
        assert np.array_equal(whole["codes"][:, sl], part["codes"]), gi
        np.testing.assert_allclose(whole["scales"][:, gi], part["scales"][:, 0], rtol=1e-9)
        assert np.array_equal(whole["zeros"][:, gi], part["zeros"][:, 0])
        np.testing.assert_allclose(whole["W_deq"][:, sl], part["W_deq"], rtol=1e-9, atol=1e-15)
        loss += part["loss"]
    np.testing.assert_allclose(whole["loss"], loss, rtol=1e-9)


def test_groupwise_sweep_against_stepwise_least_squares_with_grids_at_group_entry():
    """The in-channel sweep with (row, group) grids on coupled channels, re-derived without its factors: every step as the
    least-squares problem it solves (explicit X and X - X~), and on entering a group of columns the row's grid for that group
    from an exhaustive loop over the candidates on the columns as they stand THEN (the earlier groups' steps have moved
    them), with that group's block of H_in."""
    n, r_, L, g = 12, 4, 48, 4
    r = rng(67)
    X = r.standard_normal((n, L)); X[5] *= 3.0
    X[6:] += 0.6 * X[:6]                                      # couples the groups
    dX = 0.3 * r.standard_normal((n, L)) + 0.2 * X
    H, R = X @ X.T, dX @ X.T
    U = O.chol_inv_upper(H); P = O.sweep_P(R, U)
    Wr = r.standard_normal((r_, n))
    for bits in (2, 3):
        maxq = 2 ** bits - 1
        s = np.zeros((r_, n // g)); z = np.zeros((r_, n // g))
        Q, codes = O.gptaq_sweep(Wr, U, P, s, z, bits, group=g, H_in=H, adaptive=True)
        moved = 0
        for i in range(r_):
            w = Wr[i].copy()
            for j in range(n):
                if j % g == 0:
                    G = slice(j, j + g)
                    _, sj, zj = exhaustive_grid(w[G], H[G, G], bits)
                    assert np.isclose(s[i, j // g], sj, rtol=1e-12) and z[i, j // g] == zj, (bits, i, j)
                    moved += int(j > 0 and not np.allclose(w[G], Wr[i, G]))
                wj = w[j]
                q = min(max(np.rint(wj / sj) + zj, 0.0), maxq)
                assert codes[i, j] == q and np.isclose(Q[i, j], sj * (q - zj), rtol=1e-12)
                if j + 1 < n:
                    w[j + 1:] += np.linalg.lstsq(X[j + 1:].T, -((sj * (q - zj) - wj) * X[j] + wj * dX[j]), rcond=None)[0]
        assert moved > 0          # later groups were searched on columns that the sweep had already changed
