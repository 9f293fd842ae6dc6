"""Building blocks of the HIP library against numpy / the oracle (GPU)."""
import numpy as np
import pytest
import torch

from oracle import turboboa_ref as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context()
    yield c
    c.close()


# M <= 32 with a k-contiguous A takes the 32-row tile
@pytest.mark.parametrize("M,N,K", [(128, 128, 16), (256, 384, 64), (77, 131, 45), (1, 5, 3), (300, 64, 1000), (32, 640, 333), (20, 257, 77)])
@pytest.mark.parametrize("tA,tB", [(False, False), (False, True), (True, False), (True, True)])
def test_gemm_f64(ctx, M, N, K, tA, tB):
    print("gemm_f64", M, N, K, tA, tB, flush=True)
    r = np.random.default_rng(M * 7 + N * 3 + K)
    A = r.standard_normal((K, M) if tA else (M, K)); B = r.standard_normal((N, K) if tB else (K, N))
    C0 = r.standard_normal((M, N))
    want = 0.5 * (A.T if tA else A) @ (B.T if tB else B) - 2.0 * C0
    Cd = torch.tensor(C0, device="cuda")
    got = ctx.gemm_f64(torch.tensor(A, device="cuda"), torch.tensor(B, device="cuda"), Cd, alpha=0.5, beta=-2.0,
                       transA=tA, transB=tB).cpu().numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12 * np.abs(want).max())


def test_gemm_f64_batched(ctx):
    r = np.random.default_rng(5)
    A = r.standard_normal((3, 150, 70)); B = r.standard_normal((3, 70, 90))
    got = ctx.gemm_f64(torch.tensor(A, device="cuda"), torch.tensor(B, device="cuda")).cpu().numpy()
    assert np.allclose(got, A @ B, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("n,batch", [(64, 1), (100, 3), (256, 2), (517, 1)])
def test_chol_inv_upper(ctx, n, batch):
    print("chol_inv_upper", n, batch, flush=True)
    r = np.random.default_rng(n)
    Hs = []
    for b in range(batch):
        A = r.standard_normal((n, 2 * n)) * (1.0 + 5.0 * (r.random(n) < 0.05))[:, None]
        Hs.append((A @ A.T).astype(np.float32))
    H = np.stack(Hs)
    U = ctx.chol_inv_upper(torch.tensor(H, device="cuda"), damp=0.01).cpu().numpy()
    for b in range(batch):
        want = O.chol_inv_upper(O.damp_hessian(H[b].astype(np.float64), 0.01))
        assert np.allclose(np.tril(U[b], -1), 0.0)
        assert np.allclose(U[b], want, rtol=1e-8, atol=1e-10 * np.abs(want).max())


def test_chol_inv_upper_rejects_indefinite(ctx, lib):
    H = torch.eye(70, device="cuda"); H[40, 40] = -1.0
    with pytest.raises(lib.TurboBoAError) as e:
        ctx.chol_inv_upper(H)
    assert e.value.code == -2 and "40" in str(e.value)


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (512, 768, 256), (300, 200, 72), (32, 40, 8), (1024, 1024, 1024)])
def test_gemm_bf16_nt(ctx, M, N, K):
    print("gemm_bf16_nt", M, N, K, flush=True)
    g = torch.Generator(device="cuda"); g.manual_seed(M + N + K)
    A = torch.randn(M, K, generator=g, device="cuda").to(torch.bfloat16)
    B = torch.randn(N, K, generator=g, device="cuda").to(torch.bfloat16)
    want = A.double().cpu().numpy() @ B.double().cpu().numpy().T
    got = ctx.gemm_bf16_nt(A, B, alpha=0.5).cpu().numpy()
    assert np.allclose(got, 0.5 * want, rtol=0, atol=1e-5 * np.sqrt(K) * 4)
    got16 = ctx.gemm_bf16_nt(A, B, out_dtype=torch.bfloat16).float().cpu().numpy()
    assert np.allclose(got16, want, rtol=2 ** -8, atol=1e-3)
    C0 = torch.ones(M, N, device="cuda")
    acc = ctx.gemm_bf16_nt(A, B, C_out=C0, accumulate=True).cpu().numpy()
    assert np.allclose(acc, want + 1.0, rtol=0, atol=1e-5 * np.sqrt(K) * 4)


@pytest.mark.parametrize("M,N,K,persistent", [(512, 768, 256, False), (300, 200, 72, False), (1024, 1280, 512, True)])
def test_gemm_f16_operands(ctx, lib, M, N, K, persistent):
    """The same kernels on IEEE half operands (TBOA_GEMM_F16): three kernels (register-staged for K = 72, LDS-direct,
    persistent), fp32 and 16-bit results, the blocked result layout."""
    print("gemm f16", M, N, K, persistent, flush=True)
    g = torch.Generator(device="cuda"); g.manual_seed(M + N + K)
    A = torch.randn(M, K, generator=g, device="cuda").to(torch.float16)
    B = torch.randn(N, K, generator=g, device="cuda").to(torch.float16)
    pf = lib.GEMM_PERSISTENT if persistent else 0
    want = A.double().cpu().numpy() @ B.double().cpu().numpy().T
    got = ctx.gemm_bf16_nt(A, B, alpha=0.5, flags=pf).cpu().numpy()
    assert np.allclose(got, 0.5 * want, rtol=0, atol=1e-5 * np.sqrt(K) * 4)
    got16 = ctx.gemm_bf16_nt(A, B, out_dtype=torch.float16, flags=pf)
    assert got16.dtype == torch.float16
    assert np.allclose(got16.float().cpu().numpy(), want, rtol=2 ** -11, atol=1e-3)
    # the products of half operands are exact in fp32 just as those of bf16 operands: same result as bf16 inputs that hold
    # the same values (small integers are exact in both)
    Ai = torch.randint(-8, 9, (M, K), generator=g, device="cuda").float(); Bi = torch.randint(-8, 9, (N, K), generator=g, device="cuda").float()
    assert torch.equal(ctx.gemm_bf16_nt(Ai.half(), Bi.half(), flags=pf), ctx.gemm_bf16_nt(Ai.bfloat16(), Bi.bfloat16(), flags=pf))
    if M % 256 == 0 and N % 256 == 0:
        Ct = ctx.gemm_bf16_nt(A, B, out_dtype=torch.float16, flags=lib.GEMM_C_TILED | pf)
        assert torch.equal(to_blocks(got16), Ct)


def test_gemm_bf16_flags_and_batch(ctx, lib):
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    n, K = 768, 512
    A = torch.randn(2, n, K, generator=g, device="cuda").to(torch.bfloat16)
    want = np.einsum("bik,bjk->bij", A.double().cpu().numpy(), A.double().cpu().numpy())
    low = ctx.gemm_bf16_nt(A, A, flags=lib.GEMM_LOWER).cpu().numpy()
    for b in range(2):
        assert np.allclose(np.tril(low[b]), np.tril(want[b]), atol=1e-3)
        assert np.all(low[b][:256, 512:] == 0)             # tiles above the diagonal are not touched
    # causal: B lower triangular [N, K] with K == N
    P = torch.tril(torch.rand(n, n, generator=g, device="cuda")).to(torch.bfloat16)
    Xt = torch.randn(300, n, generator=g, device="cuda").to(torch.bfloat16)
    want2 = Xt.double().cpu().numpy() @ P.double().cpu().numpy().T
    got2 = ctx.gemm_bf16_nt(Xt, P, flags=lib.GEMM_CAUSAL_K).cpu().numpy()
    assert np.allclose(got2, want2, atol=1e-3)


@pytest.mark.parametrize("M,N,K,batch,flags", [
    (256, 256, 128, 1, 0),            # one tile, one ring fill
    (700, 900, 384, 3, 0),            # ragged edges, fewer tiles than compute units
    (2304, 2048, 256, 5, 0),          # 360 tiles: several rounds per workgroup, short tiles back to back
    (1280, 1280, 512, 9, 1),          # symmetric product, lower tiles only
    (520, 1536, 1536, 7, 2),          # causal limit: tiles of 8 different lengths, balanced lists
    (128, 1536, 1536, 12, 2),         # results of 128 rows (an attention output of one head): the lower half of every tile idles
    (96, 700, 640, 5, 0),             # ... fewer rows than that, ragged columns
    (64, 512, 256, 300, 0),           # ... many batch entries: several tiles per workgroup
])
def test_gemm_bf16_persistent_matches_dispatched(ctx, lib, M, N, K, batch, flags):
    """The persistent kernel (one resident workgroup per compute unit, one stream of stages across tiles) accumulates every
    tile in the same order as the dispatched one: identical bits; both against fp64 on sampled entries."""
    print("gemm_bf16 persistent", M, N, K, batch, flags, flush=True)
    g = torch.Generator(device="cuda"); g.manual_seed(M + N + K + batch)
    A = torch.randn(batch, M, K, generator=g, device="cuda").to(torch.bfloat16)
    B = torch.randn(batch, N, K, generator=g, device="cuda").to(torch.bfloat16)
    if flags & lib.GEMM_LOWER:
        B = A
    if flags & lib.GEMM_CAUSAL_K:
        B = torch.tril(B)
    for accumulate in (False, True):
        C0 = torch.full((batch, M, N), 0.25, device="cuda")
        want = ctx.gemm_bf16_nt(A, B, C_out=C0.clone(), accumulate=accumulate, flags=flags)
        got = ctx.gemm_bf16_nt(A, B, C_out=C0.clone(), accumulate=accumulate, flags=flags | lib.GEMM_PERSISTENT)
        assert torch.equal(got, want)
    got16 = ctx.gemm_bf16_nt(A, B, out_dtype=torch.bfloat16, flags=flags | lib.GEMM_PERSISTENT)
    want16 = ctx.gemm_bf16_nt(A, B, out_dtype=torch.bfloat16, flags=flags)
    assert torch.equal(got16, want16)
    r = np.random.default_rng(0)
    for _ in range(200):
        b, i, j = r.integers(batch), r.integers(M), r.integers(N)
        if (flags & lib.GEMM_LOWER) and j // 256 > i // 256:
            continue
        ref = float(A[b, i].double() @ B[b, j].double())
        assert abs(float(got[b, i, j]) - 0.25 - ref) <= 1e-5 * np.sqrt(K) * 4 + 1e-6 * abs(ref)


def to_blocks(M):
    """Row-major [R, K] -> the 16 x 32 block layout of TBOA_GEMM_*_TILED (an index permutation, written from the header)."""
    R, K = M.shape
    r = torch.arange(R, device=M.device)[:, None]; c = torch.arange(K, device=M.device)[None, :]
    off = ((r // 16) * (K // 32) + c // 32) * 512 + (r % 16) * 32 + (((c % 32) // 8) ^ (((r % 16) // 4) % 4)) * 8 + c % 8
    out = torch.empty(R * K, dtype=M.dtype, device=M.device)
    out[off.reshape(-1)] = M.reshape(-1)
    return out.reshape(R, K)


def from_blocks(T):
    R, K = T.shape
    r = torch.arange(R, device=T.device)[:, None]; c = torch.arange(K, device=T.device)[None, :]
    off = ((r // 16) * (K // 32) + c // 32) * 512 + (r % 16) * 32 + (((c % 32) // 8) ^ (((r % 16) // 4) % 4)) * 8 + c % 8
    return T.reshape(-1)[off.reshape(-1)].reshape(R, K)


@pytest.mark.parametrize("persistent", [False, True])
def test_gemm_bf16_blocked_layouts(ctx, lib, persistent):
    """Operands and result in 16 x 32 blocks: same bits as the row-major call, for ragged operand tiles, a batch, a
    symmetric product and a chain (the blocked bf16 result of one product read as the operand of the next)."""
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    pf = lib.GEMM_PERSISTENT if persistent else 0
    M, N, K = 528, 784, 448          # 16 | M, N; 32 | K; neither a multiple of 256
    A = torch.randn(2, M, K, generator=g, device="cuda").to(torch.bfloat16)
    B = torch.randn(2, N, K, generator=g, device="cuda").to(torch.bfloat16)
    At = torch.stack([to_blocks(a) for a in A]); Bt = torch.stack([to_blocks(b) for b in B])
    want = ctx.gemm_bf16_nt(A, B)
    assert torch.equal(ctx.gemm_bf16_nt(At, B, flags=lib.GEMM_A_TILED | pf), want)
    assert torch.equal(ctx.gemm_bf16_nt(A, Bt, flags=lib.GEMM_B_TILED | pf), want)
    assert torch.equal(ctx.gemm_bf16_nt(At, Bt, flags=lib.GEMM_A_TILED | lib.GEMM_B_TILED | pf), want)
    low = ctx.gemm_bf16_nt(A[:, :512], A[:, :512], flags=lib.GEMM_LOWER)
    assert torch.equal(ctx.gemm_bf16_nt(At[:, :512], At[:, :512], flags=lib.GEMM_LOWER | lib.GEMM_A_TILED | lib.GEMM_B_TILED), low)
    # blocked result: M, N multiples of 256
    X = torch.randn(512, 320, generator=g, device="cuda").to(torch.bfloat16)
    Y = torch.randn(768, 320, generator=g, device="cuda").to(torch.bfloat16)
    C = ctx.gemm_bf16_nt(X, Y, out_dtype=torch.bfloat16, alpha=0.5, flags=pf)
    Ct = ctx.gemm_bf16_nt(X, Y, out_dtype=torch.bfloat16, alpha=0.5, flags=lib.GEMM_C_TILED | pf)
    assert torch.equal(from_blocks(Ct), C)
    # chain: (X Y^T) as the blocked left operand of the next product, K = 768
    Z = torch.randn(256, 768, generator=g, device="cuda").to(torch.bfloat16)
    assert torch.equal(ctx.gemm_bf16_nt(Ct, Z, flags=lib.GEMM_A_TILED), ctx.gemm_bf16_nt(C, Z))
    with pytest.raises(lib.TurboBoAError):
        ctx.gemm_bf16_nt(X[:500], Y, out_dtype=torch.bfloat16, flags=lib.GEMM_C_TILED)      # M not a multiple of 256
