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


@pytest.mark.parametrize("M,N,K", [(128, 128, 16), (256, 384, 64), (77, 131, 45), (1, 5, 3), (300, 64, 1000)])
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
