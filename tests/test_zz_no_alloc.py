"""The entry point that allocates nothing (tboa_chol_inv_upper_static) against the entry point it is a variant of, through
the C-ABI, on two calls in a row, the second one smaller (GPU)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def spd_batch(batch, n, seed):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    A = torch.randn(batch, n, 3 * n, generator=g, device="cuda", dtype=torch.float64)
    return (A @ A.transpose(1, 2)).float().contiguous()


def test_static_scratch_matches_workspace_entry_point(lib):
    ctx = lib.Context()
    try:
        cases = [(64, 128, 1), (5, 200, 2), (3, 72, 3), (1, 512, 4), (7, 17, 5)]      # the second and later calls are smaller or ragged
        outs = [torch.empty(b, n, n, dtype=torch.float64, device="cuda") for b, n, _ in cases]      # allocated before any call
        Hs = [spd_batch(b, n, seed) for b, n, seed in cases]
        torch.cuda.synchronize()
        for (b, n, _), H, U in zip(cases, Hs, outs):
            print("static chol_inv_upper: batch %d, n %d" % (b, n), flush=True)
            ctx.chol_inv_upper(H, damp=0.01, out=U, static=True)
            want = ctx.chol_inv_upper(H, damp=0.01)
            # same kernels, same order of operations: identical bits
            assert torch.equal(U, want), (b, n, (U - want).abs().max().item())
            # and it is the factor: U^T U H = I (fp64 route on the host for the first matrix)
            Hd = H[0].double().cpu().numpy(); Hd = Hd + 0.01 * np.mean(np.diag(Hd)) * np.eye(n)
            U0 = U[0].cpu().numpy()
            assert np.allclose(U0.T @ U0 @ Hd, np.eye(n), atol=1e-6)
            assert np.allclose(np.tril(U0, -1), 0.0)
        # beyond the static scratch: refused with a message, nothing touched
        for b, n in ((65, 128), (1, 513), (5, 512)):
            with pytest.raises(lib.TurboBoAError) as e:
                ctx.chol_inv_upper(spd_batch(1, 8, 9).expand(b, 8, 8).contiguous() if False else torch.zeros(b, n, n, device="cuda"), static=True)
            assert e.value.code == -1 and "static scratch" in str(e.value)
        # a breakdown is still reported, and the next call works
        bad = spd_batch(2, 64, 6); bad[1, 5, :] = 0; bad[1, :, 5] = 0
        with pytest.raises(lib.TurboBoAError) as e:
            ctx.chol_inv_upper(bad, static=True)
        assert e.value.code == -2
        again = torch.empty_like(outs[0])
        ctx.chol_inv_upper(Hs[0], damp=0.01, out=again, static=True)
        assert torch.equal(again, outs[0])
    finally:
        ctx.close()
