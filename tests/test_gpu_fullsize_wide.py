"""GPU parity at full size for the other layer shapes of the workload list: the 3-bit
4096 x 4096 layer, the LLaMA-7B up_proj- and down_proj-shaped layers (11008 x 4096; 4096 x 11008
with heavy-tailed activations and outlier channels) and the Llama-3-70B down_proj-shaped layer
(8192 x 28672, 3.3 GB H and L).

Nothing here can be checked whole by the float64 oracle in seconds, so every call is checked
on what the oracle computes one by one, or on a property that holds at any size:
  H       - sampled entries against float64 dot products over all tokens; exact symmetry;
  L       - its leading principal block equals the Cholesky factor of H's leading block
            (LAPACK, float64), and L (L^T v) = H v for random probe vectors (the products are
            formed in float64 on the host from row blocks, so no library GEMM is trusted);
  S, T, loss on a seeded sample of rows with the full H and L in float64 (rows of the layer
            are independent), to the tolerances of test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref
from paper_2501_12956_amd import synth

pytestmark = pytest.mark.gpu

NEAR_TIE = 1e-6


def h_tol(p):
    return max(2e-6, 5.0 * 2.0 ** -24 * np.sqrt(p / 3.0))


def run_layer(name, rows_s, rows_t):
    from paper_2501_12956_amd import binding
    cfg = synth.CONFIGS[name]
    dev = "cuda:0"
    W = synth.make_weight(cfg, 0, dev)
    X = synth.make_activations(cfg, 0, dev)
    n, m, nbits = cfg.n, cfg.m, cfg.nbits
    ctx = binding.Context(0)
    try:
        ctx.reserve(m, n, cfg.p, nbits)
        H = ctx.build_hessian(X)

        # --- H: sampled entries (include scaled channels), symmetry
        rng = np.random.default_rng(11)
        idx = np.unique(np.concatenate([rng.choice(n, size=16, replace=False),
                                        synth.outlier_feature_rows(cfg, 0).numpy()[:4]]))
        it = torch.from_numpy(idx).to(dev)
        Xs = X[it].cpu().numpy().astype(np.float64)
        Href = Xs @ Xs.T
        Hs = H[it][:, it].cpu().numpy().astype(np.float64)
        d = np.sqrt(np.diag(Href))
        rel = float((np.abs(Hs - Href) / np.outer(d, d)).max())
        print("%s H: max |dH|/sqrt(HjjHkk) = %.2e (tol %.2e)" % (name, rel, h_tol(cfg.p)))
        assert rel <= h_tol(cfg.p)
        del X, Xs
        torch.cuda.empty_cache()
        H64 = H.cpu().numpy().astype(np.float64)
        assert np.array_equal(H64, H64.T)

        # --- L
        L, info = ctx.cholesky(H)
        assert info == 0
        L64 = L.cpu().numpy().astype(np.float64)
        assert np.all(np.diag(L64) > 0)
        assert not np.any(np.triu(L64[:2048, :2048], 1)) and not np.any(L64[0, 1:])
        nb = 1024
        Lref = np.linalg.cholesky(H64[:nb, :nb])
        r_lead = np.linalg.norm(L64[:nb, :nb] - Lref) / np.linalg.norm(Lref)
        V = rng.standard_normal((n, 3))
        LtV = np.zeros_like(V)
        LLtV = np.zeros_like(V)
        HV = np.zeros_like(V)
        blk = 2048
        for a in range(0, n, blk):                      # L^T V, accumulated by row blocks of L
            LtV += L64[a:a + blk].T @ V[a:a + blk]
        for a in range(0, n, blk):
            LLtV[a:a + blk] = L64[a:a + blk] @ LtV
            HV[a:a + blk] = H64[a:a + blk] @ V
        r_probe = np.linalg.norm(LLtV - HV) / np.linalg.norm(HV)
        print("%s L: leading %d block |L-Lref|/|Lref| = %.2e, probe |LL^Tv-Hv|/|Hv| = %.2e"
              % (name, nb, r_lead, r_probe))
        assert r_lead <= 1e-4 and r_probe <= 2e-6

        # --- T^0 on sampled rows, 1 ulp
        Wf = W.float()
        rows = np.sort(rng.choice(m, size=max(rows_s, rows_t), replace=False))
        rt = torch.from_numpy(rows).to(dev)
        Ws = Wf[rt].cpu().numpy().astype(np.float64)
        T0 = ctx.init_codebooks(W, nbits)
        T0s = T0[rt].cpu().numpy().astype(np.float64)
        T0ref = ref.init_codebooks(Ws, nbits)
        ulp = np.spacing(np.abs(T0ref).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(T0s - T0ref) <= ulp)

        # --- one S-update: every choice optimal for its float64 teacher-forced target
        Q = ctx.update_S(Wf, L, T0, nbits)
        Qs = Q[rt].cpu().numpy()
        _, gap, _ = ref.s_update_targets(Ws[:rows_s], L64, T0s[:rows_s], Qs[:rows_s])
        relgap = gap / np.abs(T0s[:rows_s]).max(axis=1)[:, None]
        viol = int((relgap >= NEAR_TIE).sum())
        print("%s S-update on %d rows: optimal %.6f, near ties %d, violations %d"
              % (name, rows_s, float((gap == 0).mean()), int(((gap > 0) & (relgap < NEAR_TIE)).sum()), viol))
        assert viol == 0

        # --- one T-update and the loss on the GPU's Q
        T1 = ctx.update_T(Wf, H, Q, T0.clone(), nbits)
        T1s = T1[rt].cpu().numpy().astype(np.float64)
        T1ref, _ = ref.update_T(Ws[:rows_t], H64, Qs[:rows_t], nbits)
        err = np.abs(T1s[:rows_t] - T1ref).max(axis=1) / np.abs(T1ref).max(axis=1)
        print("%s T-update on %d rows: max row error %.2e" % (name, rows_t, err.max()))
        assert err.max() <= 1e-4
        loss, rl = ctx.layer_loss(Wf, H, T1, Q, nbits, want_rows=True)
        _, rref = ref.layer_loss(Ws[:rows_t], H64, T1s[:rows_t], Qs[:rows_t])
        rls = rl[rt].cpu().numpy()[:rows_t]
        assert np.all(np.abs(rls - rref) <= 1e-4 * rref)
        assert abs(loss - float(rl.double().sum())) <= 1e-6 * loss
        loss0, _ = ctx.layer_loss(Wf, H, T0, Q, nbits, want_rows=True)
        assert loss <= loss0 * (1 + 1e-5)               # the T-update cannot raise the objective
        print("%s loss after S-update %.6e, after T-update %.6e" % (name, loss0, loss))
    finally:
        ctx.close()


def test_q_proj_3bit_full_size():
    run_layer("c2", rows_s=32, rows_t=16)


def test_up_proj_7b_full_size():
    run_layer("c4a", rows_s=32, rows_t=16)


def test_down_proj_7b_full_size():
    run_layer("c4b", rows_s=32, rows_t=16)


def test_down_proj_70b_full_size():
    run_layer("c5", rows_s=16, rows_t=8)
