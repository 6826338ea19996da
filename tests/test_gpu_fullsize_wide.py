"""GPU parity at full size for the other layer shapes of the workload list: the 3-bit
4096 x 4096 layer, the LLaMA-7B up_proj- and down_proj-shaped layers (11008 x 4096; 4096 x 11008
with heavy-tailed activations and outlier channels) and the Llama-3-70B down_proj-shaped layer
(8192 x 28672, 3.3 GB H and L; at 4 and at 3 bits on the same H and L).

Nothing here can be checked whole by the float64 oracle in seconds, so every call is checked
on what the oracle computes one by one, or on a property that holds at any size:
  H       - sampled entries against float64 dot products over all tokens; exact symmetry;
  L       - its leading principal block equals the Cholesky factor of H's leading block
            (LAPACK, float64), and L (L^T v) = H v for random probe vectors (the products are
            formed in float64 on the host from row blocks, so no library GEMM is trusted);
  S, T, loss on a seeded sample of rows with the full H and L in float64 (rows of the layer
            are independent), to the tolerances of test_gpu_parity.py;
  Algorithm 1 - all K alternations through ganq_quantize_layer with the factorisation done inside
            the call (the path with the second stream), on the same sampled rows: the last
            sweep's choices are optimal for their float64 targets built from T^{K-1}, T^K is the
            least-squares refit to Q^K, the loss equals the oracle's, K sweeps in one call equal
            K - 1 sweeps plus one more call bit for bit, and the oracle's own K sweeps from the
            same T^0 reach the same loss on those rows (index agreement reported).
"""
import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref
from paper_2501_12956_amd import synth

pytestmark = pytest.mark.gpu

NEAR_TIE = 1e-6


def h_tol(p, heavy=False):
    """|dH_jk| / sqrt(H_jj H_kk): the fp32 sums of the product kernel run over at most p / 16 tokens per
    partial and the partials are added pairwise, so the error grows far more slowly than a running sum's
    eps sqrt(p / 3); the factor is set about ten times above what the workloads measure (5e-7 on
    Gaussian activations at p = 262144, 4e-6 on the heavy-tailed ones at p = 131072, whose fp16 values
    reach 475 and cancel in the sums)."""
    return max(2e-6, (2.5 if heavy else 0.35) * 2.0 ** -24 * np.sqrt(p / 3.0))


def run_layer(name, rows_s, rows_t, bit_widths=None, free_rows=4):
    from paper_2501_12956_amd import binding
    cfg = synth.CONFIGS[name]
    dev = "cuda:0"
    W = synth.make_weight(cfg, 0, dev)
    X = synth.make_activations(cfg, 0, dev)
    n, m = cfg.n, cfg.m
    bit_widths = list(bit_widths or [cfg.nbits])
    ctx = binding.Context(0)
    try:
        ctx.reserve(m, n, cfg.p, max(bit_widths))
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
        heavy = cfg.x_kind == "heavy"
        print("%s H: max |dH|/sqrt(HjjHkk) = %.2e (tol %.2e)" % (name, rel, h_tol(cfg.p, heavy)))
        assert rel <= h_tol(cfg.p, heavy)
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

        Wf = W.float()
        rows = np.sort(rng.choice(m, size=max(rows_s, rows_t), replace=False))
        rt = torch.from_numpy(rows).to(dev)
        Ws = Wf[rt].cpu().numpy().astype(np.float64)
        for nbits in bit_widths:
            solver_checks(ctx, "%s/%d bit" % (name, nbits), cfg, nbits, W, Wf, H, L, H64, L64, rows, rt, Ws,
                          rows_s, rows_t, free_rows)
    finally:
        ctx.close()


def solver_checks(ctx, name, cfg, nbits, W, Wf, H, L, H64, L64, rows, rt, Ws, rows_s, rows_t, free_rows):
    # --- T^0 on sampled rows, 1 ulp
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
    del Q, T1

    # --- Algorithm 1: K alternations in one call that factors H itself (fp16 W, T^0 built inside)
    K = cfg.iters
    TK, QK = ctx.quantize_layer(W, H, nbits, K)
    Tprev, _ = ctx.quantize_layer(W, H, nbits, K - 1)
    Tr, Qr = ctx.quantize_layer(W, H, nbits, 1, T=Tprev.clone())
    # K = (K - 1) + 1: the same Q^K bit for bit; T^K agrees to rounding (the one-call run may have
    # updated S_i H S_i^T in its last sweep, the restarted one sums it afresh)
    assert torch.equal(Qr, QK)
    dT = (Tr - TK).abs().amax(dim=1) / TK.abs().amax(dim=1)
    assert float(dT.max()) <= 1e-5
    QKs = QK[rt].cpu().numpy()
    Tps = Tprev[rt].cpu().numpy().astype(np.float64)
    TKs = TK[rt].cpu().numpy().astype(np.float64)
    _, gap, _ = ref.s_update_targets(Ws[:rows_s], L64, Tps[:rows_s], QKs[:rows_s])
    relgap = gap / np.abs(Tps[:rows_s]).max(axis=1)[:, None]
    viol = int((relgap >= NEAR_TIE).sum())
    TKref, cnt = ref.update_T(Ws[:rows_t], H64, QKs[:rows_t], nbits)
    err = np.abs(TKs[:rows_t] - TKref).max(axis=1) / np.abs(TKref).max(axis=1)
    lossK, rlK = ctx.layer_loss(Wf, H, TK, QK, nbits, want_rows=True)
    _, rref = ref.layer_loss(Ws[:rows_t], H64, TKs[:rows_t], QKs[:rows_t])
    rls = rlK[rt].cpu().numpy()[:rows_t]
    print("%s K=%d in one call: last sweep optimal %.6f, violations %d; T^K max row error %.2e "
          "(unused codes on the sampled rows: %d); layer loss %.6e"
          % (name, K, float((gap == 0).mean()), viol, err.max(), int(cnt.sum()), lossK))
    assert viol == 0
    assert err.max() <= 1e-4
    assert np.all(np.abs(rls - rref) <= 1e-4 * rref)
    assert lossK < loss0
    # the oracle's own K sweeps on a few of the rows (free-running; reported, loose gate on the loss)
    if free_rows > 0:
        # (column-major copy of L: the oracle reads one column of L per step)
        To, Qo = ref.quantize_layer(Ws[:free_rows], H64, T0s[:free_rows], nbits, K, L=np.asfortranarray(L64))
        lo = ref.layer_loss(Ws[:free_rows], H64, To, Qo)[0]
        lg = float(rref[:free_rows].sum()) if free_rows <= rows_t else None
        agree = float((QKs[:free_rows] == Qo).mean())
        print("%s free-running oracle on %d rows: loss %.6e, GPU %.6e, index agreement %.6f"
              % (name, free_rows, lo, lg, agree))
        assert abs(lg - lo) <= 2e-2 * lo


def test_q_proj_3bit_full_size():
    run_layer("c2", rows_s=32, rows_t=16)


def test_up_proj_7b_full_size():
    run_layer("c4a", rows_s=32, rows_t=16)


def test_down_proj_7b_full_size():
    run_layer("c4b", rows_s=32, rows_t=16)


def test_down_proj_70b_full_size_4bit_and_3bit():
    run_layer("c5", rows_s=16, rows_t=8, bit_widths=[4, 3], free_rows=0)
