"""Seeded random shapes: every call of the library against the float64 definitions in oracle/, at
sizes drawn from ranges that straddle the kernels' tile edges (the fixed lists of the other test
files were chosen by hand; these are not).  Inputs are well conditioned on purpose, so the
tolerances are the ones stated in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref
from test_gpu_parity import NEAR_TIE, _structured_H, dev, h_tol

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2501_12956_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def _draw_n(rng, top):
    return int(rng.choice([int(rng.integers(1, 130)), int(rng.integers(130, 700)), int(rng.integers(700, top))]))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_S_and_T_updates(ctx, seed):
    rng = np.random.default_rng(seed)
    for case in range(16):
        nbits = int(rng.integers(1, 5))
        m = int(rng.integers(1, 200))
        n = _draw_n(rng, 1700)
        kind = str(rng.choice(["weak", "medium", "wide", "mixed", "dead"]))
        if kind == "dead" and n < 3:
            kind = "weak"
        # enough columns per code that the per-row systems are well conditioned (with feature
        # scales over five decades a group of two or three columns is not)
        need = 32 if kind == "wide" else 8
        while nbits > 1 and n < need << nbits:
            nbits -= 1
        label = "seed %d case %d: %dx%d N=%d %s" % (seed, case, m, n, nbits, kind)
        H32 = _structured_H(kind, n, int(rng.integers(1 << 30)))
        W = (rng.standard_normal((m, n)) * 0.02).astype(np.float32)
        # codes as an assignment step leaves them: every weight at its nearest quantile code
        # (random codes would make every codebook entry a mean of zero-mean noise, all cancellation)
        Tq = ref.init_codebooks(W, nbits)
        Q = np.abs(W[:, :, None].astype(np.float64) - Tq[:, None, :]).argmin(axis=2).astype(np.uint8)
        Tg = ctx.update_T(dev(W), dev(H32), dev(Q), dev(np.zeros((m, 1 << nbits), np.float32)), nbits)
        Tref, _ = ref.update_T(W.astype(np.float64), H32.astype(np.float64), Q, nbits)
        err = np.abs(Tg.cpu().numpy() - Tref).max(axis=1) / np.maximum(np.abs(Tref).max(axis=1), 1e-300)
        if n >= need << nbits:
            assert np.all(err <= 1e-4), (label, float(err.max()))
        # S-update on a factor of the same matrix (regularised: one feature may be dead)
        H64 = H32.astype(np.float64) + 1e-3 * np.mean(np.diag(H32)) * np.eye(n)
        L32 = np.linalg.cholesky(H64).astype(np.float32)
        T32 = np.sort(rng.standard_normal((m, 1 << nbits)) * 0.02, axis=1).astype(np.float32)
        Qg = ctx.update_S(dev(W), dev(L32), dev(T32), nbits).cpu().numpy()
        _, gap, _ = ref.s_update_targets(W.astype(np.float64), L32.astype(np.float64), T32.astype(np.float64), Qg)
        rel = gap / np.abs(T32.astype(np.float64)).max(axis=1)[:, None]
        assert int((rel >= NEAR_TIE).sum()) == 0, label


@pytest.mark.parametrize("seed", [1, 2])
def test_random_other_calls(ctx, seed):
    from paper_2501_12956_amd import binding as b
    rng = np.random.default_rng(100 + seed)
    for case in range(12):
        n = _draw_n(rng, 900)
        p = int(rng.integers(1, 3000))
        p8 = (p + 7) // 8 * 8
        label = "seed %d case %d: n=%d p=%d" % (seed, case, n, p)
        X = torch.from_numpy(rng.standard_normal((n, p8)).astype(np.float32))
        X[int(rng.integers(0, n))] *= 15.0
        Xh = X.half()

        def h_err(H, Href):
            d = np.sqrt(np.diag(Href))
            return float((np.abs(H - Href) / (np.outer(d, d) + 1e-300)).max())

        Href = ref.build_hessian(Xh.numpy())
        H = ctx.build_hessian(Xh.cuda()).cpu().numpy().astype(np.float64)
        assert h_err(H, Href) <= h_tol(p8) and np.array_equal(H, H.T), label
        Ht = ctx.build_hessian_tokens(Xh[:, :p].t().contiguous().cuda()).cpu().numpy().astype(np.float64)
        assert h_err(Ht, ref.build_hessian(Xh[:, :p].numpy())) <= h_tol(p) and np.array_equal(Ht, Ht.T), label
        Hf = ctx.build_hessian(X[:, :p].contiguous().cuda()).cpu().numpy().astype(np.float64)
        assert h_err(Hf, ref.build_hessian(X[:, :p].numpy())) <= h_tol(p, True), label     # fp32 products are rounded

        H32 = (Href + 0.05 * np.mean(np.diag(Href)) * np.eye(n)).astype(np.float32)
        H64 = H32.astype(np.float64)
        L, info = ctx.cholesky(dev(H32))
        L = L.cpu().numpy().astype(np.float64)
        Lref, _ = ref.cholesky(H64)
        assert info == 0 and np.array_equal(L, np.tril(L)), label
        assert np.linalg.norm(L @ L.T - H64) <= 2e-6 * np.linalg.norm(H64), label
        assert np.linalg.norm(L - Lref) <= 1e-4 * np.linalg.norm(Lref), label

        m = int(rng.integers(1, 150))
        nbits = int(rng.integers(1, 5))
        W = (rng.standard_t(5, size=(m, n)) * 0.02).astype(np.float32)
        for mode, omode in [(b.INIT_QUANTILE_MID, ref.INIT_QUANTILE_MID), (b.INIT_MINMAX_GRID, ref.INIT_MINMAX_GRID)]:
            T = ctx.init_codebooks(dev(W), nbits, mode).cpu().numpy()
            Tref = ref.init_codebooks(W, nbits, omode)
            ulp = np.spacing(np.abs(Tref).astype(np.float32)).astype(np.float64)
            assert np.all(np.abs(T - Tref) <= ulp), label
        Q = rng.integers(0, 1 << nbits, size=(m, n)).astype(np.uint8)
        loss = ctx.layer_loss(dev(W), dev(H32), dev(T), dev(Q), nbits)
        lref, _ = ref.layer_loss(W.astype(np.float64), H64, T.astype(np.float64), Q)
        assert abs(loss - lref) <= 1e-4 * lref, label
        r = float(rng.choice([0.0, 0.005, 0.05, 0.3]))
        Wd = ctx.outlier_split(dev(W), r)[0].cpu().numpy().astype(np.float64)
        assert np.array_equal(Wd, ref.outlier_split(W.astype(np.float64), r)[1]), label

        x = rng.standard_normal(n).astype(np.float16)
        packed, lut = ctx.pack_layer(dev(Q), dev(np.sort(T, axis=1)), nbits)
        Pref = ref.pack_codes(Q, nbits)
        assert np.array_equal(packed.cpu().numpy()[:, :Pref.shape[1]], Pref), label
        y = ctx.lut_gemv(packed, lut, nbits, n, dev(x)).cpu().numpy().astype(np.float64)
        L16 = lut.cpu().numpy()
        mag = np.abs(ref.dequantize(L16.astype(np.float64), Q)) @ np.abs(x.astype(np.float64))
        assert np.all(np.abs(y - ref.lut_matvec(L16, Q, x)) <= 64 * 2.0 ** -24 * mag + 1e-30), label
