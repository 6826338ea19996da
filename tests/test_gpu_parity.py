"""GPU parity: every C-ABI call against the float64 CPU oracle on the same seeded
inputs, stage by stage (each call of the two implementations is fed identical
inputs), plus the degenerate cases.  Sizes span several tiles and a ragged tail
while staying small enough for the oracle to finish in seconds.

Tolerances (derived from the arithmetic of the kernels):
  H        |dH_jk| <= h_tol(p) sqrt(H_jj H_kk), h_tol = max(2e-6, 0.35 eps sqrt(p/3)) (2.5 for heavy tails): fp32
           sums of p products (sequential accumulation error, 4.5 sigma over n^2 entries)
  L        |L L^T - H|_F <= 2e-6 |H|_F, |L - L_ref|_F <= 1e-4 |L_ref|_F
  T^0      1 ulp of fp32
  Q        every choice optimal for its float64 teacher-forced target, or a near tie
           (gap / max|T_i| < 1e-6); agreement fraction with the oracle's own sweep reported
  T        per row |dT|_inf <= 1e-4 |T|_inf
  loss     1e-4 relative
"""
import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref
from paper_2501_12956_amd import synth

pytestmark = pytest.mark.gpu

NEAR_TIE = 1e-6


@pytest.fixture(scope="module")
def ctx():
    from paper_2501_12956_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def make_problem(m, n, p, nbits, seed=0, x_dtype=torch.float16, w_kind="student_t"):
    base = synth.CONFIGS["c3"] if w_kind == "student_t" else synth.CONFIGS["c1"]
    if x_dtype == torch.float16:  # fp16 activations need a leading dimension that is a multiple of 8
        p = (p + 7) // 8 * 8
    cfg = synth.scaled_config(base, m=m, n=n, p=p, nbits=nbits)
    W = synth.make_weight(cfg, seed).float()
    X = synth.make_activations(cfg, seed).to(x_dtype)
    return W, X


def h_tol(p, heavy=False):
    """|dH_jk| / sqrt(H_jj H_kk): the fp32 sums of the product kernel run over at most p / 16 tokens per
    partial and the partials are added pairwise, so the error grows far more slowly than a running sum's
    eps sqrt(p / 3); the factor is set about ten times above what the workloads measure (5e-7 on
    Gaussian activations at p = 262144, 4e-6 on the heavy-tailed ones at p = 131072, whose fp16 values
    reach 475 and cancel in the sums)."""
    return max(2e-6, (2.5 if heavy else 0.35) * 2.0 ** -24 * np.sqrt(p / 3.0))


def check_H(H, Href, p, label="", wide=False):
    """wide: fp32 activations (their products are rounded, fp16 products are exact in fp32) or
    heavy-tailed ones."""
    d = np.sqrt(np.diag(Href))
    rel = np.abs(H - Href) / (np.outer(d, d) + 1e-300)
    print("%s H: max |dH|/sqrt(HjjHkk) = %.2e (tol %.2e)" % (label, rel.max(), h_tol(p, wide)))
    assert rel.max() <= h_tol(p, wide)


def check_S(W64, L64, T64, Q_gpu, label=""):
    """Teacher-forced check of a GPU assignment; returns stats."""
    tgt, gap, best = ref.s_update_targets(W64, L64, T64, Q_gpu)
    scale = np.abs(T64).max(axis=1)[:, None]
    rel = gap / scale
    exact = float((gap == 0).mean())
    near = int(((gap > 0) & (rel < NEAR_TIE)).sum())
    viol = int((rel >= NEAR_TIE).sum())
    print("%s teacher-forced: optimal %.6f, near ties %d, violations %d" % (label, exact, near, viol))
    return exact, near, viol


# ----------------------------------------------------------------------------- H
@pytest.mark.parametrize("n,p", [(300, 1096), (128, 64), (130, 8)])
def test_hessian_fp16(ctx, n, p):
    _, X = make_problem(4, n, p, 4)
    Xg = X.cuda()
    H = ctx.build_hessian(Xg).cpu().numpy().astype(np.float64)
    Href = ref.build_hessian(X.numpy())
    check_H(H, Href, p, "fp16 n=%d p=%d" % (n, p))
    assert np.array_equal(H, H.T)
    # streaming: two token chunks accumulate to the same matrix
    if p >= 16:
        half = (p // 2) // 8 * 8
        H2 = ctx.build_hessian(Xg[:, :half].contiguous())
        H2 = ctx.build_hessian(Xg[:, half:].contiguous(), H=H2, accumulate=True).cpu().numpy()
        check_H(H2, Href, p, "fp16 two chunks")


def test_hessian_fp32_and_strided(ctx):
    _, X = make_problem(4, 200, 515, 4, x_dtype=torch.float32, w_kind="gauss_outlier")
    Xg = X.cuda()
    H = ctx.build_hessian(Xg).cpu().numpy().astype(np.float64)
    Href = ref.build_hessian(X.numpy())
    check_H(H, Href, 515, "fp32")
    # a view with a leading dimension larger than p
    big = torch.zeros(200, 600, dtype=torch.float32, device="cuda")
    big[:, :515] = Xg
    Hv = ctx.build_hessian(big[:, :515]).cpu().numpy()
    assert np.array_equal(Hv, H.astype(np.float32))


@pytest.mark.parametrize("n,p,dtype", [(300, 1093, torch.float16), (130, 5, torch.float16),
                                       (200, 515, torch.float32),
                                       # n % 8 == 0 and aligned rows: the product reads Xt as it is
                                       # (transposing LDS reads), no transposed copy; several feature
                                       # blocks with a ragged last one, fewer tokens than one stage,
                                       # token counts that are no multiple of anything
                                       (304, 1093, torch.float16), (520, 2500, torch.float16),
                                       (256, 37, torch.float16), (1032, 777, torch.float16),
                                       (64, 20011, torch.float16),
                                       # more than 2^22 tokens with room to transpose them all at once: the
                                       # fp16 product takes chunks whose leading dimension stays below 2^22
                                       (8, (1 << 22) + 4104, torch.float16)])
def test_hessian_token_major(ctx, n, p, dtype):
    """Activations stored tokens x features (how calibration batches arrive): H = Xt^T Xt, any
    token count, chunks accumulated; the oracle is the same float64 X X^T."""
    g = torch.Generator().manual_seed(21)
    Xt = torch.randn(p, n, generator=g).to(dtype)
    Xt[:, 3] *= 20.0
    Href = ref.build_hessian(Xt.numpy().astype(np.float64).T)
    Xg = Xt.cuda()
    H = ctx.build_hessian_tokens(Xg).cpu().numpy().astype(np.float64)
    check_H(H, Href, p, "token-major %s n=%d p=%d" % (str(dtype), n, p))
    assert np.array_equal(H, H.T)
    if 16 <= p < 100000:
        cut = p // 3
        H2 = ctx.build_hessian_tokens(Xg[:cut])
        H2 = ctx.build_hessian_tokens(Xg[cut:], H=H2, accumulate=True).cpu().numpy().astype(np.float64)
        check_H(H2, Href, p, "token-major two chunks")
        # a strided view (leading dimension larger than n)
        big = torch.zeros(p, n + 24, dtype=dtype, device="cuda")
        big[:, :n] = Xg
        Hv = ctx.build_hessian_tokens(big[:, :n]).cpu().numpy().astype(np.float64)
        assert np.array_equal(Hv, H)


# ----------------------------------------------------------------------------- L
@pytest.mark.parametrize("n", [200, 64, 65, 1, 300, 523, 1000, 777, 1288])
def test_cholesky(ctx, n):
    _, X = make_problem(4, n, max(4 * n, 64), 4, x_dtype=torch.float32, w_kind="gauss_outlier")
    H32 = (X @ X.T).contiguous()
    L, info = ctx.cholesky(H32.cuda())
    assert info == 0
    L = L.cpu().numpy().astype(np.float64)
    H64 = H32.numpy().astype(np.float64)
    Lref, _ = ref.cholesky(H64)
    assert np.array_equal(L, np.tril(L)) and np.all(np.diag(L) > 0)
    assert np.linalg.norm(L @ L.T - H64) <= 2e-6 * np.linalg.norm(H64)
    assert np.linalg.norm(L - Lref) <= 1e-4 * np.linalg.norm(Lref)
    if n >= 300:
        # a factor written into a wider array (leading dimension larger than n, not a multiple of 4
        # for odd n: the rank-256 updates then take the general product instead of the dedicated one)
        wide = torch.full((n, n + 5 + (n & 1)), 7.0, device="cuda")
        L2, info = ctx.cholesky(H32.cuda(), L=wide[:, :n])
        assert info == 0 and torch.equal(wide[:, n:], torch.full_like(wide[:, n:], 7.0))
        assert np.linalg.norm(L2.cpu().numpy().astype(np.float64) - Lref) <= 1e-4 * np.linalg.norm(Lref)


def test_cholesky_preconditioning_modes(ctx):
    from paper_2501_12956_amd import binding as b
    rng = np.random.default_rng(3)
    X = rng.normal(size=(96, 40))                     # p < n: singular H
    H64 = X @ X.T
    Hg = dev(H64, torch.float32)
    H64 = Hg.cpu().numpy().astype(np.float64)
    L, info = ctx.cholesky(Hg, b.PRECOND_NONE, raise_on_fail=False)
    assert 40 < info <= 96                            # first failing pivot is past the rank
    with pytest.raises(b.GanqError) as exc:
        ctx.cholesky(Hg, b.PRECOND_NONE)
    assert exc.value.status == b.GANQ_ERR_NOT_PD
    for mode, lam in [(b.PRECOND_LAMBDA, 0.5), (b.PRECOND_DIAGDOM, 0.0), (b.PRECOND_AUTO, 0.0)]:
        L, info = ctx.cholesky(Hg, mode, lam)
        assert info == 0
        L = L.cpu().numpy().astype(np.float64)
        omode = ref.PRECOND_DIAGDOM if mode == b.PRECOND_AUTO else mode
        Hp = ref.precondition(H64, omode, lam)
        Lref, _ = ref.cholesky(H64, omode, lam)
        assert np.linalg.norm(L @ L.T - Hp) <= 2e-6 * np.linalg.norm(Hp)
        rl = np.linalg.norm(L - Lref) / np.linalg.norm(Lref)
        print("preconditioned factor, mode %d: |L - Lref| / |Lref| = %.2e" % (mode, rl))
        assert rl <= 5e-6


def test_cholesky_numerically_singular_is_reported(ctx):
    """Fewer tokens than features plus a diagonal shift far below fp32 resolution: in exact (and in
    float64) arithmetic the matrix is positive definite with pivots near 1e-9 of the diagonal, so a
    float64 factorisation succeeds; in fp32 those pivots are rounding noise of either sign.  The
    plain factorisation must say so (not return a factor built on noise), AUTO must fall back to the
    preconditioner of Appendix A, and a well-conditioned matrix of the same size must pass."""
    from paper_2501_12956_amd import binding as b
    rng = np.random.default_rng(5)
    n, p = 320, 300
    X = rng.normal(size=(n, p))
    H64 = X @ X.T
    H64 += 1e-9 * np.diag(np.diag(H64))
    Hg = dev(H64, torch.float32)
    Lo, _ = ref.cholesky(H64)                     # before rounding to fp32 storage: positive definite
    assert np.all(np.diag(Lo) > 0)
    L, info = ctx.cholesky(Hg, b.PRECOND_NONE, raise_on_fail=False)
    assert p < info <= n, info
    L, info = ctx.cholesky(Hg, b.PRECOND_AUTO)
    assert info == 0
    Hp = ref.precondition(Hg.cpu().numpy().astype(np.float64), ref.PRECOND_DIAGDOM)
    L = L.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(L @ L.T - Hp) <= 2e-6 * np.linalg.norm(Hp)
    # strongly correlated but well above the noise floor: pivots near 1e-3 of the diagonal pass
    Y = rng.normal(size=(n, 4 * n))
    Y[1] = Y[0] + 0.03 * Y[1]
    G = dev(Y @ Y.T, torch.float32)
    L, info = ctx.cholesky(G, b.PRECOND_NONE)
    assert info == 0


# ----------------------------------------------------------------------------- T^0
@pytest.mark.parametrize("m,n,nbits,dtype", [(37, 300, 4, torch.float16), (5, 64, 3, torch.float32),
                                             (3, 1, 2, torch.float32), (2, 1000, 1, torch.float16)])
def test_init_codebooks(ctx, m, n, nbits, dtype):
    from paper_2501_12956_amd import binding as b
    W, _ = make_problem(m, n, 8, nbits)
    W = W.to(dtype)
    for mode, omode in [(b.INIT_QUANTILE_MID, ref.INIT_QUANTILE_MID),
                        (b.INIT_QUANTILE_ENDPOINTS, ref.INIT_QUANTILE_ENDPOINTS),
                        (b.INIT_MINMAX_GRID, ref.INIT_MINMAX_GRID)]:
        T = ctx.init_codebooks(W.cuda(), nbits, mode).cpu().numpy()
        Tref = ref.init_codebooks(W.float().numpy(), nbits, omode)
        ulp = np.spacing(np.abs(Tref).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(T.astype(np.float64) - Tref) <= ulp)
        assert np.all(np.diff(T, axis=1) >= 0)


# ----------------------------------------------------------------------------- S-update
@pytest.mark.parametrize("m,n,nbits", [(40, 200, 4), (16, 64, 3), (33, 65, 4), (1, 1, 2), (7, 130, 1),
                                       (50, 257, 2),
                                       # long enough that part of a block's sum over later columns is
                                       # taken one block early, with and without its row limit, even
                                       # and odd row strides of L
                                       (20, 1501, 4), (16, 1536, 4), (17, 2901, 3), (5, 2880, 2)])
def test_update_S_stagewise(ctx, m, n, nbits):
    W, X = make_problem(m, n, max(4 * n, 64), nbits)
    H64 = ref.build_hessian(X.numpy())
    L32 = torch.from_numpy(ref.cholesky(H64)[0]).float()
    T32 = torch.from_numpy(ref.init_codebooks(W.numpy(), nbits)).float()
    Q, E = ctx.update_S(W.cuda(), L32.cuda(), T32.cuda(), nbits, want_E=True)
    Q = Q.cpu().numpy()
    E = E.cpu().numpy()
    W64, L64, T64 = W.numpy().astype(np.float64), L32.numpy().astype(np.float64), T32.numpy().astype(np.float64)
    assert Q.max() < (1 << nbits)
    # residual output is exactly W - T[Q] in fp32
    assert np.array_equal(E, W.numpy() - np.take_along_axis(T32.numpy(), Q.astype(np.int64), axis=1))
    exact, near, viol = check_S(W64, L64, T64, Q, "S %dx%d N=%d" % (m, n, nbits))
    assert viol == 0
    Qref, _ = ref.update_S(W64, L64, T64)
    agree = float((Q == Qref).mean())
    rows_same = float((Q == Qref).all(axis=1).mean())
    print("free-running agreement: indices %.6f, rows %.4f" % (agree, rows_same))
    assert agree >= 0.999


@pytest.mark.parametrize("m,n,nbits", [(40, 200, 4), (33, 65, 4), (1, 1, 2), (7, 130, 1), (70, 1000, 3), (64, 777, 4)])
def test_update_S_32_row_slabs(ctx, m, n, nbits, monkeypatch):
    """The 32-row kernel of the S-update (chosen by the library for wide layers with many rows), forced
    here at small sizes: every choice is optimal for its float64 target, the residual output is exact,
    strided operands work, and it agrees with the 16-row kernel up to near ties."""
    W, X = make_problem(m, n, max(4 * n, 64), nbits)
    H64 = ref.build_hessian(X.numpy())
    L32 = torch.from_numpy(ref.cholesky(H64)[0]).float()
    T32 = torch.from_numpy(ref.init_codebooks(W.numpy(), nbits)).float()
    monkeypatch.setenv("GANQ_S_SLAB_ROWS", "16")
    Q16 = ctx.update_S(W.cuda(), L32.cuda(), T32.cuda(), nbits).cpu().numpy()
    monkeypatch.setenv("GANQ_S_SLAB_ROWS", "32")
    Q, E = ctx.update_S(W.cuda(), L32.cuda(), T32.cuda(), nbits, want_E=True)
    # odd leading dimension of L (no 8-byte loads) and of W
    Lw = torch.zeros(n, n + 3, device="cuda")
    Lw[:, :n] = L32.cuda()
    Ww = torch.zeros(m, n + 5, device="cuda")
    Ww[:, :n] = W.cuda()
    Qs = ctx.update_S(Ww[:, :n], Lw[:, :n], T32.cuda(), nbits).cpu().numpy()
    monkeypatch.delenv("GANQ_S_SLAB_ROWS")
    Q = Q.cpu().numpy()
    E = E.cpu().numpy()
    W64, L64, T64 = W.numpy().astype(np.float64), L32.numpy().astype(np.float64), T32.numpy().astype(np.float64)
    assert Q.max() < (1 << nbits)
    assert np.array_equal(E, W.numpy() - np.take_along_axis(T32.numpy(), Q.astype(np.int64), axis=1))
    _, _, viol = check_S(W64, L64, T64, Q, "S32 %dx%d N=%d" % (m, n, nbits))
    assert viol == 0
    _, _, viol = check_S(W64, L64, T64, Qs, "S32 strided %dx%d N=%d" % (m, n, nbits))
    assert viol == 0
    assert float((Q == Q16).mean()) >= 0.999 and float((Qs == Q16).mean()) >= 0.999


def test_update_S_ties_and_identity(ctx):
    # H = I: plain nearest rounding; duplicated codebook entries: lowest index wins
    T = np.array([[0.0, 1.0, 1.0, 0.0], [-1.0, -1.0, 2.0, 2.0]], dtype=np.float32)
    W = np.array([[0.5, 0.9, 0.1, 0.25, 1.5], [0.5, -3.0, 0.49, 0.51, 2.0]], dtype=np.float32)
    L = np.eye(5, dtype=np.float32) * 3.0
    Q = ctx.update_S(dev(W), dev(L), dev(T), 2).cpu().numpy()
    Qref, _ = ref.update_S(W, L, T)
    assert np.array_equal(Q, Qref)
    assert list(Q[0]) == [0, 1, 0, 0, 1] and list(Q[1]) == [0, 0, 0, 2, 2]


def test_updates_on_strided_views(ctx):
    """W, L, H and Q as views with leading dimensions larger than n, L additionally starting at an
    address that is only 4-byte aligned (the S-update then fetches L element by element): same
    indices and codebooks as the contiguous calls, bit for bit."""
    m, n, nbits = 37, 900, 4
    W, X = make_problem(m, n, 4 * n, nbits, seed=9)
    H64 = ref.build_hessian(X.numpy())
    L32 = torch.from_numpy(ref.cholesky(H64)[0]).float().cuda()
    H32 = torch.from_numpy(H64).float().cuda()
    T32 = torch.from_numpy(ref.init_codebooks(W.numpy(), nbits)).float().cuda()
    Wg = W.cuda()
    Q0 = ctx.update_S(Wg, L32, T32, nbits)
    T0 = ctx.update_T(Wg, H32, Q0, T32.clone(), nbits)

    def wide(t, pad, shift=0):
        big = torch.zeros(t.shape[0], t.shape[1] + pad + shift, dtype=t.dtype, device="cuda")
        view = big[:, shift:shift + t.shape[1]]
        view.copy_(t)
        return view

    Wv, Lv, Hv = wide(Wg, 12), wide(L32, 6, shift=1), wide(H32, 20)
    assert Lv.data_ptr() % 16 != 0 and Lv.stride(0) % 4 != 0
    Qv = wide(torch.zeros_like(Q0), 5)
    ctx.update_S(Wv, Lv, T32, nbits, Q=Qv)
    assert torch.equal(Qv, Q0)
    T1 = ctx.update_T(Wv, Hv, Qv, T32.clone(), nbits)
    assert torch.equal(T1, T0)


# ----------------------------------------------------------------------------- T-update
@pytest.mark.parametrize("m,n,nbits", [(40, 200, 4), (16, 64, 3), (33, 300, 4), (3, 130, 1), (20, 257, 2),
                                       (2, 1, 2)])
def test_update_T_stagewise(ctx, m, n, nbits):
    W, X = make_problem(m, n, max(4 * n, 64), nbits)
    H32 = ctx.build_hessian(X.cuda()).cpu()
    H64 = H32.numpy().astype(np.float64)
    L64, _ = ref.cholesky(H64)
    T0 = ref.init_codebooks(W.numpy(), nbits)
    Q, _ = ref.update_S(W.numpy().astype(np.float64), L64, T0)
    Tg = dev(T0, torch.float32)
    Tg, cnt = ctx.update_T(W.cuda(), H32.cuda(), dev(Q), Tg, nbits, want_counts=True)
    Tg = Tg.cpu().numpy().astype(np.float64)
    Tref, cref = ref.update_T(W.numpy().astype(np.float64), H64, Q, nbits)
    err = np.abs(Tg - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    print("T-update %dx%d N=%d: max row error %.2e" % (m, n, nbits, err.max()))
    assert np.all(err <= 1e-4)
    assert np.array_equal(cnt.cpu().numpy(), cref)


def test_update_T_prepared_inputs(ctx):
    """ganq_update_T_prepare leaves G = W H and the digits of H in the workspace: the T-updates (and
    the S-updates and loss evaluations between them) of a caller-driven alternation then give bit for
    bit what the unprepared calls give, at lower cost; after H changes in place a new prepare call
    brings the results into line with the new H."""
    m, n, nbits = 48, 320, 4
    W, X = make_problem(m, n, 2048, nbits)
    Wg = W.cuda()
    H = ctx.build_hessian(X.cuda())
    L, info = ctx.cholesky(H)
    assert info == 0
    T0 = ctx.init_codebooks(Wg, nbits)

    def alternate(prepared):
        T = T0.clone()
        outs = []
        if prepared:
            ctx.update_T_prepare(Wg, H, nbits)
        ctx.profile_enable(True)
        for _ in range(3):
            Q = ctx.update_S(Wg, L, T, nbits)
            T = ctx.update_T(Wg, H, Q, T, nbits)
            outs.append((Q.clone(), T.clone(), ctx.layer_loss(Wg, H, T, Q, nbits)))
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        ctx.update_T_prepare(None, None, nbits)
        return outs, prof

    plain, prof_plain = alternate(False)
    prep, prof_prep = alternate(True)
    assert prof_plain["gemm_wh"][1] == 3 and prof_plain["t_prep"][1] == 3
    assert prof_prep["gemm_wh"][1] == 0 and prof_prep["t_prep"][1] == 0      # prepared outside the bracket
    for (Qa, Ta, la), (Qb, Tb, lb) in zip(plain, prep):
        assert torch.equal(Qa, Qb) and torch.equal(Ta, Tb) and la == lb
    # H changes in place: prepare again, and the result is that of the new H
    Q = plain[-1][0]
    H2 = H.clone()
    ctx.update_T_prepare(Wg, H2, nbits)
    Told = ctx.update_T(Wg, H2, Q, T0.clone(), nbits)
    H2 *= 1.0 + 0.5 * torch.eye(n, device="cuda")            # another matrix in the same memory
    ctx.update_T_prepare(Wg, H2, nbits)
    Tnew = ctx.update_T(Wg, H2, Q, T0.clone(), nbits)
    ctx.update_T_prepare(None, None, nbits)
    Tfresh = ctx.update_T(Wg, H2, Q, T0.clone(), nbits)
    assert torch.equal(Tnew, Tfresh) and not torch.equal(Tnew, Told)
    Tref, _ = ref.update_T(W.numpy().astype(np.float64), H2.cpu().numpy().astype(np.float64), Q.cpu().numpy(), nbits)
    err = np.abs(Tnew.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    assert err.max() <= 1e-4


def _structured_H(kind, n, seed):
    """Second-moment matrices that drive the integer representation of H in the T-update through
    its cases: weakly or strongly correlated features (two or three digits per entry), feature
    scales far beyond the range of the column factors, both kinds of rows in one matrix, and a
    feature that is never active."""
    rng = np.random.default_rng(seed)
    p = 4096
    Z = rng.standard_normal((n, p))
    f = rng.standard_normal((1, p))
    rho = {"weak": 0.0, "medium": 0.4, "strong": 0.8, "wide": 0.0, "vwide": 0.2, "mixed": 0.0, "dead": 0.3}[kind]
    X = np.sqrt(1 - rho) * Z + np.sqrt(rho) * f
    d = np.exp(rng.uniform(np.log(0.5), np.log(8.0), size=n))
    if kind == "wide":
        d = np.exp(rng.uniform(np.log(1e-2), np.log(1e3), size=n))
    if kind == "vwide":       # eight decades of feature scale: H spans 2^53
        d = np.exp(rng.uniform(np.log(1e-4), np.log(1e4), size=n))
    if kind == "mixed":
        X[n // 2:] = np.sqrt(0.1) * Z[n // 2:] + np.sqrt(0.9) * f
    if kind == "dead":
        d[n // 3] = 0.0
    X = X * d[:, None]
    return (X @ X.T).astype(np.float32)


@pytest.mark.parametrize("kind,nbits,m,n", [(k, b, 40, 300) for b in (3, 4)
                                            for k in ("weak", "strong", "wide", "mixed", "dead")]
                         + [("medium", 4, 16, 1100), ("mixed", 3, 70, 1100), ("weak", 2, 130, 700),
                            ("wide", 2, 168, 43), ("wide", 1, 60, 90), ("vwide", 4, 40, 300), ("vwide", 3, 33, 520)])
def test_update_T_structured_H(ctx, kind, nbits, m, n):
    H32 = _structured_H(kind, n, 11)
    rng = np.random.default_rng(12)
    W = (rng.standard_normal((m, n)) * 0.02).astype(np.float32)
    Q = rng.integers(0, 1 << nbits, size=(m, n)).astype(np.uint8)
    Tg = ctx.update_T(dev(W), dev(H32), dev(Q), dev(np.zeros((m, 1 << nbits), np.float32)), nbits)
    Tg = (Tg[0] if isinstance(Tg, tuple) else Tg).cpu().numpy().astype(np.float64)
    Tref, _ = ref.update_T(W.astype(np.float64), H32.astype(np.float64), Q, nbits)
    err = np.abs(Tg - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    print("T-update, %s H %dx%d, N=%d: max row error %.2e" % (kind, m, n, nbits, err.max()))
    assert np.all(err <= 1e-4)


@pytest.mark.parametrize("kind", ["wide", "vwide", "strong"])
def test_layer_loss_structured_H(ctx, kind):
    """The two split-fp16 products (F = E H of the loss here) scale H by one power of two for the
    whole matrix; feature scales spread over five and eight decades must not cost accuracy in the
    objective, nor in its per-row values."""
    m, n, nbits = 40, 300, 4
    H32 = _structured_H(kind, n, 21)
    rng = np.random.default_rng(22)
    W = (rng.standard_normal((m, n)) * 0.02).astype(np.float32)
    T0 = ref.init_codebooks(W, nbits).astype(np.float32)
    Q = rng.integers(0, 1 << nbits, size=(m, n)).astype(np.uint8)
    loss, rows = ctx.layer_loss(dev(W), dev(H32), dev(T0), dev(Q), nbits, want_rows=True)
    lref, rref = ref.layer_loss(W, H32, T0, Q)
    rel = np.abs(rows.cpu().numpy() - rref) / np.abs(rref)
    print("loss, %s H: total off by %.2e relative, worst row %.2e" % (kind, abs(loss - lref) / lref, rel.max()))
    assert abs(loss - lref) <= 1e-5 * lref
    assert rel.max() <= 1e-4


def test_update_T_magnitude_and_diagonal_H(ctx):
    """The codebooks do not depend on the scale of H: a power-of-two factor moves the row exponents
    of the integer representation and nothing else.  And a diagonal H (no off-diagonal digits at
    all) gives the H_jj-weighted mean of each group."""
    m, n, nbits = 24, 300, 4
    H32 = _structured_H("mixed", n, 3)
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((m, n)) * 0.02).astype(np.float32)
    Q = rng.integers(0, 1 << nbits, size=(m, n)).astype(np.uint8)
    T0 = dev(np.zeros((m, 1 << nbits), np.float32))
    base = ctx.update_T(dev(W), dev(H32), dev(Q), T0.clone(), nbits).cpu().numpy()
    for e in (-60, 45):
        Hs = np.ldexp(H32, e).astype(np.float32)
        assert np.isfinite(Hs).all() and Hs.min() != 0
        got = ctx.update_T(dev(W), dev(Hs), dev(Q), T0.clone(), nbits).cpu().numpy()
        assert np.abs(got - base).max() <= 1e-6 * np.abs(base).max(), e
    d = rng.uniform(0.5, 4.0, size=n).astype(np.float32)
    got = ctx.update_T(dev(W), dev(np.diag(d)), dev(Q), T0.clone(), nbits).cpu().numpy().astype(np.float64)
    want = np.zeros_like(got)
    for i in range(m):
        for c in range(1 << nbits):
            sel = Q[i] == c
            if sel.any():
                want[i, c] = (W[i, sel].astype(np.float64) * d[sel]).sum() / d[sel].astype(np.float64).sum()
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


@pytest.mark.parametrize("eps,loss_tol", [(1e-2, 1e-5), (1e-3, 1e-4), (1e-4, 1e-2)])
def test_update_T_ill_conditioned_rows(ctx, eps, loss_tol):
    """Features that are copies of one signal plus noise of relative variance eps make every
    S_i H S_i^T nearly rank one: cond(A_i) is about 1e5, 1e6, 1e7 for eps = 1e-2, 1e-3, 1e-4.  The
    codebook is then determined only up to (input rounding) x cond, so T itself is compared with what
    a plain float32 evaluation of A_i and b_i (float64 solve) achieves on the same rows, and the
    quantity that is well determined - the objective of Eq. (9) at the returned codebook - against
    the oracle's optimum."""
    m, n, nbits, p = 24, 512, 4, 4096
    C = 1 << nbits
    rng = np.random.default_rng(5)
    common = rng.standard_normal(p)
    X = common[None, :] * (1 + 0.2 * rng.standard_normal((n, 1))) + np.sqrt(eps) * rng.standard_normal((n, p))
    H32 = (X @ X.T).astype(np.float32)
    W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    Q = rng.integers(0, C, (m, n)).astype(np.uint8)
    H64, W64 = H32.astype(np.float64), W.astype(np.float64)
    Tref, _ = ref.update_T(W64, H64, Q, nbits)
    Tg = ctx.update_T(dev(W), dev(H32), dev(Q), dev(np.zeros((m, C), np.float32)), nbits)
    Tg = (Tg[0] if isinstance(Tg, tuple) else Tg).cpu().numpy().astype(np.float64)
    # the same rows with A_i and b_i summed in float32 (what a straightforward fp32 program has)
    G32 = W @ H32
    T32 = np.zeros_like(Tref)
    conds = []
    for i in range(m):
        S32 = ref.one_hot(Q[i], C).astype(np.float32)
        A32 = (S32 @ H32) @ S32.T
        b32 = G32[i] @ S32.T
        T32[i] = np.linalg.solve(A32.astype(np.float64), b32.astype(np.float64))
        S = S32.astype(np.float64)
        conds.append(np.linalg.cond(S @ H64 @ S.T))
    scale = np.abs(Tref).max()
    err_g, err_32 = np.abs(Tg - Tref).max() / scale, np.abs(T32 - Tref).max() / scale
    _, l_ref = ref.layer_loss(W64, H64, Tref, Q)
    _, l_g = ref.layer_loss(W64, H64, Tg, Q)
    excess = ((l_g - l_ref) / l_ref).max()
    print("T-update, cond(A_i) %.1e..%.1e: |T - oracle| / |T| = %.2e (plain float32: %.2e), "
          "objective above the optimum by %.2e relative" % (min(conds), max(conds), err_g, err_32, excess))
    assert err_g <= 3.0 * err_32 + 1e-6
    assert excess <= loss_tol


def test_update_T_empty_codes(ctx):
    from paper_2501_12956_amd import binding as b
    m, n, nbits = 6, 96, 3
    W, X = make_problem(m, n, 512, nbits)
    H32 = ctx.build_hessian(X.cuda()).cpu()
    rng = np.random.default_rng(5)
    Q = rng.integers(0, 8, size=(m, n)).astype(np.uint8)
    Q[1][Q[1] == 3] = 4            # code 3 unused in row 1
    Q[2][:] = 5                    # a single code in row 2
    Q[4][(Q[4] == 0) | (Q[4] == 7)] = 1
    Tprev = rng.normal(size=(m, 8)).astype(np.float32)
    W64, H64 = W.numpy().astype(np.float64), H32.numpy().astype(np.float64)
    for mode, omode in [(b.EMPTY_ZERO, ref.EMPTY_ZERO), (b.EMPTY_KEEP, ref.EMPTY_KEEP)]:
        Tg, cnt = ctx.update_T(W.cuda(), H32.cuda(), dev(Q), dev(Tprev), nbits, empty=mode, want_counts=True)
        Tref, cref = ref.update_T(W64, H64, Q, nbits, T_prev=Tprev, empty=omode)
        err = np.abs(Tg.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
        assert np.all(err <= 1e-4), err
        assert list(cnt.cpu().numpy()) == list(cref) == [0, 1, 7, 0, 2, 0]


# ----------------------------------------------------------------------------- loss
@pytest.mark.parametrize("m,n,nbits", [(40, 200, 4), (3, 65, 2), (130, 129, 3)])
def test_layer_loss(ctx, m, n, nbits):
    W, X = make_problem(m, n, max(4 * n, 64), nbits)
    H32 = ctx.build_hessian(X.cuda()).cpu()
    T0 = ref.init_codebooks(W.numpy(), nbits).astype(np.float32)
    rng = np.random.default_rng(6)
    Q = rng.integers(0, 1 << nbits, size=(m, n)).astype(np.uint8)
    loss, rows = ctx.layer_loss(W.cuda(), H32.cuda(), dev(T0), dev(Q), nbits, want_rows=True)
    lref, rref = ref.layer_loss(W.numpy(), H32.numpy(), T0, Q)
    assert abs(loss - lref) <= 1e-4 * lref
    assert np.all(np.abs(rows.cpu().numpy() - rref) <= 1e-4 * rref)
    # and against the literal Eq. (1) with the fp16 activations
    ldir = ref.layer_loss_direct(W.numpy(), X.numpy(), T0, Q)
    assert abs(loss - ldir) <= 1e-4 * ldir


# ----------------------------------------------------------------------------- Algorithm 1
def test_quantize_layer_config1(ctx):
    """The tiny configuration end to end: K = 10 from quantile codebooks."""
    cfg = synth.CONFIGS["c1"]
    W, X = synth.make_layer(cfg, 0)
    Wg, Xg = W.cuda(), X.cuda()
    H = ctx.build_hessian(Xg)
    Href = ref.build_hessian(X.numpy())
    check_H(H.cpu().numpy().astype(np.float64), Href, cfg.p, "c1", wide=True)      # fp32 activations
    L, info = ctx.cholesky(H)
    assert info == 0
    K = cfg.iters
    T, Q, hist = ctx.quantize_layer(Wg, H, cfg.nbits, K, L=L, history=True)
    T2, Q2 = ctx.quantize_layer(Wg, H, cfg.nbits, K, L=L)
    assert torch.equal(T, T2) and torch.equal(Q, Q2)            # bit-reproducible
    # restartable: K = 10 equals 5 + 5 with T carried over - bit for bit when every sweep sums
    # S_i H S_i^T again (a call that may update it from the changed columns starts its first sweep
    # with a fresh sum, so the split call rounds differently in the last bits)
    Tf, Qf = ctx.quantize_layer(Wg, H, cfg.nbits, K, L=L, full_t_update=True)
    Ta, _ = ctx.quantize_layer(Wg, H, cfg.nbits, 5, L=L, full_t_update=True)
    Tb, Qb = ctx.quantize_layer(Wg, H, cfg.nbits, 5, T=Ta.clone(), L=L, full_t_update=True)
    assert torch.equal(Tb, Tf) and torch.equal(Qb, Qf)
    # the default call did update in some sweeps, and agrees with the always-summing one
    ctx.profile_enable(True)
    ctx.quantize_layer(Wg, H, cfg.nbits, K, L=L)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    # (with this layer's four scaled channels some tiles of H take three digits, and then every
    # sweep sums; test_quantize_layer_updates_from_changed_columns covers the other case)
    print("c1: sweeps that summed %d, that updated %d" % (prof["t_accum"][1], prof["t_delta"][1]))
    assert prof["t_accum"][1] + prof["t_delta"][1] == K
    same = (Q == Qf).all(dim=1)
    assert float(same.float().mean()) >= 0.99
    dT = (T[same] - Tf[same]).abs().amax(dim=1) / Tf[same].abs().amax(dim=1)
    assert float(dT.max()) <= 1e-5
    # factoring inside the call gives the same result as passing L
    T3, Q3 = ctx.quantize_layer(Wg, H, cfg.nbits, K)
    assert torch.equal(T3, T) and torch.equal(Q3, Q)

    H64 = H.cpu().numpy().astype(np.float64)
    L64 = L.cpu().numpy().astype(np.float64)
    W64 = W.numpy().astype(np.float64)
    # stage-wise on the last sweep: Q^K is optimal against T^{K-1}, T^K is the refit to Q^K
    Tprev, _ = ctx.quantize_layer(Wg, H, cfg.nbits, K - 1, L=L)
    _, _, viol = check_S(W64, L64, Tprev.cpu().numpy().astype(np.float64), Q.cpu().numpy(), "c1 last sweep")
    assert viol == 0
    Tref, _ = ref.update_T(W64, H64, Q.cpu().numpy(), cfg.nbits)
    err = np.abs(T.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    assert np.all(err <= 1e-4)
    # loss history: T-steps never increase the objective; final loss matches the oracle's
    # evaluation of the GPU's (T, Q) and beats rounding onto T^0
    for k in range(K):
        assert hist[2 * k + 1] <= hist[2 * k] * (1 + 1e-5)
    lref = ref.layer_loss(W64, H64, T.cpu().numpy(), Q.cpu().numpy())[0]
    assert abs(hist[-1] - lref) <= 1e-4 * lref
    # free-running oracle from the same T^0 (reported; rows that hit a near tie may diverge)
    T0 = ref.init_codebooks(W64, cfg.nbits)
    To, Qo, ho = ref.quantize_layer(W64, H64, T0, cfg.nbits, K, L=L64, history=True)
    agree = float((Q.cpu().numpy() == Qo).mean())
    rows_same = float((Q.cpu().numpy() == Qo).all(axis=1).mean())
    print("c1 free-running: index agreement %.6f, identical rows %.4f, loss gpu %.6e oracle %.6e"
          % (agree, rows_same, hist[-1], ho[-1]))
    assert hist[-1] < 0.8 * ho[0]
    assert abs(hist[-1] - ho[-1]) <= 1e-3 * ho[-1]
    same = (Q.cpu().numpy() == Qo).all(axis=1)
    errT = np.abs(T.cpu().numpy()[same] - To[same]).max(axis=1) / np.abs(To[same]).max(axis=1)
    assert np.all(errT <= 1e-4)


@pytest.mark.parametrize("m,n,nbits", [(70, 640, 4), (33, 1100, 3), (130, 900, 4)])
def test_quantize_layer_updates_from_changed_columns(ctx, m, n, nbits):
    """Sweeps that change few indices bring S_i H S_i^T up to date from the changed columns instead
    of summing it again.  On a layer where that happens (checked through the per-class launch
    counts): the final codebooks are the oracle's least-squares refit to the final indices, the last
    sweep's choices are optimal for their float64 targets, the call is bit-reproducible, and it
    agrees with the always-summing call row for row except where a near tie parted them."""
    K = 24              # small layers settle more slowly than the 4096-wide ones
    W, X = make_problem(m, n, 16 * n, nbits)
    Wg = W.cuda()
    H = ctx.build_hessian(X.cuda())
    L, info = ctx.cholesky(H)
    assert info == 0
    ctx.profile_enable(True)
    T, Q = ctx.quantize_layer(Wg, H, nbits, K, L=L)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    print("%dx%d N=%d: sweeps that summed %d, that updated %d" % (m, n, nbits, prof["t_accum"][1], prof["t_delta"][1]))
    assert prof["t_delta"][1] >= 3 and prof["t_accum"][1] + prof["t_delta"][1] == K
    assert prof["t_skip"][1] == 2 * (K - 1) - K + 1
    T2, Q2 = ctx.quantize_layer(Wg, H, nbits, K, L=L)
    assert torch.equal(T, T2) and torch.equal(Q, Q2)
    W64 = W.numpy().astype(np.float64)
    H64 = H.cpu().numpy().astype(np.float64)
    L64 = L.cpu().numpy().astype(np.float64)
    Qh = Q.cpu().numpy()
    Tref, _ = ref.update_T(W64, H64, Qh, nbits)
    err = np.abs(T.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    Tsa = ctx.update_T(Wg, H, Q, T.clone(), nbits)          # the same refit, summed afresh by the stand-alone call
    errsa = np.abs(Tsa.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    print("T^K after updating sweeps: max row error %.2e (summed afresh: %.2e); log %s"
          % (err.max(), errsa.max(), ctx.sweep_log()[-3:]))
    assert err.max() <= 1e-4
    Tprev, _ = ctx.quantize_layer(Wg, H, nbits, K - 1, L=L)
    _, _, viol = check_S(W64, L64, Tprev.cpu().numpy().astype(np.float64), Qh, "updating sweeps")
    assert viol == 0
    # T^{K-1} too (it came out of an updating sweep and fed the last S-update)
    _, Qp = ctx.quantize_layer(Wg, H, nbits, K - 1, L=L)
    Tpref, _ = ref.update_T(W64, H64, Qp.cpu().numpy(), nbits)
    errp = np.abs(Tprev.cpu().numpy() - Tpref).max(axis=1) / np.abs(Tpref).max(axis=1)
    assert errp.max() <= 1e-4
    Tf, Qf = ctx.quantize_layer(Wg, H, nbits, K, L=L, full_t_update=True)
    # (reported; over 24 sweeps a difference in the last bits of T parts rows at near ties)
    same = (Q == Qf).all(dim=1)
    print("rows identical to the always-summing call after %d sweeps: %.3f" % (K, float(same.float().mean())))
    assert float(same.float().mean()) >= 0.8
    dT = (T[same] - Tf[same]).abs().amax(dim=1) / Tf[same].abs().amax(dim=1)
    assert float(dT.max()) <= 2e-5


def test_quantize_layer_fp16_weights_and_init_inside(ctx):
    m, n, nbits = 48, 192, 3
    W, X = make_problem(m, n, 1024, nbits)
    W16 = W.half()
    H = ctx.build_hessian(X.cuda())
    T, Q = ctx.quantize_layer(W16.cuda(), H, nbits, 3)
    # same as the explicit pipeline on the fp32 upcast
    Wf = W16.float().cuda()
    T0 = ctx.init_codebooks(W16.cuda(), nbits)
    T1, Q1 = ctx.quantize_layer(Wf, H, nbits, 3, T=T0.clone())
    assert torch.equal(T, T1) and torch.equal(Q, Q1)


@pytest.mark.parametrize("mode", ["lambda", "diagdom", "auto"])
def test_quantize_layer_rank_deficient_activations(ctx, mode):
    """Fewer calibration tokens than input features (p < n): H = X X^T is singular and the
    plain factorization fails (Remark 3.1, Appendix A).  The preconditioned factor drives the
    S-update; the T-update and the objective keep the raw H.  Stage-wise against the oracle."""
    from paper_2501_12956_amd import binding as b
    m, n, p, nbits, K = 40, 320, 160, 4, 4
    g = torch.Generator().manual_seed(5)
    W = (torch.randn(m, n, generator=g) * 0.02).float()
    Xt = torch.randn(p, n, generator=g).float()          # tokens x features
    Xt[:, 7] *= 20.0
    Wg = W.cuda()
    H = ctx.build_hessian_tokens(Xt.cuda())
    with pytest.raises(b.GanqError) as exc:
        ctx.quantize_layer(Wg, H, nbits, 1, precond=b.PRECOND_NONE)
    assert exc.value.status == b.GANQ_ERR_NOT_PD
    gmode = {"lambda": b.PRECOND_LAMBDA, "diagdom": b.PRECOND_DIAGDOM, "auto": b.PRECOND_AUTO}[mode]
    omode = {"lambda": ref.PRECOND_LAMBDA, "diagdom": ref.PRECOND_DIAGDOM, "auto": ref.PRECOND_DIAGDOM}[mode]
    H64 = H.cpu().numpy().astype(np.float64)
    lam = 1e-2 * float(np.mean(np.diag(H64))) if mode == "lambda" else 0.0
    T, Q, hist = ctx.quantize_layer(Wg, H, nbits, K, precond=gmode, lam=lam, history=True)
    Tprev, _ = ctx.quantize_layer(Wg, H, nbits, K - 1, precond=gmode, lam=lam)
    W64 = W.numpy().astype(np.float64)
    # the oracle's factor of the preconditioned matrix; the GPU's own factor is checked against it
    Lref, _ = ref.cholesky(H64, omode, lam)
    Lg, info = ctx.cholesky(H, gmode, lam)
    assert info == 0
    rl = np.linalg.norm(Lg.cpu().numpy() - Lref) / np.linalg.norm(Lref)
    print("rank-deficient %s: |L - Lref| / |Lref| = %.2e" % (mode, rl))
    assert rl <= 1e-4
    L64 = Lg.cpu().numpy().astype(np.float64)
    _, _, viol = check_S(W64, L64, Tprev.cpu().numpy().astype(np.float64), Q.cpu().numpy(), "rank-deficient " + mode)
    assert viol == 0
    Tref, _ = ref.update_T(W64, H64, Q.cpu().numpy(), nbits)        # raw H
    err = np.abs(T.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    print("rank-deficient %s: T-update max row error %.2e" % (mode, err.max()))
    assert np.all(err <= 1e-4)
    lref = ref.layer_loss(W64, H64, T.cpu().numpy(), Q.cpu().numpy())[0]
    assert abs(hist[-1] - lref) <= 1e-4 * lref
    for k in range(K):
        assert hist[2 * k + 1] <= hist[2 * k] * (1 + 1e-5)
    # it beats rounding every weight onto T^0 in the same objective
    T0 = ref.init_codebooks(W64, nbits)
    Q0 = np.abs(W64[:, :, None] - T0[:, None, :]).argmin(axis=2)
    l0 = ref.layer_loss(W64, H64, T0, Q0)[0]
    print("rank-deficient %s: loss %.4e vs nearest rounding onto T0 %.4e" % (mode, hist[-1], l0))
    assert hist[-1] < l0


# ----------------------------------------------------------------------------- Algorithm 2
@pytest.mark.parametrize("m,n,r,dtype", [(37, 300, 0.05, torch.float32), (8, 1000, 0.005, torch.float16),
                                         (3, 64, 0.0, torch.float32), (5, 17, 0.3, torch.float16),
                                         # n r / 2 an integer that binary rounding of r or of 1 - r/2 could miss
                                         (4, 2000, 0.01, torch.float32), (3, 1000, 0.1, torch.float16),
                                         (6, 400, 0.07, torch.float32), (5, 50, 0.28, torch.float32)])
def test_outlier_split_matches_oracle(ctx, m, n, r, dtype):
    """W = W_sparse + W_dense: no arithmetic on the values, so the split is compared exactly."""
    g = torch.Generator().manual_seed(9)
    W = (torch.randn(m, n, generator=g) * 0.02).to(dtype)
    W[torch.rand(m, n, generator=g) < 0.01] *= 10.0
    Ws_ref, Wd_ref = ref.outlier_split(W.numpy().astype(np.float64), r)
    Wd, row_ptr, col, val = ctx.outlier_split(W.cuda(), r)
    Wd = Wd.cpu().numpy().astype(np.float64)
    assert np.array_equal(Wd, Wd_ref)
    row_ptr, col, val = row_ptr.cpu().numpy(), col.cpu().numpy(), val.cpu().numpy().astype(np.float64)
    assert row_ptr[0] == 0 and row_ptr[-1] == len(col) == len(val) == _count_masked(W.numpy().astype(np.float64), r)
    dense = np.zeros((m, n))
    for i in range(m):
        cs = col[row_ptr[i]:row_ptr[i + 1]]
        assert np.all(np.diff(cs) > 0)                  # ascending, no duplicates
        dense[i, cs] = val[row_ptr[i]:row_ptr[i + 1]]
    assert np.array_equal(dense, Ws_ref)
    assert np.array_equal(dense + Wd, W.numpy().astype(np.float64))


def _count_masked(W, r):
    """Number of outlier positions of Algorithm 2 (zeros that fall in a tail count too)."""
    n = W.shape[1]
    lower, upper = ref.outlier_cutoff_positions(n, r)
    Ws = np.sort(W, axis=1)
    return int(((W >= Ws[:, upper][:, None]) | (W <= Ws[:, lower][:, None])).sum())


def test_outlier_split_ties_and_capacity(ctx):
    """Many equal values at a cut-off all become outliers (comparisons are >= and <=); a CSR
    capacity that is too small is reported with the needed size, and nothing else changes."""
    from paper_2501_12956_amd import binding as b
    W = torch.zeros(4, 40)
    W[:, :10] = -1.0
    W[:, 30:] = 2.0
    W[0, 5] = -3.0
    Ws_ref, Wd_ref = ref.outlier_split(W.numpy().astype(np.float64), 0.1)
    nnz_ref = _count_masked(W.numpy().astype(np.float64), 0.1)
    assert nnz_ref == 4 * 20                             # all the -1 and all the 2 of every row
    Wg = W.cuda()
    with pytest.raises(b.GanqError) as exc:
        Wd = torch.empty(4, 40, device="cuda")
        rp = torch.empty(5, dtype=torch.int64, device="cuda")
        col = torch.empty(8, dtype=torch.int32, device="cuda")
        val = torch.empty(8, device="cuda")
        import ctypes
        nnz = ctypes.c_int64(0)
        st = ctx.lib.ganq_outlier_split(ctx.handle, b._ptr(Wg), b.GANQ_F32, 4, 40, 40, 0.1, b._ptr(Wd), 40,
                                        b._ptr(rp), b._ptr(col), b._ptr(val), 8, ctypes.byref(nnz))
        assert st == b.GANQ_ERR_INVALID_ARG and nnz.value == nnz_ref
        assert np.array_equal(Wd.cpu().numpy().astype(np.float64), Wd_ref)
        ctx._check(st)
    assert exc.value.status == b.GANQ_ERR_INVALID_ARG
    Wd, row_ptr, col, val = ctx.outlier_split(Wg, 0.1, capacity=8)       # the binding retries
    assert len(col) == nnz_ref and np.array_equal(Wd.cpu().numpy().astype(np.float64), Wd_ref)


def test_outlier_split_lowers_the_layer_loss(ctx):
    """Section 3.3: quantising W_dense and keeping W_sparse exact gives a lower layer error than
    quantising W itself (config-1 recipe: 0.5 % of the weights are scaled by 10)."""
    cfg = synth.CONFIGS["c1"]
    W = synth.make_weight(cfg, 0, "cpu")
    X = synth.make_activations(cfg, 0, "cpu")
    H = ctx.build_hessian(X.cuda())
    Wg = W.cuda()
    T, Q, hist = ctx.quantize_layer(Wg, H, cfg.nbits, cfg.iters, history=True)
    Wd, row_ptr, col, val = ctx.outlier_split(Wg, 0.005)
    assert 0 < len(col) <= 0.02 * W.numel()
    Td, Qd, histd = ctx.quantize_layer(Wd, H, cfg.nbits, cfg.iters, history=True)
    # error of (T_d[Q_d] + W_sparse) against W equals the error of T_d[Q_d] against W_dense
    H64 = H.cpu().numpy().astype(np.float64)
    lsplit = ref.layer_loss(Wd.cpu().numpy().astype(np.float64), H64, Td.cpu().numpy(), Qd.cpu().numpy())[0]
    Ws_ref, Wd_ref = ref.outlier_split(W.numpy().astype(np.float64), 0.005)
    deq = ref.dequantize(Td.cpu().numpy().astype(np.float64), Qd.cpu().numpy()) + Ws_ref
    R = W.numpy().astype(np.float64) - deq
    ldirect = float(np.einsum("ij,jk,ik->", R, H64, R))
    assert abs(lsplit - ldirect) <= 1e-9 * ldirect
    assert abs(histd[-1] - lsplit) <= 1e-4 * lsplit
    print("config 1: loss %.4e plain, %.4e with %.2f %% of the weights kept exact"
          % (hist[-1], lsplit, 100.0 * len(col) / W.numel()))
    assert lsplit < 0.8 * hist[-1]


def test_layers_sharing_activations_can_be_stacked(ctx):
    """Layers that see the same input (q/k/v, gate/up) share H and L, and rows are independent
    (Section 3.1): quantising their weights stacked row-wise in one call gives, row for row,
    what separate calls give, and what the oracle gives for the stacked matrix."""
    n, nbits, K = 192, 4, 3
    _, X = make_problem(8, n, 1024, nbits)
    g = torch.Generator().manual_seed(17)
    Ws = [(torch.randn(mm, n, generator=g) * 0.02).float().cuda() for mm in (40, 24, 9)]
    H = ctx.build_hessian(X.cuda())
    L, info = ctx.cholesky(H)
    assert info == 0
    Wall = torch.cat(Ws, 0).contiguous()
    # (every sweep sums S_i H S_i^T again here: whether a sweep updates it instead depends on the
    # changes of all rows of a call, which differ between the stacked and the separate calls)
    Tall, Qall = ctx.quantize_layer(Wall, H, nbits, K, L=L, full_t_update=True)
    r0 = 0
    for W in Ws:
        T, Q = ctx.quantize_layer(W, H, nbits, K, L=L, full_t_update=True)
        mm = W.shape[0]
        assert torch.equal(Q, Qall[r0:r0 + mm])
        assert torch.equal(T, Tall[r0:r0 + mm])
        r0 += mm
    # the stacked call against the oracle: the last sweep's choices are optimal for their float64
    # targets, T^K is the least-squares refit to Q^K, and the oracle's own K sweeps on the stacked
    # matrix agree (a near-tie flip may change the earlier columns of single rows)
    W64 = Wall.cpu().numpy().astype(np.float64)
    H64 = H.cpu().numpy().astype(np.float64)
    L64 = L.cpu().numpy().astype(np.float64)
    Tprev, _ = ctx.quantize_layer(Wall, H, nbits, K - 1, L=L, full_t_update=True)
    Qh = Qall.cpu().numpy()
    _, _, viol = check_S(W64, L64, Tprev.cpu().numpy().astype(np.float64), Qh, "stacked")
    assert viol == 0
    Tref, _ = ref.update_T(W64, H64, Qh, nbits)
    err = np.abs(Tall.cpu().numpy() - Tref).max(axis=1) / np.abs(Tref).max(axis=1)
    assert err.max() <= 1e-4
    T0 = ctx.init_codebooks(Wall, nbits).cpu().numpy().astype(np.float64)
    To, Qo = ref.quantize_layer(W64, H64, T0, nbits, K, L=L64)
    same = (Qh == Qo).all(axis=1)
    print("stacked q/k/v: %d of %d rows identical to the oracle's free-running result" % (same.sum(), len(same)))
    assert same.mean() >= 0.9
    errT = np.abs(Tall.cpu().numpy()[same] - To[same]).max(axis=1) / np.abs(To[same]).max(axis=1)
    assert errT.max() <= 1e-4


# ----------------------------------------------------------------------------- seeded shape sweep
def _sweep_shapes():
    """Shapes that straddle the kernels' tile edges (16-row slabs, 64-column blocks, 128 x 512
    accumulation tiles, 256-column panels) without being multiples of any of them."""
    shapes = [(1, 2, 1), (15, 63, 4), (17, 66, 3), (31, 127, 2), (100, 255, 4), (129, 258, 3),
              (260, 513, 4), (17, 640, 2), (31, 777, 3), (129, 777, 4), (260, 66, 1)]
    return [(m, n, nbits, 37 * i + 1) for i, (m, n, nbits) in enumerate(shapes)]


@pytest.mark.parametrize("m,n,nbits,seed", _sweep_shapes())
def test_pipeline_shape_sweep(ctx, m, n, nbits, seed):
    """Two iterations of the whole path on an odd shape; each stage against the float64 definition."""
    W, X = make_problem(m, n, 3 * n + 40, nbits, seed=seed)
    Wg = W.cuda()
    H = ctx.build_hessian(X.cuda())
    check_H(H.cpu().numpy().astype(np.float64), ref.build_hessian(X.numpy()), X.shape[1], "sweep")
    L, info = ctx.cholesky(H)
    assert info == 0
    H64 = H.cpu().numpy().astype(np.float64)
    L64 = L.cpu().numpy().astype(np.float64)
    W64 = W.numpy().astype(np.float64)
    Lref = np.linalg.cholesky(H64)
    assert np.linalg.norm(L64 - Lref) <= 1e-4 * np.linalg.norm(Lref)
    assert not np.any(np.triu(L64, 1))
    T1, _ = ctx.quantize_layer(Wg, H, nbits, 1, L=L)
    T2, Q2, hist = ctx.quantize_layer(Wg, H, nbits, 2, L=L, history=True)
    _, _, viol = check_S(W64, L64, T1.cpu().numpy().astype(np.float64), Q2.cpu().numpy(),
                         "sweep %dx%d N=%d" % (m, n, nbits))
    assert viol == 0
    Tref, _ = ref.update_T(W64, H64, Q2.cpu().numpy(), nbits, T_prev=T1.cpu().numpy().astype(np.float64))
    scale = np.maximum(np.abs(Tref).max(axis=1), 1e-300)
    assert np.all(np.abs(T2.cpu().numpy() - Tref).max(axis=1) / scale <= 1e-4)
    lref = ref.layer_loss(W64, H64, T2.cpu().numpy(), Q2.cpu().numpy())[0]
    base = float(((W64 @ H64) * W64).sum())          # ||W X||^2: the scale of fp32 noise when the fit is exact
    # (2e-7 of ||W X||^2 is the fp32 floor of the loss product when the fit is exact and lref is ~0)
    assert abs(hist[-1] - lref) <= 1e-4 * lref + 2e-7 * base
    assert hist[3] <= hist[2] * (1 + 1e-5) + 2e-7 * base
