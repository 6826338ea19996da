"""Pins for the float64 CPU oracle: each test checks the oracle against
something other than itself - a definition written out as loops, a closed
form, a library routine that solves the same problem another way, an
invariant the paper's equations imply, or brute force on a tiny case.
No test here needs a GPU."""
import itertools
import os

import numpy as np
import pytest

from oracle import ganq_ref as ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_problem(m=6, n=10, p=40, nbits=2, seed=0, outlier=True):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.02, size=(m, n))
    X = rng.normal(0, 1, size=(n, p))
    if outlier:
        X[1] *= 20.0
    H = X @ X.T
    T0 = ref.init_codebooks(W, nbits)
    return W, X, H, T0


# ------------------------------------------------------------------ H
def test_hessian_entries_are_dot_products():
    rng = np.random.default_rng(1)
    X = rng.normal(size=(7, 33))
    H = ref.build_hessian(X)
    for j in range(7):
        for k in range(7):
            acc = 0.0
            for t in range(33):
                acc += X[j, t] * X[k, t]
            assert abs(H[j, k] - acc) <= 1e-12 * max(1.0, abs(acc))
    assert np.array_equal(H, H.T)
    assert np.all(np.linalg.eigvalsh(H) > -1e-9)


def test_hessian_chunked_equals_one_shot_and_fp16_upcast():
    rng = np.random.default_rng(2)
    X = rng.normal(size=(9, 100)).astype(np.float16)
    H1 = ref.build_hessian(X)
    H2 = ref.build_hessian(X, chunk=17)
    assert np.allclose(H1, H2, rtol=1e-13, atol=0)
    # the stored fp16 values are upcast, not re-rounded
    assert np.allclose(H1, X.astype(np.float64) @ X.astype(np.float64).T, rtol=1e-13)


# ------------------------------------------------------------------ L
def test_cholesky_reconstructs_and_is_lower():
    _, _, H, _ = small_problem(n=12, p=60)
    L, mode = ref.cholesky(H)
    assert mode == ref.PRECOND_NONE
    assert np.linalg.norm(L @ L.T - H) <= 1e-12 * np.linalg.norm(H)
    assert np.array_equal(L, np.tril(L))
    assert np.all(np.diag(L) > 0)
    # first column has the textbook closed form L[:,0] = H[:,0]/sqrt(H00)
    assert np.allclose(L[:, 0], H[:, 0] / np.sqrt(H[0, 0]), rtol=1e-13)


def test_cholesky_2x2_closed_form():
    H = np.array([[4.0, 2.0], [2.0, 10.0]])
    L, _ = ref.cholesky(H)
    assert np.allclose(L, [[2.0, 0.0], [1.0, 3.0]])


def test_rank_deficient_needs_preconditioning():
    rng = np.random.default_rng(3)
    X = rng.normal(size=(12, 5))          # p < n: X X^T is singular
    H = X @ X.T
    with pytest.raises(ref.NotPositiveDefinite):
        ref.cholesky(H, ref.PRECOND_NONE)
    # Remark 3.1: v^T (H + lam I) v = |X^T v|^2 + lam |v|^2 > 0
    L, _ = ref.cholesky(H, ref.PRECOND_LAMBDA, lam=0.5)
    assert np.linalg.norm(L @ L.T - (H + 0.5 * np.eye(12))) <= 1e-12 * np.linalg.norm(H)
    # Appendix A: diagonal dominance
    Hp = ref.precondition(H, ref.PRECOND_DIAGDOM)
    off = np.abs(Hp).sum(axis=1) - np.abs(np.diag(Hp))
    assert np.all(np.diag(Hp) > 0)
    assert np.all(np.diag(Hp) >= off - 1e-9 * np.abs(np.diag(Hp)))
    L, _ = ref.cholesky(H, ref.PRECOND_DIAGDOM)
    assert np.linalg.norm(L @ L.T - Hp) <= 1e-12 * np.linalg.norm(Hp)
    # AUTO = NONE, then DIAGDOM on failure
    L2, used = ref.cholesky(H, ref.PRECOND_AUTO)
    assert used == ref.PRECOND_DIAGDOM and np.array_equal(L2, L)


def test_diagdom_delta_formula_by_hand():
    H = np.array([[2.0, -3.0, 1.0], [-3.0, 10.0, 0.5], [1.0, 0.5, 1.0]])
    # delta_i = max(sum_j |H_ij| - 2 H_ii, 1e-8), sum over the whole row
    expect = np.array([max(6.0 - 4.0, 1e-8), max(13.5 - 20.0, 1e-8), max(2.5 - 2.0, 1e-8)])
    Hp = ref.precondition(H, ref.PRECOND_DIAGDOM)
    assert np.array_equal(np.diag(Hp), np.diag(H) + expect)
    # the diagonally dominant row gets the floor of Eq. (23), not zero
    assert Hp[1, 1] == 10.0 + 1e-8 and Hp[1, 1] > 10.0
    assert np.array_equal(Hp - np.diag(np.diag(Hp)), H - np.diag(np.diag(H)))


# ------------------------------------------------------------------ T^0
def test_init_codebooks_closed_form_on_arange():
    n, nbits = 101, 3
    C = 8
    W = np.arange(n, dtype=np.float64)[None, :].repeat(2, axis=0)
    W[1] = W[1][::-1] * 2.0                      # order of the input must not matter
    T = ref.init_codebooks(W, nbits)
    expect = (np.arange(C) + 0.5) / C * (n - 1)
    assert np.allclose(T[0], expect, rtol=1e-14)
    assert np.allclose(T[1], 2.0 * expect, rtol=1e-14)


def test_init_codebooks_matches_library_quantile_and_is_sorted():
    rng = np.random.default_rng(4)
    W = rng.standard_t(5, size=(5, 257))
    for nbits in (1, 2, 3, 4):
        C = 1 << nbits
        T = ref.init_codebooks(W, nbits, ref.INIT_QUANTILE_MID)
        qs = (np.arange(C) + 0.5) / C
        assert np.allclose(T, np.quantile(W, qs, axis=1, method="linear").T, rtol=1e-13)
        assert np.all(np.diff(T, axis=1) >= 0)
        Te = ref.init_codebooks(W, nbits, ref.INIT_QUANTILE_ENDPOINTS)
        assert np.allclose(Te[:, 0], W.min(axis=1)) and np.allclose(Te[:, -1], W.max(axis=1))
        Tg = ref.init_codebooks(W, nbits, ref.INIT_MINMAX_GRID)
        assert np.allclose(np.diff(Tg, axis=1), (W.max(1) - W.min(1))[:, None] / (C - 1))


# ------------------------------------------------------------------ T-update
def test_update_T_equals_brute_force_least_squares():
    """Eq. (4): T_i minimises |W_i X - T_i S_i X|^2, a linear least-squares
    problem in T_i with design matrix (S_i X)^T."""
    W, X, H, T0 = small_problem(m=5, n=14, p=50, nbits=2, seed=5)
    rng = np.random.default_rng(55)
    Q = rng.integers(0, 4, size=W.shape).astype(np.uint8)
    T, cnt = ref.update_T(W, H, Q, 2)
    for i in range(W.shape[0]):
        S = np.zeros((4, W.shape[1]))
        for j in range(W.shape[1]):
            S[Q[i, j], j] = 1.0
        t_ls, *_ = np.linalg.lstsq((S @ X).T, (W[i] @ X), rcond=None)
        assert np.allclose(T[i], t_ls, rtol=1e-9, atol=1e-14)
        # Eq. (6): gradient vanishes
        grad = 2.0 * (W[i] @ X - T[i] @ S @ X) @ X.T @ S.T
        assert np.linalg.norm(grad) <= 1e-9 * np.linalg.norm(W[i] @ H)
    assert np.all(cnt == 0)


def test_update_T_never_increases_loss_and_beats_perturbations():
    W, X, H, T0 = small_problem(m=8, n=20, p=80, nbits=3, seed=6)
    L, _ = ref.cholesky(H)
    Q, _ = ref.update_S(W, L, T0)
    before = ref.layer_loss(W, H, T0, Q)[1]
    T1, _ = ref.update_T(W, H, Q, 3, T_prev=T0)
    after = ref.layer_loss(W, H, T1, Q)[1]
    assert np.all(after <= before * (1 + 1e-12) + 1e-18)
    rng = np.random.default_rng(66)
    for _ in range(5):
        Tp = T1 + 1e-3 * np.abs(T1).max() * rng.normal(size=T1.shape)
        assert np.all(ref.layer_loss(W, H, Tp, Q)[1] >= after * (1 - 1e-12))


def test_update_T_identity_hessian_gives_cluster_means_and_empty_rules():
    # With H = I, Eq. (7) reduces to the mean of each cluster (one weight per
    # code -> that weight itself).
    W = np.array([[0.3, -1.0, 2.0, 0.5], [1.0, 1.0, 3.0, 5.0]])
    Q = np.array([[2, 0, 3, 1], [0, 0, 3, 3]], dtype=np.uint8)
    T, cnt = ref.update_T(W, np.eye(4), Q, 2)
    assert np.allclose(T[0], [-1.0, 0.5, 0.3, 2.0])
    assert np.allclose(T[1], [1.0, 0.0, 0.0, 4.0])      # codes 1, 2 unused -> 0 (pseudo-inverse)
    assert list(cnt) == [0, 2]
    Tprev = np.full((2, 4), 7.0)
    Tk, _ = ref.update_T(W, np.eye(4), Q, 2, T_prev=Tprev, empty=ref.EMPTY_KEEP)
    assert np.allclose(Tk[1], [1.0, 7.0, 7.0, 4.0])


# ------------------------------------------------------------------ S-update
def nearest_lowest(t_row, x):
    best, bd = 0, abs(x - t_row[0])
    for s in range(1, len(t_row)):
        d = abs(x - t_row[s])
        if d < bd:
            best, bd = s, d
    return best


def test_update_S_diagonal_H_is_nearest_rounding():
    rng = np.random.default_rng(7)
    W = rng.normal(size=(6, 15))
    T = np.sort(rng.normal(size=(6, 4)), axis=1)
    L = np.diag(rng.uniform(0.5, 3.0, size=15))
    Q, E = ref.update_S(W, L, T)
    for i in range(6):
        for j in range(15):
            assert Q[i, j] == nearest_lowest(T[i], W[i, j])
            assert E[i, j] == W[i, j] - T[i, Q[i, j]]


def test_update_S_every_column_minimises_its_term_of_eq16():
    """Independent loops for Eq. (16): term_j(s) = (sum_{u>=j} r_u L_uj)^2 with
    r_j = W_ij - T_is; the chosen code must minimise it given later columns,
    and the last column must be plain nearest rounding (Eq. (18))."""
    W, X, H, T0 = small_problem(m=4, n=9, p=30, nbits=2, seed=8)
    L, _ = ref.cholesky(H)
    Q, E = ref.update_S(W, L, T0)
    m, n = W.shape
    for i in range(m):
        assert Q[i, n - 1] == nearest_lowest(T0[i], W[i, n - 1])
        for j in range(n):
            tail = 0.0
            for u in range(j + 1, n):
                tail += (W[i, u] - T0[i, Q[i, u]]) * L[u, j]
            terms = [((W[i, j] - T0[i, s]) * L[j, j] + tail) ** 2 for s in range(4)]
            assert terms[Q[i, j]] <= min(terms) * (1 + 1e-12) + 1e-30
    # Eq. (13)-(16): the terms add up to E H E^T
    total = 0.0
    for i in range(m):
        for j in range(n):
            acc = 0.0
            for u in range(j, n):
                acc += E[i, u] * L[u, j]
            total += acc * acc
    assert np.isclose(total, ref.layer_loss(W, H, T0, Q)[0], rtol=1e-10)


def test_update_S_uses_column_of_L_not_row():
    """A hand-built 2-column case where using L[j, u] instead of L[u, j], or a
    wrong sign on the feedback, picks a different code."""
    L = np.array([[1.0, 0.0], [0.8, 1.0]])
    T = np.array([[0.0, 1.0]])
    W = np.array([[0.45, 0.3]])
    # column 1: nearest of 0.3 -> code 0, residual r = 0.3
    # column 0: target = 0.45 + 0.3 * L[1,0] / L[0,0] = 0.69 -> code 1
    Q, E = ref.update_S(W, L, T)
    assert list(Q[0]) == [1, 0]
    assert np.allclose(E[0], [0.45 - 1.0, 0.3])


def test_update_S_exact_representation_gives_zero_error():
    rng = np.random.default_rng(9)
    T = np.array([[-1.0, -0.25, 0.5, 2.0]])
    W = T[0][rng.integers(0, 4, size=(1, 12))]
    X = rng.normal(size=(12, 40))
    L, _ = ref.cholesky(X @ X.T)
    Q, E = ref.update_S(W, L, T)
    assert np.all(E == 0.0)
    assert ref.layer_loss(W, X @ X.T, T, Q)[0] == 0.0


def test_update_S_ties_pick_lowest_index():
    T = np.array([[0.0, 1.0, 1.0, 0.0]])           # duplicates on purpose
    W = np.array([[0.5, 0.9, 0.1]])
    Q, _ = ref.update_S(W, np.eye(3), T)
    assert list(Q[0]) == [0, 1, 0]


def test_greedy_is_bounded_by_exhaustive_optimum_on_tiny_problems():
    for seed in range(4):
        W, X, H, T0 = small_problem(m=2, n=5, p=12, nbits=2, seed=20 + seed)
        L, _ = ref.cholesky(H)
        Q, _ = ref.update_S(W, L, T0)
        greedy = ref.layer_loss(W, H, T0, Q)[1]
        for i in range(2):
            best = np.inf
            for assign in itertools.product(range(4), repeat=5):
                e = W[i] - T0[i, list(assign)]
                best = min(best, e @ H @ e)
            assert greedy[i] >= best * (1 - 1e-12)
    # n = 1: the greedy choice is the optimum
    W = np.array([[0.37]])
    T = np.array([[0.0, 0.3, 0.5, 1.0]])
    Q, _ = ref.update_S(W, np.array([[2.0]]), T)
    assert Q[0, 0] == 1


def test_teacher_forced_targets_reproduce_update_S():
    W, X, H, T0 = small_problem(m=5, n=16, p=64, nbits=3, seed=10)
    L, _ = ref.cholesky(H)
    Q, _ = ref.update_S(W, L, T0)
    tgt, gap, best = ref.s_update_targets(W, L, T0, Q)
    assert np.array_equal(best, Q)
    assert np.all(gap == 0.0)
    # flipping one code must show up as a positive gap at that element
    Q2 = Q.copy()
    Q2[2, 7] = (Q2[2, 7] + 1) % 8
    _, gap2, _ = ref.s_update_targets(W, L, T0, Q2)
    assert gap2[2, 7] > 0


# ------------------------------------------------------------------ loss
def test_three_forms_of_the_loss_agree():
    W, X, H, T0 = small_problem(m=7, n=18, p=70, nbits=3, seed=11)
    L, _ = ref.cholesky(H)
    Q, _ = ref.update_S(W, L, T0)
    a = ref.layer_loss(W, H, T0, Q)[0]
    b = ref.layer_loss_direct(W, X, T0, Q)
    c = ref.layer_loss_chol(W, L, T0, Q)
    assert np.isclose(a, b, rtol=1e-10) and np.isclose(a, c, rtol=1e-10)
    # and by loops, for one row
    Wq = ref.dequantize(T0, Q)
    i = 3
    tot = 0.0
    for t in range(X.shape[1]):
        d = 0.0
        for j in range(W.shape[1]):
            d += (W[i, j] - Wq[i, j]) * X[j, t]
        tot += d * d
    assert np.isclose(tot, ref.layer_loss(W, H, T0, Q)[1][i], rtol=1e-10)


# ------------------------------------------------------------------ Algorithm 1
def test_alternation_history_and_restartability():
    W, X, H, T0 = small_problem(m=12, n=32, p=200, nbits=3, seed=12)
    T, Q, hist = ref.quantize_layer(W, H, T0, 3, 6, history=True)
    assert len(hist) == 13
    for k in range(6):
        assert hist[2 * k + 2] <= hist[2 * k + 1] * (1 + 1e-12)      # T-step never increases
    assert hist[-1] < hist[0]                                         # beats rounding onto T^0
    # K = 6 in one call == 3 + 3 with T carried over (S^0 is never read)
    Ta, Qa = ref.quantize_layer(W, H, T0, 3, 3)
    Tb, Qb = ref.quantize_layer(W, H, Ta, 3, 3)
    assert np.array_equal(Qb, Q) and np.array_equal(Tb, T)
    # returned Q was chosen against T^{K-1}; T^K is refit to it
    Tc, _ = ref.update_T(W, H, Q, 3)
    assert np.allclose(Tc, T, rtol=1e-12, atol=0)


@pytest.mark.parametrize("mode,lam", [(ref.PRECOND_DIAGDOM, 0.0), (ref.PRECOND_LAMBDA, 3.0),
                                      (ref.PRECOND_AUTO, 0.0)])
def test_preconditioned_run_refits_codebooks_on_the_raw_hessian(mode, lam):
    """Reading of Algorithm 1 with Appendix A: the factor L of the S-update comes from the
    preconditioned matrix, while the T-update (Eq. (4)-(7)) and the objective (Eq. (1)) keep the
    raw H = X X^T.  So T^K must be the least-squares fit to the activations themselves - checked
    by lstsq on explicit X, not through update_T - and must differ from the fit on L L^T."""
    rng = np.random.default_rng(31)
    m, n, p, nbits = 6, 20, 14, 2                       # p < n: H is singular, NONE must fail
    W = rng.normal(0, 0.02, size=(m, n))
    X = rng.normal(0, 1, size=(n, p))
    X[2] *= 8.0
    H = X @ X.T
    T0 = ref.init_codebooks(W, nbits)
    with pytest.raises(ref.NotPositiveDefinite):
        ref.quantize_layer(W, H, T0, nbits, 2, precond=ref.PRECOND_NONE)
    T, Q, hist = ref.quantize_layer(W, H, T0, nbits, 3, precond=mode, lam=lam, history=True)
    Lp, _ = ref.cholesky(H, mode, lam)
    Hp = Lp @ Lp.T
    C = 1 << nbits
    differs = 0
    for i in range(m):
        S = np.zeros((C, n))
        S[Q[i].astype(int), np.arange(n)] = 1.0
        used = S.sum(axis=1) > 0
        t_raw = np.zeros(C)
        t_raw[used] = np.linalg.lstsq((S[used] @ X).T, W[i] @ X, rcond=None)[0]
        assert np.allclose(T[i], t_raw, rtol=1e-8, atol=1e-12)
        # the fit against the preconditioned matrix is another vector
        Xp = Lp                                          # Hp = Lp Lp^T plays X X^T
        t_pre = np.zeros(C)
        t_pre[used] = np.linalg.lstsq((S[used] @ Xp).T, W[i] @ Xp, rcond=None)[0]
        differs += int(not np.allclose(t_pre, t_raw, rtol=1e-3, atol=0))
    assert differs == m
    # the recorded objective is the raw one, Eq. (1) evaluated on X itself
    assert np.isclose(hist[-1], ref.layer_loss_direct(W, X, T, Q), rtol=1e-9)
    # and the S-update did use the preconditioned factor: every choice of the last sweep is the
    # argmin for targets built from Lp, not necessarily for targets from another factor
    Tprev, _ = ref.quantize_layer(W, H, T0, nbits, 2, precond=mode, lam=lam)
    _, gap, _ = ref.s_update_targets(W, Lp, Tprev, Q)
    assert np.all(gap == 0)


def test_scaling_invariances():
    W, X, H, T0 = small_problem(m=6, n=20, p=90, nbits=2, seed=13)
    T, Q = ref.quantize_layer(W, H, T0, 2, 3)
    # X -> cX: H -> c^2 H, L -> cL, targets unchanged
    T2, Q2 = ref.quantize_layer(W, 9.0 * H, T0, 2, 3)
    assert np.array_equal(Q, Q2) and np.allclose(T, T2, rtol=1e-10)
    # row scaling of W and T^0 (power of two: exact)
    c = np.array([1.0, 2.0, 0.5, 4.0, 1.0, 8.0])[:, None]
    T3, Q3 = ref.quantize_layer(c * W, H, c * T0, 2, 3)
    assert np.array_equal(Q, Q3) and np.allclose(T3, c * T, rtol=1e-10)


def test_config1_sized_run_reduces_loss():
    """The tiny configuration at reduced iteration count: the solver must end
    well below rounding onto the initial codebook."""
    import torch
    from paper_2501_12956_amd import synth
    cfg = synth.scaled_config(synth.CONFIGS["c1"], m=32, p=1024)
    W = synth.make_weight(cfg, 0).numpy()
    X = synth.make_activations(cfg, 0).numpy()
    H = ref.build_hessian(X)
    T0 = ref.init_codebooks(W, cfg.nbits)
    T, Q, hist = ref.quantize_layer(W, H, T0, cfg.nbits, 3, history=True)
    assert hist[-1] < 0.7 * hist[0]
    assert np.isclose(ref.layer_loss_direct(W, X, T, Q), hist[-1], rtol=1e-9)


# ------------------------------------------------------------------ Algorithm 2
def test_outlier_split_by_hand():
    # n = 8, r = 0.5: p = 0.75, upper = floor(6) = 6, lower = ceil(2) = 2
    W = np.array([[5.0, -7.0, 0.1, 0.2, -0.3, 9.0, 0.0, -4.0]])
    Ws, Wd = ref.outlier_split(W, 0.5)
    # sorted: -7 -4 -0.3 0 0.1 0.2 5 9 ; c_upper = 5, c_lower = -0.3
    assert np.array_equal(Ws, [[5.0, -7.0, 0.0, 0.0, -0.3, 9.0, 0.0, -4.0]])
    assert np.array_equal(Ws + Wd, W)
    assert np.all((Ws == 0) | (Wd == 0))


def test_outlier_split_fractional_positions_by_hand():
    """Algorithm 2 with n r / 2 not an integer: n = 10, r = 0.3, p = 0.85, n p = 8.5,
    n (1 - p) = 1.5, so upper = floor(8.5) = 8 and lower = ceil(1.5) = 2.  All values are
    distinct and non-zero, so floor <-> ceil or +-1 on either position changes the mask."""
    srt = np.array([-9.0, -7.0, -5.0, -3.0, -1.0, 1.0, 3.0, 5.0, 7.0, 9.0])
    perm = np.array([4, 9, 0, 7, 2, 5, 8, 1, 6, 3])
    W = srt[perm][None, :]
    Ws, Wd = ref.outlier_split(W, 0.3)
    # c_lower = sorted[2] = -5 (entries -9, -7, -5), c_upper = sorted[8] = 7 (entries 7, 9)
    want = np.where((W <= -5.0) | (W >= 7.0), W, 0.0)
    assert np.array_equal(Ws, want)
    assert int((Ws != 0).sum()) == 5
    assert np.array_equal(Ws + Wd, W)
    # second row shape: n = 7, r = 0.5 -> n r / 2 = 1.75: lower = 2, upper = floor(5.25) = 5
    srt = np.array([-6.0, -4.0, -2.0, 0.5, 2.0, 4.0, 6.0])
    W = srt[[3, 0, 6, 1, 5, 2, 4]][None, :]
    Ws, _ = ref.outlier_split(W, 0.5)
    assert np.array_equal(Ws, np.where((W <= -2.0) | (W >= 4.0), W, 0.0))


@pytest.mark.parametrize("n,r,lower,upper", [(2000, 0.01, 10, 1990), (1000, 0.1, 50, 950),
                                              (400, 0.07, 14, 386), (50, 0.28, 7, 43),
                                              (4096, 0.005, 11, 4085), (10, 0.3, 2, 8),
                                              (16, 0.0, 0, 15)])
def test_outlier_cutoff_positions_exact_products(n, r, lower, upper):
    """ceil(n (1 - p)) and floor(n p) as real-number expressions (Algorithm 2): when n r / 2
    is an integer the positions are that integer and n minus it, whatever the rounding of r,
    1 - r/2 or the product in binary floating point (n = 2000, r = 0.01 is 10, not 11)."""
    assert ref.outlier_cutoff_positions(n, r) == (lower, upper)
    # the count of outliers in a row of distinct values follows: positions 0..lower and upper..n-1
    W = np.arange(1, n + 1, dtype=np.float64)[None, ::-1].copy()
    Ws, _ = ref.outlier_split(W, r)
    assert int((Ws != 0).sum()) == (lower + 1) + (n - upper)


# ------------------------------------------------------------------ Table 1
def test_storage_model_matches_table1():
    with open(os.path.join(GOLDEN, "table1_storage.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for m, n, uni, lut in rows:
        m, n = int(m), int(n)
        assert round(100 * ref.uniform_storage_fraction(m, n), 2) == float(uni)
        assert round(100 * ref.lut_storage_fraction(m, n), 2) == float(lut)


# ------------------------------------------------------------------ deployment format
def test_pack_codes_hand_written_bytes():
    # 4 bits: two codes per byte, the even column in the low nibble
    P = ref.pack_codes(np.array([[0x1, 0x2, 0xF, 0x0, 0x7]], dtype=np.uint8), 4)
    assert P.tolist() == [[0x21, 0x0F, 0x07]]
    # 3 bits: 8 codes fill 3 bytes; codes 1..7,0 -> bit stream 001 010 011 100 101 110 111 000 (LSB first)
    # byte0 = c0 | c1<<3 | (c2&3)<<6 = 1 | 16 | 192 = 0xD1; byte1 = c2>>2 | c3<<1 | c4<<4 | (c5&1)<<7 = 0|8|80|0 = 0x58
    # byte2 = c5>>1 | c6<<2 | c7<<5 = 3 | 28 | 0 = 0x1F
    P = ref.pack_codes(np.array([[1, 2, 3, 4, 5, 6, 7, 0]], dtype=np.uint8), 3)
    assert P.tolist() == [[0xD1, 0x58, 0x1F]]
    # 2 bits and 1 bit
    assert ref.pack_codes(np.array([[3, 0, 1, 2, 2]], dtype=np.uint8), 2).tolist() == [[0x93, 0x02]]
    assert ref.pack_codes(np.array([[1, 0, 0, 1, 1, 1, 0, 0, 1]], dtype=np.uint8), 1).tolist() == [[0x39, 0x01]]


@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
def test_pack_codes_round_trip_and_table1_bytes(nbits):
    rng = np.random.default_rng(nbits)
    for n in (1, 7, 8, 31, 32, 33, 100):
        Q = rng.integers(0, 1 << nbits, size=(5, n)).astype(np.uint8)
        P = ref.pack_codes(Q, nbits)
        assert P.shape == (5, ref.packed_row_bytes(n, nbits))
        assert np.array_equal(ref.unpack_codes(P, n, nbits), Q)
    # Table 1: codes plus a 2-byte table entry per code value make 0.5 m n + 32 m bytes at 4 bits
    for m, n in ((2048, 2048), (4096, 4096), (8192, 8192)):
        total = m * ref.packed_row_bytes(n, 4) + m * 16 * 2
        assert total == 0.5 * m * n + 32 * m
        assert total / (2.0 * m * n) == ref.lut_storage_fraction(m, n)


def test_lut_matvec_special_cases_and_brute_force():
    rng = np.random.default_rng(3)
    m, n, nbits = 6, 19, 3
    C = 1 << nbits
    T16 = ref.lut_table_fp16(rng.normal(size=(m, C)))
    assert T16.dtype == np.float16
    Q = rng.integers(0, C, size=(m, n)).astype(np.uint8)
    # a unit vector picks one table entry per row
    for j in (0, 7, n - 1):
        e = np.zeros(n, dtype=np.float16)
        e[j] = 1
        assert np.array_equal(ref.lut_matvec(T16, Q, e), T16[np.arange(m), Q[:, j]].astype(np.float64))
    # a table constant along each row gives that constant times sum(x)
    x = rng.normal(size=n).astype(np.float16)
    Tc = np.repeat(T16[:, :1], C, axis=1)
    assert np.allclose(ref.lut_matvec(Tc, Q, x), Tc[:, 0].astype(np.float64) * x.astype(np.float64).sum(),
                       rtol=0, atol=1e-12)
    # explicit loops, with a sparse part
    Ws = np.zeros((m, n))
    Ws[1, 4], Ws[5, 0], Ws[5, 18] = 2.5, -1.25, 0.75
    y = ref.lut_matvec(T16, Q, x, Ws)
    for i in range(m):
        acc = 0.0
        for j in range(n):
            acc += float(T16[i, Q[i, j]]) * float(x[j]) + Ws[i, j] * float(x[j])
        assert abs(y[i] - acc) <= 1e-12 * max(1.0, abs(acc))
    # the product of the table look-up equals the product with the dequantised matrix of Eq. (1)
    assert np.array_equal(ref.lut_matvec(T16, Q, x), ref.dequantize(T16, Q) @ x.astype(np.float64))
