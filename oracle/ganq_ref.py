"""Float64 CPU oracle for the GANQ per-layer solver (arXiv 2501.12956).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, obviously-correct
NumPy implementation of what the GPU library computes.  It is imported only
by tests, by the smoke check and by the benchmark's CPU-baseline leg; the
product path never calls it and shares no code with it.

Every function follows one passage of the paper, cited in its docstring.
All arithmetic is float64.  Nothing here is blocked, fused or reordered
beyond what the cited definition states.

Pinned (see the CPU test-suite):
  build_hessian   direct dot products, symmetry, chunked == one-shot
  cholesky        L L^T = H', lower, positive diagonal; Remark 3.1 and
                  Appendix A modes succeed on rank-deficient input
  init_codebooks  closed form on an arithmetic progression, library quantile
  update_S        reduces to nearest rounding for diagonal H; brute-force
                  check of every column against Eq. (16) term j; exhaustive
                  search on tiny problems
  update_T        brute-force least squares on explicit X; zero gradient;
                  monotone decrease
  layer_loss      three algebraically equal forms, Eq. (1), (9), (13)
  quantize_layer  half-step monotonicity of the T-step, restartability,
                  scaling invariances
  outlier_split   hand-worked rows where floor/ceil and +-1 of either cut-off
                  position change the result; integer n r / 2 cases
  lut_storage_fraction   Table 1 printed percentages
  pack_codes      hand-written byte patterns, round trip, Table 1 byte counts
  lut_matvec      unit vectors pick single table entries, constant tables give
                  scaled sums, explicit triple loop on tiny cases
End-to-end solver outputs: parity unpinned by the paper (it prints no
solver-level numbers); only the self-consistency pins above apply.
"""
from __future__ import annotations

import numpy as np

PRECOND_NONE = 0
PRECOND_LAMBDA = 1
PRECOND_DIAGDOM = 2
PRECOND_AUTO = 3

INIT_QUANTILE_MID = 0
INIT_QUANTILE_ENDPOINTS = 1
INIT_MINMAX_GRID = 2

EMPTY_ZERO = 0
EMPTY_KEEP = 1


class NotPositiveDefinite(Exception):
    """Raised by cholesky() when the (possibly preconditioned) matrix is not PD."""


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# H = X X^T                                             Algorithm 1, Eq. (9)
# --------------------------------------------------------------------------
def build_hessian(X, chunk=None):
    """H = X X^T for X of shape (n, p) (features x tokens), Algorithm 1.

    With ``chunk`` set the token axis is summed chunk by chunk, which is the
    same sum in a different order (used for inputs too large to upcast whole).
    """
    n, p = X.shape
    if chunk is None:
        Xd = _f64(X)
        return Xd @ Xd.T
    H = np.zeros((n, n), dtype=np.float64)
    for t0 in range(0, p, chunk):
        Xc = _f64(X[:, t0:t0 + chunk])
        H += Xc @ Xc.T
    return H


# --------------------------------------------------------------------------
# Preconditioning + Cholesky          Eq. (10), Remark 3.1, Appendix A
# --------------------------------------------------------------------------
def precondition(H, mode=PRECOND_NONE, lam=0.0):
    """Matrix that is handed to the Cholesky factorisation.

    NONE    : H itself, Eq. (10).
    LAMBDA  : H + lam*I, Remark 3.1.
    DIAGDOM : H + Diag(delta), delta_i = max(sum_j |H_ij| - 2 H_ii, 1e-8)
              with the sum over the whole row (j = i included), Appendix A
              Eq. (23)-(24).
    """
    H = _f64(H)
    if mode == PRECOND_NONE:
        return H.copy()
    if mode == PRECOND_LAMBDA:
        return H + lam * np.eye(H.shape[0])
    if mode == PRECOND_DIAGDOM:
        delta = np.maximum(np.abs(H).sum(axis=1) - 2.0 * np.diag(H), 1e-8)
        return H + np.diag(delta)
    raise ValueError("unknown preconditioning mode")


def cholesky(H, mode=PRECOND_NONE, lam=0.0):
    """Lower-triangular L with L L^T = precondition(H), Eq. (10) / Eq. (24).

    AUTO tries NONE first and falls back to DIAGDOM when a pivot fails.
    Returns (L, mode_used).
    """
    if mode == PRECOND_AUTO:
        try:
            return cholesky(H, PRECOND_NONE)[0], PRECOND_NONE
        except NotPositiveDefinite:
            return cholesky(H, PRECOND_DIAGDOM)[0], PRECOND_DIAGDOM
    Hp = precondition(H, mode, lam)
    try:
        L = np.linalg.cholesky(Hp)
    except np.linalg.LinAlgError as exc:
        raise NotPositiveDefinite(str(exc)) from exc
    if not np.all(np.isfinite(L)):
        raise NotPositiveDefinite("non-finite factor")
    return L, mode


# --------------------------------------------------------------------------
# Initial codebook T^0                 Algorithm 1 input (rule: per-row quantiles)
# --------------------------------------------------------------------------
def init_codebooks(W, nbits, mode=INIT_QUANTILE_MID):
    """T^0 of shape (m, 2^nbits).  The paper takes T^0 as an input of
    Algorithm 1 and does not say how it is built; the rule here is per-row
    quantiles of W.

    QUANTILE_MID       level s sits at quantile (s + 1/2) / C
    QUANTILE_ENDPOINTS level s sits at quantile s / (C - 1)
    MINMAX_GRID        C equally spaced values from the row min to the row max
    Quantiles use linear interpolation between order statistics:
    h = q (n - 1), value = w_(floor h) + (h - floor h)(w_(floor h + 1) - w_(floor h)).
    """
    W = _f64(W)
    m, n = W.shape
    C = 1 << nbits
    T = np.empty((m, C), dtype=np.float64)
    Ws = np.sort(W, axis=1)
    for s in range(C):
        if mode == INIT_MINMAX_GRID:
            frac = s / (C - 1) if C > 1 else 0.0
            T[:, s] = Ws[:, 0] + frac * (Ws[:, n - 1] - Ws[:, 0])
            continue
        if mode == INIT_QUANTILE_MID:
            q = (s + 0.5) / C
        elif mode == INIT_QUANTILE_ENDPOINTS:
            q = s / (C - 1) if C > 1 else 0.5
        else:
            raise ValueError("unknown init mode")
        h = q * (n - 1)
        lo = int(np.floor(h))
        hi = min(lo + 1, n - 1)
        T[:, s] = Ws[:, lo] + (h - lo) * (Ws[:, hi] - Ws[:, lo])
    return T


# --------------------------------------------------------------------------
# S-update: back-substitution on L          Eq. (13)-(22), Algorithm 1 inner loop
# --------------------------------------------------------------------------
def update_S(W, L, T):
    """Column-sequential assignment update, all rows at once.

    For j = n-1 down to 0 (Eq. (22)):
        tgt_i = W_ij + (sum_{u>j} r_iu L_uj) / L_jj,   r_iu = W_iu - T_i[Q_iu]
        Q_ij  = argmin_s |tgt_i - T_is|                (ties: lowest s)
    Returns (Q uint8 (m, n), E float64 (m, n)) with E = W - T[Q].
    The residuals are kept transposed (n, m) only so that the per-column
    product is a contiguous matrix-vector product; it is the plain sum above.
    """
    W = _f64(W)
    L = _f64(L)
    T = _f64(T)
    m, n = W.shape
    Q = np.zeros((m, n), dtype=np.uint8)
    Et = np.zeros((n, m), dtype=np.float64)
    rows = np.arange(m)
    for j in range(n - 1, -1, -1):
        if j + 1 < n:
            fb = L[j + 1:, j] @ Et[j + 1:, :]
            tgt = W[:, j] + fb / L[j, j]
        else:
            tgt = W[:, j].copy()
        idx = np.argmin(np.abs(tgt[:, None] - T), axis=1)   # first minimum = lowest s
        Q[:, j] = idx
        Et[j, :] = W[:, j] - T[rows, idx]
    return Q, np.ascontiguousarray(Et.T)


def s_update_targets(W, L, T, Q):
    """Targets of Eq. (22) recomputed for a GIVEN assignment Q ("teacher
    forced"): tgt_ij uses the residuals of the columns u > j that Q itself
    fixes.  Returns (tgt, gap, best) where, for every element,
      best_ij = argmin_s |tgt_ij - T_is| (lowest s on ties) and
      gap_ij  = |tgt_ij - T_i[Q_ij]| - min_s |tgt_ij - T_is|  (>= 0; 0 iff Q_ij
                attains the minimum of the j-th squared term of Eq. (16)).
    """
    W = _f64(W)
    L = _f64(L)
    T = _f64(T)
    m, n = W.shape
    E = W - np.take_along_axis(T, Q.astype(np.int64), axis=1)
    Ls = np.tril(L, -1)
    tgt = W + (E @ Ls) / np.diag(L)[None, :]
    d = np.abs(tgt[:, :, None] - T[:, None, :])
    best = np.argmin(d, axis=2)
    dq = np.take_along_axis(d, Q.astype(np.int64)[:, :, None], axis=2)[:, :, 0]
    gap = dq - d.min(axis=2)
    return tgt, gap, best.astype(np.uint8)


# --------------------------------------------------------------------------
# T-update: closed-form least squares        Eq. (4)-(7), Algorithm 1 batch update
# --------------------------------------------------------------------------
def one_hot(q_row, C):
    """S_i of Eq. (2): (C, n), column j has its single 1 in row q_row[j]."""
    n = q_row.shape[0]
    S = np.zeros((C, n), dtype=np.float64)
    S[q_row.astype(np.int64), np.arange(n)] = 1.0
    return S


def update_T(W, H, Q, nbits, T_prev=None, empty=EMPTY_ZERO):
    """T_i = W_i H S_i^T (S_i H S_i^T)^dagger for every row, Eq. (7).

    The dagger is the Moore-Penrose inverse.  A code that no column of row i
    uses gives a zero row/column in S_i H S_i^T, so the pseudo-inverse returns
    0 for it (EMPTY_ZERO, the literal reading); EMPTY_KEEP keeps the previous
    value T_prev[i, a] instead (the objective does not depend on it).
    Returns (T, empty_count) with empty_count[i] = number of unused codes.
    """
    W = _f64(W)
    H = _f64(H)
    m, n = W.shape
    C = 1 << nbits
    T = np.zeros((m, C), dtype=np.float64)
    empty_count = np.zeros(m, dtype=np.int32)
    for i in range(m):
        S = one_hot(Q[i], C)
        SH = S @ H
        A = SH @ S.T
        b = (W[i] @ H) @ S.T
        T[i] = b @ np.linalg.pinv(A, hermitian=True)
        used = S.sum(axis=1) > 0
        empty_count[i] = int(C - used.sum())
        if empty == EMPTY_KEEP and T_prev is not None:
            T[i, ~used] = _f64(T_prev)[i, ~used]
    return T, empty_count


# --------------------------------------------------------------------------
# Objective                                       Eq. (1), Eq. (9), Eq. (13)
# --------------------------------------------------------------------------
def dequantize(T, Q):
    """W~_ij = T_i[Q_ij], the constraint of Eq. (1)."""
    return np.take_along_axis(_f64(T), Q.astype(np.int64), axis=1)


def layer_loss(W, H, T, Q):
    """sum_i E_i H E_i^T with E = W - W~, Eq. (9).  Returns (total, per_row)."""
    E = _f64(W) - dequantize(T, Q)
    per_row = np.einsum("ij,ij->i", E @ _f64(H), E)
    return float(per_row.sum()), per_row


def layer_loss_direct(W, X, T, Q):
    """||W X - W~ X||_F^2 evaluated literally, Eq. (1)."""
    Xd = _f64(X)
    R = _f64(W) @ Xd - dequantize(T, Q) @ Xd
    return float((R * R).sum())


def layer_loss_chol(W, L, T, Q):
    """||(W - W~) L||_F^2, Eq. (13)."""
    R = (_f64(W) - dequantize(T, Q)) @ _f64(L)
    return float((R * R).sum())


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------
def quantize_layer(W, H, T0, nbits, iters, L=None, precond=PRECOND_NONE, lam=0.0,
                   empty=EMPTY_ZERO, history=False):
    """K alternations of (S-update against T^k, T-update refit to S^{k+1}),
    Algorithm 1.  L comes from the (possibly preconditioned) matrix; the
    T-update and the loss use the raw H.  Returns (T^K, Q^K[, losses]) where
    losses[0] is unavailable before the first S-step and is reported as the
    loss of nearest rounding onto T^0, losses[2k+1] after the S-step of sweep
    k and losses[2k+2] after its T-step.
    """
    W = _f64(W)
    H = _f64(H)
    if L is None:
        L, _ = cholesky(H, precond, lam)
    T = _f64(T0).copy()
    m, n = W.shape
    Q = np.zeros((m, n), dtype=np.uint8)
    losses = []
    if history:
        Q0 = np.argmin(np.abs(W[:, :, None] - T[:, None, :]), axis=2).astype(np.uint8)
        losses.append(layer_loss(W, H, T, Q0)[0])
    for _ in range(iters):
        Q, _E = update_S(W, L, T)
        if history:
            losses.append(layer_loss(W, H, T, Q)[0])
        T, _cnt = update_T(W, H, Q, nbits, T_prev=T, empty=empty)
        if history:
            losses.append(layer_loss(W, H, T, Q)[0])
    if history:
        return T, Q, losses
    return T, Q


# --------------------------------------------------------------------------
# Outlier split                                   Appendix B, Algorithm 2
# --------------------------------------------------------------------------
def outlier_cutoff_positions(n, r):
    """Sorted positions (lower, upper) of the two cut-offs of Algorithm 2:
    lower = ceil(n (1 - p)) and upper = floor(n p) with p = 1 - r/2, i.e.
    ceil(n r / 2) and floor(n - n r / 2) as real-number expressions.  They are
    evaluated from x = n r / 2 so that 1 - (1 - r/2) is never formed in floating
    point, and x is taken as an integer when it is one up to rounding (within
    1e-9 relative): n = 2000, r = 0.01 gives positions 10 and 1990.  The upper
    position is clamped to n - 1 (r = 0 would index past the row)."""
    x = n * (0.5 * r)
    k = float(np.round(x))
    if abs(x - k) <= 1e-9 * max(1.0, abs(x)):
        x = k
    lower = int(np.ceil(x))
    upper = min(int(np.floor(n - x)), n - 1)
    return lower, upper


def outlier_split(W, r):
    """W = W_sparse + W_dense, Algorithm 2: per row, entries at or beyond the
    symmetric tail cut-offs (the values at the sorted positions of
    outlier_cutoff_positions; comparisons are >= and <=) go to W_sparse, the
    rest to W_dense.
    """
    W = _f64(W)
    m, n = W.shape
    lower, upper = outlier_cutoff_positions(n, r)
    Ws = np.sort(W, axis=1)
    c_up = Ws[:, upper][:, None]
    c_lo = Ws[:, lower][:, None]
    mask = (W >= c_up) | (W <= c_lo)
    W_sparse = W * mask
    return W_sparse, W - W_sparse


# --------------------------------------------------------------------------
# Storage model                                                     Table 1
# --------------------------------------------------------------------------
def lut_storage_fraction(m, n, nbits=4, lut_bytes_per_entry=2):
    """Bytes of (N-bit Q + fp16 codebook) over bytes of fp16 W, Table 1:
    (N/8 m n + 2 * 2^N m) / (2 m n); 0.5mn + 32m at 4 bits."""
    q_bytes = nbits / 8.0 * m * n
    t_bytes = lut_bytes_per_entry * (1 << nbits) * m
    return (q_bytes + t_bytes) / (2.0 * m * n)


def uniform_storage_fraction(m, n, nbits=4):
    """Per-channel uniform quantisation (fp16 scale + zero point per row),
    Table 1: (0.5mn + 4m) / (2mn) at 4 bits."""
    return (nbits / 8.0 * m * n + 4.0 * m) / (2.0 * m * n)


# --------------------------------------------------------------------------
# Deployment format and LUT-based product      Table 1, Figure 1(a), Section 4.4
# --------------------------------------------------------------------------
def packed_row_bytes(n, nbits):
    """Bytes of one row of N-bit codes: ceil(n N / 8) (0.5 n at 4 bits, Table 1)."""
    return (n * nbits + 7) // 8


def pack_codes(Q, nbits):
    """Row i of Q as a little-endian bit stream: code j occupies bits
    [N j, N j + N) of the row, bit b of the stream being bit (b mod 8) of byte
    b // 8; the last byte is padded with zero bits.  Returns uint8 (m, ceil(nN/8))."""
    Q = np.asarray(Q)
    m, n = Q.shape
    assert Q.max(initial=0) < (1 << nbits)
    bits = ((Q.astype(np.int64)[:, :, None] >> np.arange(nbits)) & 1).astype(np.uint8)
    return np.packbits(bits.reshape(m, n * nbits), axis=1, bitorder="little")


def unpack_codes(P, n, nbits):
    """Inverse of pack_codes."""
    P = np.asarray(P, dtype=np.uint8)
    bits = np.unpackbits(P, axis=1, bitorder="little")[:, : n * nbits]
    bits = bits.reshape(P.shape[0], n, nbits).astype(np.int64)
    return (bits << np.arange(nbits)).sum(axis=2).astype(np.uint8)


def lut_table_fp16(T):
    """The stored per-row table: T rounded to fp16 (2 bytes per entry, Table 1)."""
    return np.asarray(T, dtype=np.float64).astype(np.float16)


def lut_matvec(T16, Q, x, W_sparse=None):
    """y_i = sum_j T16_i[Q_ij] x_j (+ (W_sparse x)_i): the look-up-table product
    of Figure 1(a) for one activation vector (batch 1, Section 4.4), with the
    outlier part of GANQ* added as a separate sparse product.  T16 holds the
    fp16 table values, x the fp16 activations; the sums are float64."""
    Wq = dequantize(_f64(T16), Q)
    y = Wq @ _f64(x)
    if W_sparse is not None:
        y = y + _f64(W_sparse) @ _f64(x)
    return y
