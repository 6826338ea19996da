"""GPU parity of the deployment side: stored form (N-bit code stream + fp16 tables, Table 1) and
the look-up-table product for one activation vector (Figure 1(a); Section 4.4), against the
float64 definitions in oracle/.

Tolerance of the product: the kernel multiplies fp16 by fp16 (exact in fp32) and accumulates in
fp32 along a chain of at most 16 * ceil(segments / segment lanes) + 6 + 8 additions per output,
so |y - y_ref| <= chain * 2^-24 * sum_j |T_i[Q_ij] x_j|; chain <= 64 for every shape here.
Packing and table rounding are bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref
from paper_2501_12956_amd import synth

pytestmark = pytest.mark.gpu

GAMMA = 64 * 2.0 ** -24


@pytest.fixture(scope="module")
def ctx():
    from paper_2501_12956_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def random_layer(m, n, nbits, seed):
    rng = np.random.default_rng(seed)
    C = 1 << nbits
    T = np.sort(rng.standard_normal((m, C)) * 0.02, axis=1).astype(np.float32)
    # a skewed code distribution, as a solver produces: central codes more frequent
    pr = np.exp(-0.5 * ((np.arange(C) - (C - 1) / 2) / (C / 4)) ** 2)
    Q = rng.choice(C, size=(m, n), p=pr / pr.sum()).astype(np.uint8)
    x = rng.standard_normal(n).astype(np.float16)
    return T, Q, x


def check_product(y, T16, Q, x, Ws=None, rows=None):
    yref = ref.lut_matvec(T16, Q, x, Ws)
    mag = np.abs(ref.dequantize(T16.astype(np.float64), Q)) @ np.abs(x.astype(np.float64))
    if Ws is not None:
        mag = mag + np.abs(Ws) @ np.abs(x.astype(np.float64))
    err = np.abs(y - yref)
    worst = float((err / np.maximum(mag, 1e-300)).max())
    assert np.all(err <= GAMMA * mag + 1e-30), worst
    return worst


@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
@pytest.mark.parametrize("m,n", [(5, 1), (3, 31), (7, 32), (4, 33), (9, 300), (2, 8200)])
def test_pack_layer_is_bit_exact(ctx, m, n, nbits):
    T, Q, _ = random_layer(m, n, nbits, 100 * nbits + n)
    T[0, 0] = 65504.0 * 0.999          # near the fp16 maximum
    T[m - 1, -1] = 3.0e-6              # fp16 subnormal range
    packed, lut = ctx.pack_layer(torch.from_numpy(Q).cuda(), torch.from_numpy(T).cuda(), nbits)
    P = packed.cpu().numpy()
    Pref = ref.pack_codes(Q, nbits)
    assert P.shape[1] % 16 == 0 and P.shape[1] >= Pref.shape[1]
    assert np.array_equal(P[:, :Pref.shape[1]], Pref)
    assert not P[:, Pref.shape[1]:].any()
    assert np.array_equal(lut.cpu().numpy().view(np.uint16), ref.lut_table_fp16(T).view(np.uint16))


@pytest.mark.parametrize("m,n,nbits", [(1, 1, 2), (37, 300, 4), (16, 2048, 3), (50, 2049, 4), (33, 4100, 3),
                                       (130, 5000, 2), (20, 9000, 4), (17, 20000, 3), (40, 16384, 1),
                                       (260, 777, 4)])
def test_lut_gemv_matches_oracle(ctx, m, n, nbits):
    T, Q, x = random_layer(m, n, nbits, 7 * m + n)
    packed, lut = ctx.pack_layer(torch.from_numpy(Q).cuda(), torch.from_numpy(T).cuda(), nbits)
    xg = torch.from_numpy(x).cuda()
    y = ctx.lut_gemv(packed, lut, nbits, n, xg)
    y2 = ctx.lut_gemv(packed, lut, nbits, n, xg)
    assert torch.equal(y, y2)                                   # bit-reproducible
    worst = check_product(y.cpu().numpy().astype(np.float64), lut.cpu().numpy(), Q, x)
    print("lut_gemv %dx%d N=%d: max |dy| / sum|terms| = %.2e (bound %.2e)" % (m, n, nbits, worst, GAMMA))


def test_lut_gemv_unit_vectors_pick_table_entries(ctx):
    # x = e_j returns the table entry of column j exactly, for columns around every group edge
    m, n, nbits = 19, 4200, 3
    T, Q, _ = random_layer(m, n, nbits, 5)
    packed, lut = ctx.pack_layer(torch.from_numpy(Q).cuda(), torch.from_numpy(T).cuda(), nbits)
    L16 = lut.cpu().numpy()
    for j in (0, 1, 9, 10, 11, 20, 21, 31, 32, 2047, 2048, 4095, 4096, n - 1):
        x = np.zeros(n, dtype=np.float16)
        x[j] = 1
        y = ctx.lut_gemv(packed, lut, nbits, n, torch.from_numpy(x).cuda()).cpu().numpy()
        assert np.array_equal(y, L16[np.arange(m), Q[:, j]].astype(np.float32)), j


@pytest.mark.parametrize("nbits", [3, 4])
def test_quantize_split_pack_and_multiply(ctx, nbits):
    """GANQ* end to end on a small layer: outlier split, solver on the dense part, stored form,
    product with the sparse part; against the oracle on the GPU's (T, Q, W_sparse)."""
    cfg = synth.scaled_config(synth.CONFIGS["c1"], m=96, n=320, p=1536, nbits=nbits)
    W, X = synth.make_layer(cfg, 3)
    Wg = W.cuda()
    H = ctx.build_hessian(X.cuda())
    Wd, row_ptr, col, val = ctx.outlier_split(Wg, 0.02)
    T, Q = ctx.quantize_layer(Wd, H, nbits, 3)
    packed, lut = ctx.pack_layer(Q, T, nbits)
    x = X[:, 5].contiguous().cuda().half()
    y = ctx.lut_gemv(packed, lut, nbits, cfg.n, x, outliers=(row_ptr, col, val))
    Ws = (Wg.float() - Wd).cpu().numpy().astype(np.float64)
    assert int((Ws != 0).sum()) == col.numel() > 0
    check_product(y.cpu().numpy().astype(np.float64), lut.cpu().numpy(), Q.cpu().numpy(), x.cpu().numpy(), Ws)
    # and it approximates the full-precision layer output: the point of the whole exercise
    yfull = W.numpy().astype(np.float64) @ x.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(y.cpu().numpy() - yfull) / np.linalg.norm(yfull)
    print("GANQ* N=%d: |y - W x| / |W x| = %.3e" % (nbits, rel))
    assert rel < (0.2 if nbits == 3 else 0.1)


@pytest.mark.parametrize("name,nbits", [("c3", 4), ("c3", 3), ("c5", 4)])
def test_lut_gemv_full_size(ctx, name, nbits):
    """Layer shapes of the workload list, in the launch configuration the timing uses; 48 sampled
    rows against the oracle, every row finite, two calls identical."""
    cfg = synth.CONFIGS[name]
    m, n = cfg.m, cfg.n
    C = 1 << nbits
    g = torch.Generator(device="cuda").manual_seed(1)
    Q = torch.randint(0, C, (m, n), dtype=torch.uint8, device="cuda", generator=g)
    T = (torch.randn(m, C, device="cuda", generator=g) * 0.02).sort(dim=1).values.contiguous()
    x = torch.randn(n, device="cuda", generator=g).half()
    packed, lut = ctx.pack_layer(Q, T, nbits)
    assert packed.shape[1] == n * nbits // 8           # Table 1: N/8 bytes per weight, no padding at these n
    y = ctx.lut_gemv(packed, lut, nbits, n, x)
    assert torch.equal(y, ctx.lut_gemv(packed, lut, nbits, n, x))
    assert bool(torch.isfinite(y).all())
    rows = np.sort(np.random.default_rng(2).choice(m, size=48, replace=False))
    rt = torch.from_numpy(rows).cuda()
    Pr = packed[rt].cpu().numpy()
    assert np.array_equal(Pr, ref.pack_codes(Q[rt].cpu().numpy(), nbits))
    worst = check_product(y[rt].cpu().numpy().astype(np.float64), lut[rt].cpu().numpy(), Q[rt].cpu().numpy(),
                          x.cpu().numpy())
    print("%s N=%d full size: max |dy| / sum|terms| = %.2e" % (name, nbits, worst))


def test_lut_gemv_strided_storage_unaligned_x_and_empty_outlier_rows(ctx):
    """Rows of the stored form further apart than their bytes, an activation vector that is only
    2-byte aligned (the lanes then fetch it element by element) and CSR rows without entries."""
    m, n, nbits = 21, 2100, 4
    T, Q, x = random_layer(m, n, nbits, 77)
    packed, lut = ctx.pack_layer(torch.from_numpy(Q).cuda(), torch.from_numpy(T).cuda(), nbits)
    rb = packed.shape[1]
    wide = torch.zeros(m, rb + 48, dtype=torch.uint8, device="cuda")
    wide[:, :rb] = packed
    xbuf = torch.zeros(n + 1, dtype=torch.float16, device="cuda")
    xbuf[1:] = torch.from_numpy(x).cuda()
    rng = np.random.default_rng(4)
    Ws = np.zeros((m, n))
    for i in (0, 5, 20):                                   # all other rows have no outliers
        cols = rng.choice(n, size=70, replace=False)       # more than one wavefront pass
        Ws[i, cols] = rng.standard_normal(70)
    Ws = Ws.astype(np.float32)
    nz = [np.flatnonzero(Ws[i]) for i in range(m)]
    row_ptr = torch.tensor(np.concatenate([[0], np.cumsum([len(c) for c in nz])]), dtype=torch.int64).cuda()
    col = torch.tensor(np.concatenate(nz), dtype=torch.int32).cuda()
    val = torch.tensor(np.concatenate([Ws[i, c] for i, c in enumerate(nz)]), dtype=torch.float32).cuda()
    y = ctx.lut_gemv(wide[:, :rb], lut, nbits, n, xbuf[1:], outliers=(row_ptr, col, val))
    check_product(y.cpu().numpy().astype(np.float64), lut.cpu().numpy(), Q, x, Ws.astype(np.float64))
    y0 = ctx.lut_gemv(packed, lut, nbits, n, torch.from_numpy(x).cuda(), outliers=(row_ptr, col, val))
    assert torch.equal(y, y0)
