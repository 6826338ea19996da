"""The allocation-free outlier split (ganq_outlier_split_noalloc) against the workspace-based
entry point it is a variant of: same kernels, scratch in an array of the library's device image.
Called through the C ABI on a context that never received a workspace; two calls in a row, the
second on a smaller layer (the shared array then still holds the first call's entries beyond the
second call's rows); results must be bit-identical to ganq_outlier_split and to the oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ganq_ref as ref

pytestmark = pytest.mark.gpu


def _layer(m, n, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    W = (torch.randn(m, n, generator=g) * 0.02).to(dtype)
    W[torch.rand(m, n, generator=g) < 0.01] *= 10.0
    return W


def _split_through_abi(b, ctx, fn, Wg, r, capacity):
    m, n = Wg.shape
    Wd = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    rp = torch.full((m + 1,), -1, dtype=torch.int64, device="cuda")
    col = torch.full((capacity,), -1, dtype=torch.int32, device="cuda")
    val = torch.full((capacity,), float("nan"), dtype=torch.float32, device="cuda")
    nnz = ctypes.c_int64(-1)
    st = fn(ctx.handle, b._ptr(Wg), b._dtype_code(Wg), m, n, Wg.stride(0), float(r), b._ptr(Wd), n, b._ptr(rp),
            b._ptr(col), b._ptr(val), capacity, ctypes.byref(nnz))
    assert st == b.GANQ_OK, ctx.lib.ganq_last_error(ctx.handle).decode()
    return Wd.cpu(), rp.cpu(), col.cpu()[:nnz.value], val.cpu()[:nnz.value], nnz.value


def test_noalloc_outlier_split_twice_second_call_smaller():
    from paper_2501_12956_amd import binding as b
    plain = b.Context(0)            # the existing entry point, with a workspace
    bare = b.Context(0)             # never gets a workspace
    try:
        for (m, n, r, dtype, seed) in [(300, 1000, 0.01, torch.float16, 5), (37, 300, 0.05, torch.float32, 6)]:
            W = _layer(m, n, dtype, seed)
            Wg = W.cuda()
            cap = m * (int(n * r) + 16)
            plain.reserve(m, n, 0, 4)
            want = _split_through_abi(b, plain, plain.lib.ganq_outlier_split, Wg, r, cap)
            got = _split_through_abi(b, bare, bare.lib.ganq_outlier_split_noalloc, Wg, r, cap)
            assert got[4] == want[4] > 0
            for a, c in zip(got[:4], want[:4]):
                assert torch.equal(a, c)
            # and against the oracle, exactly (no arithmetic on the values)
            Ws_ref, Wd_ref = ref.outlier_split(W.numpy().astype(np.float64), r)
            assert np.array_equal(got[0].numpy().astype(np.float64), Wd_ref)
            dense = np.zeros((m, n))
            rp = got[1].numpy()
            for i in range(m):
                dense[i, got[2].numpy()[rp[i]:rp[i + 1]]] = got[3].numpy()[rp[i]:rp[i + 1]]
            assert np.array_equal(dense, Ws_ref)
        assert bare._ws is None
        # beyond the stated maximum: a clear error, nothing launched
        nnz = ctypes.c_int64(0)
        big = torch.zeros(8, 8, device="cuda")
        st = bare.lib.ganq_outlier_split_noalloc(bare.handle, b._ptr(big), b.GANQ_F32, 65537, 8, 8, 0.1, b._ptr(big),
                                                 8, b._ptr(big), b._ptr(big), b._ptr(big), 0, ctypes.byref(nnz))
        assert st == b.GANQ_ERR_UNSUPPORTED
        assert b"65536" in bare.lib.ganq_last_error(bare.handle)
    finally:
        plain.close()
        bare.close()
