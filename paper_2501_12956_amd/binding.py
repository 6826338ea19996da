"""Thin ctypes binding over libganq.so (argument marshalling only).

Every step of the GANQ layer solver runs in the HIP kernels behind the C ABI of
``include/ganq.h``; torch is used here for device memory and the current
stream.  There is no fallback: if the library has not been built the import of
the library raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libganq.so")

GANQ_OK, GANQ_ERR_INVALID_ARG, GANQ_ERR_UNSUPPORTED, GANQ_ERR_NOT_PD, GANQ_ERR_WORKSPACE, GANQ_ERR_HIP = range(6)
GANQ_F16, GANQ_F32 = 0, 1
PRECOND_NONE, PRECOND_LAMBDA, PRECOND_DIAGDOM, PRECOND_AUTO = range(4)
INIT_QUANTILE_MID, INIT_QUANTILE_ENDPOINTS, INIT_MINMAX_GRID = range(3)
EMPTY_ZERO, EMPTY_KEEP = 0, 1

EXPORTS = ["ganq_create", "ganq_destroy", "ganq_workspace_bytes", "ganq_set_workspace",
           "ganq_status_string", "ganq_last_error", "ganq_build_hessian", "ganq_build_hessian_tokens",
           "ganq_cholesky",
           "ganq_init_codebooks", "ganq_update_S", "ganq_update_T", "ganq_update_T_prepare", "ganq_layer_loss",
           "ganq_quantize_layer", "ganq_outlier_split", "ganq_outlier_split_noalloc", "ganq_packed_row_bytes", "ganq_pack_layer",
           "ganq_lut_gemv", "ganq_profile_enable", "ganq_profile_read", "ganq_measure_peaks", "ganq_sweep_log"]

KERNEL_CLASSES = ["hessian", "cholesky", "init", "gemm_wh", "update_s", "t_prep", "t_pad", "t_accum",
                  "t_solve", "loss", "outlier", "pack", "lut_gemv", "t_delta", "t_skip"]
OPT_FULL_T_UPDATE = 1


class GanqOptions(ctypes.Structure):
    _fields_ = [("precond", ctypes.c_int), ("lambda_", ctypes.c_float), ("init", ctypes.c_int),
                ("init_codebooks", ctypes.c_int), ("empty", ctypes.c_int), ("flags", ctypes.c_int)]


class GanqError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("ganq status %d: %s" % (status, text))
        self.status = status


_lib = None


def load_library():
    """Loads libganq.so; raises if it has not been built (python -m paper_2501_12956_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libganq.so is missing: build it with `python -m paper_2501_12956_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, cf = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    lib.ganq_create.argtypes = [ctypes.POINTER(vp), ci, vp]
    lib.ganq_create.restype = ci
    lib.ganq_destroy.argtypes = [vp]
    lib.ganq_destroy.restype = ci
    lib.ganq_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.ganq_workspace_bytes.restype = ctypes.c_size_t
    lib.ganq_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.ganq_set_workspace.restype = ci
    lib.ganq_status_string.argtypes = [ci]
    lib.ganq_status_string.restype = ctypes.c_char_p
    lib.ganq_last_error.argtypes = [vp]
    lib.ganq_last_error.restype = ctypes.c_char_p
    lib.ganq_build_hessian.argtypes = [vp, vp, ci, i64, i64, i64, vp, i64, ci]
    lib.ganq_build_hessian.restype = ci
    lib.ganq_build_hessian_tokens.argtypes = [vp, vp, ci, i64, i64, i64, vp, i64, ci]
    lib.ganq_build_hessian_tokens.restype = ci
    lib.ganq_cholesky.argtypes = [vp, vp, i64, i64, ci, cf, vp, i64, ctypes.POINTER(i64)]
    lib.ganq_cholesky.restype = ci
    lib.ganq_init_codebooks.argtypes = [vp, vp, ci, i64, i64, i64, ci, ci, vp]
    lib.ganq_init_codebooks.restype = ci
    lib.ganq_packed_row_bytes.argtypes = [i64, ci]
    lib.ganq_packed_row_bytes.restype = i64
    lib.ganq_pack_layer.argtypes = [vp, vp, i64, i64, i64, vp, ci, vp, i64, vp]
    lib.ganq_pack_layer.restype = ci
    lib.ganq_lut_gemv.argtypes = [vp, vp, i64, vp, ci, i64, i64, vp, vp, vp, vp, vp]
    lib.ganq_lut_gemv.restype = ci
    lib.ganq_update_S.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, ci, vp, i64, vp, i64]
    lib.ganq_update_S.restype = ci
    lib.ganq_update_T.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, i64, ci, ci, vp, vp]
    lib.ganq_update_T.restype = ci
    lib.ganq_update_T_prepare.argtypes = [vp, vp, i64, i64, i64, vp, i64, ci]
    lib.ganq_update_T_prepare.restype = ci
    lib.ganq_layer_loss.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, vp, i64, ci,
                                    ctypes.POINTER(ctypes.c_double), vp]
    lib.ganq_layer_loss.restype = ci
    lib.ganq_quantize_layer.argtypes = [vp, vp, ci, i64, i64, i64, vp, i64, vp, i64, ci, ci,
                                        ctypes.POINTER(GanqOptions), vp, vp, i64,
                                        ctypes.POINTER(ctypes.c_double)]
    lib.ganq_quantize_layer.restype = ci
    lib.ganq_outlier_split.argtypes = [vp, vp, ci, i64, i64, i64, ctypes.c_double, vp, i64, vp, vp, vp, i64,
                                       ctypes.POINTER(i64)]
    lib.ganq_outlier_split.restype = ci
    lib.ganq_outlier_split_noalloc.argtypes = lib.ganq_outlier_split.argtypes
    lib.ganq_outlier_split_noalloc.restype = ci
    lib.ganq_profile_enable.argtypes = [vp, ci]
    lib.ganq_profile_enable.restype = ci
    lib.ganq_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.ganq_profile_read.restype = ci
    lib.ganq_sweep_log.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ci, ctypes.POINTER(ci)]
    lib.ganq_sweep_log.restype = ci
    lib.ganq_measure_peaks.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    lib.ganq_measure_peaks.restype = ci
    _lib = lib
    return lib


def _dtype_code(t):
    if t.dtype == torch.float16:
        return GANQ_F16
    if t.dtype == torch.float32:
        return GANQ_F32
    raise TypeError("expected a float16 or float32 tensor, got %s" % t.dtype)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _rowmajor(t, name):
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be a 2-D row-major tensor" % name)
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


class Context:
    """One ganq_ctx bound to a device, to torch's current stream at creation and to a
    torch-owned workspace that grows on demand."""

    def __init__(self, device=0, stream=None):
        self.lib = load_library()
        self.device = torch.device("cuda", device) if isinstance(device, int) else torch.device(device)
        dev_index = self.device.index or 0
        if stream is None and torch.cuda.is_available():
            stream = torch.cuda.current_stream(self.device).cuda_stream
        handle = ctypes.c_void_p()
        st = self.lib.ganq_create(ctypes.byref(handle), dev_index, ctypes.c_void_p(stream or 0))
        if st != GANQ_OK:
            raise GanqError(st, self.lib.ganq_status_string(st).decode())
        self.handle = handle
        self._ws = None

    def close(self):
        if getattr(self, "handle", None):
            self.lib.ganq_destroy(self.handle)
            self.handle = None
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != GANQ_OK:
            raise GanqError(st, self.lib.ganq_last_error(self.handle).decode() or
                            self.lib.ganq_status_string(st).decode())

    def reserve(self, m, n, p=0, nbits=4, extra=0):
        need = self.lib.ganq_workspace_bytes(m, n, p, nbits)
        if need == 0:
            raise ValueError("invalid shape for workspace query")
        need += extra
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            self._check(self.lib.ganq_set_workspace(self.handle, _ptr(self._ws), need))
        return need

    # ---- per-kernel-class timing ----------------------------------------
    def profile_enable(self, on=True):
        self._check(self.lib.ganq_profile_enable(self.handle, int(on)))

    def profile_read(self):
        """{class name: (milliseconds, launches)} accumulated since profile_enable(True)."""
        k = len(KERNEL_CLASSES)
        ms = (ctypes.c_double * k)()
        cnt = (ctypes.c_int64 * k)()
        self._check(self.lib.ganq_profile_read(self.handle, ms, cnt))
        return {name: (ms[i], cnt[i]) for i, name in enumerate(KERNEL_CLASSES)}

    def sweep_log(self):
        """[(updated?, largest number of changed indices in a row, total changed)] per sweep of the last
        quantize_layer call."""
        n = ctypes.c_int(0)
        buf = (ctypes.c_int32 * (3 * 64))()
        self._check(self.lib.ganq_sweep_log(self.handle, buf, 64, ctypes.byref(n)))
        return [(int(buf[3 * k]), int(buf[3 * k + 1]), int(buf[3 * k + 2])) for k in range(n.value)]

    def measure_peaks(self):
        """Sustained on-box rates: {"f16_mfma_tflops", "f32_mfma_tflops", "i8_mfma_tops", "copy_gbs"}."""
        if self._ws is None:
            self._ws = torch.empty(2 << 30, dtype=torch.uint8, device=self.device)
            self._check(self.lib.ganq_set_workspace(self.handle, _ptr(self._ws), self._ws.numel()))
        out = (ctypes.c_double * 4)()
        self._check(self.lib.ganq_measure_peaks(self.handle, out))
        return {"f16_mfma_tflops": out[0], "f32_mfma_tflops": out[1], "i8_mfma_tops": out[2], "copy_gbs": out[3]}

    # ---- the seven calls -------------------------------------------------
    def build_hessian(self, X, H=None, accumulate=False):
        n, p = X.shape
        ldx = _rowmajor(X, "X")
        if H is None:
            H = torch.empty(n, n, dtype=torch.float32, device=X.device)
        self.reserve(0, n, p, 4)
        self._check(self.lib.ganq_build_hessian(self.handle, _ptr(X), _dtype_code(X), n, p, ldx,
                                                _ptr(H), _rowmajor(H, "H"), int(accumulate)))
        return H

    def build_hessian_tokens(self, Xt, H=None, accumulate=False):
        p, n = Xt.shape
        ldxt = _rowmajor(Xt, "Xt")
        if H is None:
            H = torch.empty(n, n, dtype=torch.float32, device=Xt.device)
        # room to transpose all tokens at once (the library takes what the workspace holds)
        self.reserve(0, n, p, 4, extra=min(n * (p + 8) * Xt.element_size(), 8 << 30))
        self._check(self.lib.ganq_build_hessian_tokens(self.handle, _ptr(Xt), _dtype_code(Xt), n, p, ldxt,
                                                       _ptr(H), _rowmajor(H, "H"), int(accumulate)))
        return H

    def cholesky(self, H, precond=PRECOND_NONE, lam=0.0, L=None, raise_on_fail=True):
        n = H.shape[0]
        if L is None:
            L = torch.empty(n, n, dtype=torch.float32, device=H.device)
        self.reserve(0, n, 0, 4)
        info = ctypes.c_int64(0)
        st = self.lib.ganq_cholesky(self.handle, _ptr(H), n, _rowmajor(H, "H"), precond, lam,
                                    _ptr(L), _rowmajor(L, "L"), ctypes.byref(info))
        if st == GANQ_ERR_NOT_PD and not raise_on_fail:
            return L, info.value
        self._check(st)
        return L, info.value

    def init_codebooks(self, W, nbits, init=INIT_QUANTILE_MID, T=None):
        m, n = W.shape
        if T is None:
            T = torch.empty(m, 1 << nbits, dtype=torch.float32, device=W.device)
        self._check(self.lib.ganq_init_codebooks(self.handle, _ptr(W), _dtype_code(W), m, n,
                                                 _rowmajor(W, "W"), nbits, init, _ptr(T)))
        return T

    def update_S(self, W, L, T, nbits, Q=None, want_E=False):
        m, n = W.shape
        if Q is None:
            Q = torch.empty(m, n, dtype=torch.uint8, device=W.device)
        E = torch.empty(m, n, dtype=torch.float32, device=W.device) if want_E else None
        self.reserve(m, n, 0, nbits)
        self._check(self.lib.ganq_update_S(self.handle, _ptr(W), m, n, _rowmajor(W, "W"), _ptr(L),
                                           _rowmajor(L, "L"), _ptr(T), nbits, _ptr(Q),
                                           _rowmajor(Q, "Q"), _ptr(E), n if want_E else 0))
        return (Q, E) if want_E else Q

    def update_T_prepare(self, W, H, nbits):
        """Computes what ganq_update_T needs from W and H alone once; later update_T calls with the same
        tensors reuse it.  W=None, H=None drops it."""
        if W is None and H is None:
            self._check(self.lib.ganq_update_T_prepare(self.handle, None, 0, 0, 0, None, 0, nbits))
            return
        m, n = W.shape
        self.reserve(m, n, 0, nbits)
        self._check(self.lib.ganq_update_T_prepare(self.handle, _ptr(W), m, n, _rowmajor(W, "W"), _ptr(H),
                                                   _rowmajor(H, "H"), nbits))

    def update_T(self, W, H, Q, T, nbits, empty=EMPTY_ZERO, want_counts=False):
        m, n = W.shape
        cnt = torch.zeros(m, dtype=torch.int32, device=W.device) if want_counts else None
        self.reserve(m, n, 0, nbits)
        self._check(self.lib.ganq_update_T(self.handle, _ptr(W), m, n, _rowmajor(W, "W"), _ptr(H),
                                           _rowmajor(H, "H"), _ptr(Q), _rowmajor(Q, "Q"), nbits,
                                           empty, _ptr(T), _ptr(cnt)))
        return (T, cnt) if want_counts else T

    def layer_loss(self, W, H, T, Q, nbits, want_rows=False):
        m, n = W.shape
        rows = torch.empty(m, dtype=torch.float32, device=W.device) if want_rows else None
        self.reserve(m, n, 0, nbits)
        out = ctypes.c_double(0.0)
        self._check(self.lib.ganq_layer_loss(self.handle, _ptr(W), m, n, _rowmajor(W, "W"), _ptr(H),
                                             _rowmajor(H, "H"), _ptr(T), _ptr(Q), _rowmajor(Q, "Q"),
                                             nbits, ctypes.byref(out), _ptr(rows)))
        return (out.value, rows) if want_rows else out.value

    def outlier_split(self, W, r, capacity=None, noalloc=False):
        """(W_dense fp32, row_ptr int64, col_idx int32, values fp32) of Algorithm 2; the CSR
        arrays are trimmed to the number of outliers.  noalloc=True takes the entry point whose
        scratch is part of the library image (no workspace is reserved or used)."""
        m, n = W.shape
        dev = W.device
        Wd = torch.empty(m, n, dtype=torch.float32, device=dev)
        row_ptr = torch.empty(m + 1, dtype=torch.int64, device=dev)
        fn = self.lib.ganq_outlier_split_noalloc if noalloc else self.lib.ganq_outlier_split
        if not noalloc:
            self.reserve(m, n, 0, 4)
        if capacity is None:
            capacity = m * (2 * (int(n * r * 0.5) + 2) + 8)
        nnz = ctypes.c_int64(0)
        for _ in range(2):
            col = torch.empty(max(capacity, 1), dtype=torch.int32, device=dev)
            val = torch.empty(max(capacity, 1), dtype=torch.float32, device=dev)
            st = fn(self.handle, _ptr(W), _dtype_code(W), m, n, _rowmajor(W, "W"),
                    float(r), _ptr(Wd), n, _ptr(row_ptr), _ptr(col), _ptr(val),
                    capacity, ctypes.byref(nnz))
            if st == GANQ_ERR_INVALID_ARG and nnz.value > capacity:
                capacity = nnz.value          # ties at a cut-off: size the arrays exactly and repeat
                continue
            break
        self._check(st)
        return Wd, row_ptr, col[:nnz.value], val[:nnz.value]

    def pack_layer(self, Q, T, nbits):
        """Stored form of a quantized layer: (packed uint8 (m, row bytes), lut float16 (m, 2^N))."""
        m, n = Q.shape
        rb = int(self.lib.ganq_packed_row_bytes(n, nbits))
        if rb <= 0:
            raise ValueError("nbits must be 1..4 and n positive")
        packed = torch.empty(m, rb, dtype=torch.uint8, device=Q.device)
        lut = torch.empty(m, 1 << nbits, dtype=torch.float16, device=Q.device)
        if T.dtype != torch.float32 or not T.is_contiguous() or tuple(T.shape) != (m, 1 << nbits):
            raise ValueError("T must be a contiguous float32 (m, 2^N) tensor")
        self._check(self.lib.ganq_pack_layer(self.handle, _ptr(Q), m, n, _rowmajor(Q, "Q"), _ptr(T), nbits,
                                             _ptr(packed), rb, _ptr(lut)))
        return packed, lut

    def lut_gemv(self, packed, lut, nbits, n, x, y=None, outliers=None):
        """y = W~ x (+ W_sparse x) from the stored form; x float16 (n,), y float32 (m,).
        outliers = (row_ptr int64, col_idx int32, values float32) or None.  Asynchronous."""
        m = packed.shape[0]
        if x.dtype != torch.float16 or x.dim() != 1 or x.shape[0] != n or not x.is_contiguous():
            raise ValueError("x must be a contiguous float16 vector of n entries")
        if lut.dtype != torch.float16 or not lut.is_contiguous() or tuple(lut.shape) != (m, 1 << nbits):
            raise ValueError("lut must be a contiguous float16 (m, 2^N) tensor")
        if y is None:
            y = torch.empty(m, dtype=torch.float32, device=x.device)
        rp, ci_, va = outliers if outliers is not None else (None, None, None)
        self._check(self.lib.ganq_lut_gemv(self.handle, _ptr(packed), _rowmajor(packed, "packed"), _ptr(lut),
                                           nbits, m, n, _ptr(x), _ptr(y), _ptr(rp), _ptr(ci_), _ptr(va)))
        return y

    def quantize_layer(self, W, H, nbits, iters, T=None, L=None, precond=PRECOND_NONE, lam=0.0,
                       init=INIT_QUANTILE_MID, empty=EMPTY_ZERO, Q=None, history=False, full_t_update=False):
        m, n = W.shape
        opts = GanqOptions(precond, lam, init, 1 if T is None else 0, empty,
                           OPT_FULL_T_UPDATE if full_t_update else 0)
        if T is None:
            T = torch.empty(m, 1 << nbits, dtype=torch.float32, device=W.device)
        if Q is None:
            Q = torch.empty(m, n, dtype=torch.uint8, device=W.device)
        hist = (ctypes.c_double * (2 * iters))() if history and iters > 0 else None
        self.reserve(m, n, 0, nbits)
        self._check(self.lib.ganq_quantize_layer(
            self.handle, _ptr(W), _dtype_code(W), m, n, _rowmajor(W, "W"), _ptr(H),
            _rowmajor(H, "H"), _ptr(L), _rowmajor(L, "L") if L is not None else 0, nbits, iters,
            ctypes.byref(opts), _ptr(T), _ptr(Q), _rowmajor(Q, "Q"), hist))
        if history:
            return T, Q, list(hist) if hist is not None else []
        return T, Q
