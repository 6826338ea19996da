"""CPU-only checks of the C-ABI boundary: the built library loads, exports every
symbol the header declares, and rejects bad arguments on the host before any GPU
work (so these run without a device)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ganq.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2501_12956_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2501_12956_amd import build
        build.build(verbose=False)
    return binding.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ganq_[A-Za-z_]+)\s*\(", text)))


def test_header_declares_the_seven_calls():
    names = declared_symbols()
    for want in ["ganq_build_hessian", "ganq_cholesky", "ganq_init_codebooks", "ganq_update_S",
                 "ganq_update_T", "ganq_layer_loss", "ganq_quantize_layer"]:
        assert want in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2501_12956_amd import binding
    names = declared_symbols()
    assert len(names) >= 13
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names


def test_status_strings(lib):
    seen = set()
    for code in range(6):
        s = lib.ganq_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 6
    assert lib.ganq_status_string(99).decode() == "unknown status"


def test_workspace_query(lib):
    assert lib.ganq_workspace_bytes(0, 0, 0, 4) == 0
    assert lib.ganq_workspace_bytes(16, 64, 0, 5) == 0
    small = lib.ganq_workspace_bytes(256, 512, 4096, 4)
    big = lib.ganq_workspace_bytes(4096, 4096, 262144, 4)
    assert 0 < small < big
    # the headline layer fits comfortably in one GPU's memory
    assert big < 8 * (1 << 30)


def test_argument_checks_run_on_the_host(lib):
    from paper_2501_12956_amd import binding as b
    h = ctypes.c_void_p()
    assert lib.ganq_create(None, 0, None) == b.GANQ_ERR_INVALID_ARG
    assert lib.ganq_create(ctypes.byref(h), -1, None) == b.GANQ_ERR_INVALID_ARG
    assert lib.ganq_create(ctypes.byref(h), 0, None) == b.GANQ_OK and h.value
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    info = ctypes.c_int64(7)
    loss = ctypes.c_double(0)
    inv = b.GANQ_ERR_INVALID_ARG
    # null context
    assert lib.ganq_update_S(None, fake, 1, 1, 1, fake, 1, fake, 4, fake, 1, None, 0) == inv
    # bad sizes / leading dimensions / nbits / enums
    assert lib.ganq_build_hessian(h, fake, 0, 0, 8, 8, fake, 8, 0) == inv
    assert lib.ganq_build_hessian(h, fake, 0, 8, 16, 8, fake, 8, 0) == inv          # ldx < p
    assert lib.ganq_build_hessian(h, fake, 7, 8, 16, 16, fake, 8, 0) == inv         # dtype
    assert lib.ganq_build_hessian(h, fake, 0, 8, 16, 20, fake, 8, 0) == b.GANQ_ERR_UNSUPPORTED
    assert lib.ganq_cholesky(h, fake, 8, 4, 0, 0.0, ctypes.c_void_p(0x2000), 8, ctypes.byref(info)) == inv
    assert info.value == 0
    assert lib.ganq_cholesky(h, fake, 8, 8, 0, 0.0, fake, 8, ctypes.byref(info)) == inv    # alias
    assert lib.ganq_cholesky(h, fake, 8, 8, 1, 0.0, ctypes.c_void_p(0x2000), 8, ctypes.byref(info)) == inv  # lambda
    assert lib.ganq_cholesky(h, fake, 8, 8, 9, 0.0, ctypes.c_void_p(0x2000), 8, ctypes.byref(info)) == inv
    assert lib.ganq_init_codebooks(h, fake, 1, 4, 8, 8, 0, 0, fake) == inv
    assert lib.ganq_init_codebooks(h, fake, 1, 4, 8, 8, 5, 0, fake) == inv
    assert lib.ganq_init_codebooks(h, fake, 1, 4, 8, 8, 4, 3, fake) == inv
    assert lib.ganq_init_codebooks(h, fake, 1, 4, 40000, 40000, 4, 0, fake) == b.GANQ_ERR_UNSUPPORTED
    assert lib.ganq_update_S(h, fake, 4, 8, 7, fake, 8, fake, 4, fake, 8, None, 0) == inv
    assert lib.ganq_update_S(h, fake, 4, 8, 8, None, 8, fake, 4, fake, 8, None, 0) == inv
    assert lib.ganq_update_S(h, fake, 4, 8, 8, fake, 8, fake, 4, fake, 8, fake, 4) == inv   # lde
    assert lib.ganq_update_T(h, fake, 4, 8, 8, fake, 8, fake, 8, 4, 2, fake, None) == inv   # empty mode
    assert lib.ganq_update_T(h, fake, 4, 8, 8, fake, 8, None, 8, 4, 0, fake, None) == inv
    assert lib.ganq_layer_loss(h, fake, 4, 8, 8, fake, 8, fake, fake, 8, 4, None, None) == inv
    assert lib.ganq_layer_loss(h, fake, 4, -1, 8, fake, 8, fake, fake, 8, 4, ctypes.byref(loss), None) == inv
    opts = b.GanqOptions(0, 0.0, 0, 0, 0, 2)
    assert lib.ganq_quantize_layer(h, fake, 1, 4, 8, 8, fake, 8, None, 0, 4, 1, ctypes.byref(opts),
                                   fake, fake, 8, None) == inv                       # unknown flag bit
    assert lib.ganq_quantize_layer(h, fake, 1, 4, 8, 8, fake, 8, None, 0, 4, -1, None,
                                   fake, fake, 8, None) == inv
    # deployment calls: stored-form geometry, alignment, CSR arrays all or none
    assert lib.ganq_packed_row_bytes(4096, 4) == 2048 and lib.ganq_packed_row_bytes(4096, 3) == 1536
    assert lib.ganq_packed_row_bytes(33, 3) == 32 and lib.ganq_packed_row_bytes(1, 1) == 16
    assert lib.ganq_packed_row_bytes(0, 4) == 0 and lib.ganq_packed_row_bytes(8, 5) == 0
    al = ctypes.c_void_p(0x1000)
    assert lib.ganq_pack_layer(h, fake, 4, 64, 64, fake, 5, al, 32, fake) == inv        # nbits
    assert lib.ganq_pack_layer(h, fake, 4, 64, 32, fake, 4, al, 32, fake) == inv        # ldq < n
    assert lib.ganq_pack_layer(h, fake, 4, 64, 64, fake, 4, al, 16, fake) == inv        # ldp too small
    assert lib.ganq_pack_layer(h, fake, 4, 64, 64, fake, 4, ctypes.c_void_p(0x1004), 32, fake) == inv
    assert lib.ganq_pack_layer(h, fake, 70000, 64, 64, fake, 4, al, 32, fake) == b.GANQ_ERR_UNSUPPORTED
    assert lib.ganq_lut_gemv(h, al, 24, fake, 4, 4, 64, fake, fake, None, None, None) == inv     # ldp % 16
    assert lib.ganq_lut_gemv(h, al, 32, fake, 0, 4, 64, fake, fake, None, None, None) == inv     # nbits
    assert lib.ganq_lut_gemv(h, al, 32, fake, 4, 4, 64, None, fake, None, None, None) == inv     # x
    assert lib.ganq_lut_gemv(h, al, 32, fake, 4, 4, 64, fake, fake, fake, None, None) == inv     # partial CSR
    assert lib.ganq_lut_gemv(None, al, 32, fake, 4, 4, 64, fake, fake, None, None, None) == inv
    assert b"" != lib.ganq_last_error(h)
    # empty problems are accepted without touching the GPU
    assert lib.ganq_update_S(h, None, 0, 8, 8, fake, 8, None, 4, None, 8, None, 0) == b.GANQ_OK
    assert lib.ganq_layer_loss(h, None, 0, 8, 8, fake, 8, None, None, 8, 4, ctypes.byref(loss), None) == b.GANQ_OK
    assert loss.value == 0.0
    # workspace plumbing
    assert lib.ganq_set_workspace(h, ctypes.c_void_p(0x1001), 64) == inv              # alignment
    assert lib.ganq_set_workspace(h, None, 64) == inv
    assert lib.ganq_set_workspace(h, None, 0) == b.GANQ_OK
    assert lib.ganq_destroy(h) == b.GANQ_OK
    assert lib.ganq_destroy(None) == inv


def test_product_path_has_no_oracle_import():
    pkg = os.path.join(ROOT, "paper_2501_12956_amd")
    for dirpath, _dirs, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text or f == "synth.py", f
    text = open(os.path.join(pkg, "synth.py")).read()
    assert "import oracle" not in text and "from oracle" not in text


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
