"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2110_08688_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2110_08688_amd.build import build

        build()
    binding.lib()
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mggcn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mggcn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(B):
    names = declared_symbols()
    assert len(names) >= 25
    handle = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), f"{n} declared in mggcn.h but not exported"
        assert n in B.SIGNATURES, f"{n} has no ctypes signature in the binding"
    assert sorted(B.SIGNATURES) == names


def test_version(B):
    assert B.lib().mggcn_version() >= 100


def test_argument_errors_need_no_device(B):
    L = B.lib()
    # GeMM
    assert L.mggcn_gemm(0, 0, -1, 2, 3, None, 0, None, 0, 0.0, 0, None, 0, None, 0, None) == B.E_INVALID_ARG
    assert "negative" in B.last_error()
    assert L.mggcn_gemm(5, 0, 1, 2, 3, None, 3, None, 2, 0.0, 0, None, 2, None, 0, None) == B.E_INVALID_ARG
    assert L.mggcn_gemm(0, 0, 4, 4, 4, 16, 2, 16, 4, 0.0, 0, 16, 4, None, 0, None) == B.E_INVALID_ARG  # lda < K
    assert L.mggcn_gemm(0, 0, 4, 4, 4, 16, 4, 16, 4, 0.5, 0, 16, 4, None, 0, None) == B.E_INVALID_ARG  # beta
    assert L.mggcn_gemm(0, 0, 4, 4, 4, 16, 4, 16, 4, 1.0, 2, 16, 4, None, 0, None) == B.E_INVALID_ARG  # mask+beta
    assert L.mggcn_gemm(0, 0, 4, 4, 4, None, 4, 16, 4, 0.0, 0, 16, 4, None, 0, None) == B.E_INVALID_ARG  # NULL A
    # split-K weight-gradient shape without workspace
    need = L.mggcn_gemm_workspace_bytes(1, 0, 602, 128, 232965)
    assert need > 0
    assert L.mggcn_gemm(1, 0, 602, 128, 232965, 256, 602, 256, 128, 0.0, 0, 256, 128, None, 0, None) == B.E_WORKSPACE
    assert L.mggcn_gemm(1, 0, 602, 128, 232965, 256, 602, 256, 128, 0.0, 0, 256, 128, 256, need - 1, None) == B.E_WORKSPACE
    assert L.mggcn_gemm_workspace_bytes(0, 0, 232965, 128, 602) == 0
    # normalise
    assert L.mggcn_csr_normalize_workspace_bytes(10, 10) > 0
    nnz = C.c_int64(0)
    assert L.mggcn_csr_normalize_count(-1, 2, 256, 256, 0, 256, C.byref(nnz), 256, 1 << 20, None) == B.E_INVALID_ARG
    assert L.mggcn_csr_normalize_count(4, 4, None, 256, 0, 256, C.byref(nnz), 256, 1 << 20, None) == B.E_INVALID_ARG
    assert L.mggcn_csr_normalize_count(4, 4, 256, 256, 0, 256, C.byref(nnz), None, 0, None) == B.E_WORKSPACE
    assert L.mggcn_csr_normalize_count(4, 4, 256, 256, 0, 256, C.byref(nnz), 257, 1 << 20, None) == B.E_WORKSPACE
    assert L.mggcn_csr_normalize_count(4, 4, 256, 256, 0, 256, C.byref(nnz), 256, 8, None) == B.E_WORKSPACE
    assert L.mggcn_csr_normalize(4, 4, 256, 256, 7, None, None, 256, 256, 256, 256, 1 << 20, None) == B.E_INVALID_ARG
    assert L.mggcn_csr_normalize(4, 9, 256, 256, 0, None, None, 256, 256, 256, 256, 1 << 20, None) == B.E_INVALID_ARG
    assert "deg_row" in B.last_error()
    # transpose
    assert L.mggcn_csr_transpose(4, 4, 1 << 31, 256, 256, 256, 256, 256, 256, 256, 1 << 20, None) == B.E_OVERFLOW
    assert L.mggcn_csr_transpose(4, 4, 3, 256, 256, 256, 256, 256, 256, 256, 16, None) == B.E_WORKSPACE
    # graph / spmm
    h = C.c_void_p(None)
    assert L.mggcn_graph_create(-3, 3, 256, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_graph_create(3, 4, 256, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert "symmetric" in B.last_error()
    assert L.mggcn_graph_create(3, 3, None, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_graph_create(3, 3, 256, 256, 256, None, None, None, 0, 65, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_spmm(None, 0, 256, 4, 4, 0.0, 0, 256, 4, None) == B.E_INVALID_ARG
    # the 64-bit-offset forms and the bfloat16 forms check their arguments the same way
    assert L.mggcn_graph_create64(-3, 3, 256, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_graph_create64(3, 4, 256, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_graph_create64(3, 3, None, 256, 256, None, None, None, 0, 0, None, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_csr_normalize_count64(4, 4, None, 256, 0, 256, C.byref(nnz), 256, 1 << 20, None) == B.E_INVALID_ARG
    assert L.mggcn_csr_normalize_count64(4, 4, 256, 256, 0, 256, C.byref(nnz), 256, 8, None) == B.E_WORKSPACE
    assert L.mggcn_csr_normalize64(4, 9, 256, 256, 0, None, None, 256, 256, 256, 256, 1 << 20, None) == B.E_INVALID_ARG
    assert L.mggcn_spmm_bf16(None, 0, 256, 8, 8, 0.0, 0, 256, 8, None) == B.E_INVALID_ARG
    assert L.mggcn_f32_to_bf16(-1, 4, 256, 4, 256, 4, None) == B.E_INVALID_ARG
    assert L.mggcn_f32_to_bf16(4, 4, 256, 3, 256, 4, None) == B.E_INVALID_ARG
    assert L.mggcn_f32_to_bf16(4, 4, None, 4, 256, 4, None) == B.E_INVALID_ARG
    assert L.mggcn_f32_to_bf16(0, 4, None, 4, None, 4, None) == B.OK
    assert L.mggcn_model_gather_operand(None, 4, None, None) == B.E_INVALID_ARG
    # loss / relu
    assert L.mggcn_softmax_ce(0, 4, 256, 4, 256, 256, 256, 4, 256, 1024, None) == B.E_INVALID_ARG
    assert L.mggcn_softmax_ce(8, 4, 256, 3, 256, 256, 256, 4, 256, 1024, None) == B.E_INVALID_ARG
    assert L.mggcn_softmax_ce(8, 4, 256, 4, 256, 256, 256, 4, None, 0, None) == B.E_WORKSPACE
    assert L.mggcn_relu_bwd(4, 4, 256, 2, 256, 4, None) == B.E_INVALID_ARG
    assert L.mggcn_adam_step(8, 256, 256, 256, 256, 0, 0.01, 0.9, 0.999, 1e-8, None) == B.E_INVALID_ARG
    assert L.mggcn_adam_step(8, 256, 256, 256, 256, 1, 0.01, 1.0, 0.999, 1e-8, None) == B.E_INVALID_ARG
    # model
    dims = (C.c_int32 * 3)(602, 128, 41)
    assert L.mggcn_model_create(None, 2, dims, None, 0, C.byref(h)) == B.E_INVALID_ARG
    assert L.mggcn_model_cache_input(None, 256, 4, None) == B.E_INVALID_ARG
    assert L.mggcn_epoch(None, 256, 4, 256, None, 256, None, None) == B.E_INVALID_ARG
    assert L.mggcn_layer_fwd(None, 0, 256, 4, 256, 4, 1, 256, 4, None) == B.E_INVALID_ARG


def test_spmm_width_rule(B):
    """SpMM runs at min(d_l, d_{l+1}): SpMM first iff d_l < d_{l+1}, tie -> GeMM first."""
    L = B.lib()

    def width(dims, orders=None, flags=0):
        d = (C.c_int32 * len(dims))(*dims)
        o = (C.c_int32 * (len(dims) - 1))(*orders) if orders else None
        return L.mggcn_model_spmm_width_max(d, o, len(dims) - 1, flags)

    assert width((602, 128, 41)) == 128
    assert width((100, 256, 256, 47)) == 256  # layer 2 is a tie -> GeMM first at width 256
    assert width((128, 256)) == 128
    assert width((128, 256), [B.ORDER_GEMM_FIRST]) == 256
    assert width((64, 16, 8)) == 16
    assert width((602, 128, 41), flags=B.MODEL_CACHE_INPUT) == 602  # the one-off A^ X product


def test_product_does_not_import_the_oracle():
    """The HIP package must never route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2110_08688_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "mggcn_ref" not in text and "import oracle" not in text and "from oracle" not in text, f


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on exactly one GPU: any other --gpus exits with a message and no JSON line."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
