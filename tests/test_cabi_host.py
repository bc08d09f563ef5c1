"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU.  No compute calls: runs without a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2402_02446_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2402_02446_amd import build
        build.build(verbose=False)
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "lqer.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lqer_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings(L):
    seen = {binding.lqer_status_string(i) for i in range(9)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert binding.lqer_status_string(99) == "unknown status"


def test_quantize_argument_errors(L):
    q = L.lqer_quantize_mx
    assert q(None, 4, 32, 32, 5, 8, None, None, None) == 3          # mantissa width
    assert q(None, 4, 32, 32, 8, 4, None, None, None) == 3          # exponent width
    assert q(None, 4, 40, 40, 8, 8, None, None, None) == 2          # cols % 16
    assert q(None, 4, 32, 16, 8, 8, None, None, None) == 2          # ld < cols
    assert q(None, -1, 32, 32, 8, 8, None, None, None) == 2
    assert q(None, 0, 32, 32, 8, 8, None, None, None) == 0          # empty is a no-op
    assert q(None, 4, 32, 32, 8, 8, None, None, None) == 1          # null pointers


def test_import_argument_errors(L):
    out = C.c_void_p()
    imp = L.lqer_layer_import
    Wc = np.zeros((16, 8), np.uint8)
    We = np.zeros((16, 1), np.uint8)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert imp(100, 10, 0, p(Wc), p(We), None, None, None, None, C.byref(out)) == 2     # K % 16
    assert imp(16, 16, 17, p(Wc), p(We), None, None, None, None, C.byref(out)) == 2     # k > min(K, N)
    assert imp(16, 16, 0, None, p(We), None, None, None, None, C.byref(out)) == 1
    assert imp(16, 16, 4, p(Wc), p(We), None, None, None, None, C.byref(out)) == 1      # factors missing
    assert imp(16, 16, 0, p(Wc), p(We), None, None, None, None, None) == 1
    assert imp(4096, 4096, 257, p(Wc), p(We), p(Wc), p(We), p(Wc), p(We), C.byref(out)) == 3  # padded rank > 256


def test_build_factors_argument_errors(L):
    out = C.c_void_p()
    bf = L.lqer_build_factors
    W = np.zeros((16, 16), np.float32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert bf(p(W), 16, 16, None, 0, 0, 2, 1, None, C.byref(out)) == 1       # L2QER needs calibration data
    assert bf(p(W), 20, 16, None, 0, 0, 2, 0, None, C.byref(out)) == 2
    assert bf(p(W), 16, 16, None, 0, 0, 2, 5, None, C.byref(out)) == 3
    cfg = binding.Config(3, 8, 8, 16)
    assert bf(p(W), 16, 16, None, 0, 0, 2, 0, C.byref(cfg), C.byref(out)) == 3
    calib = np.ones((1, 4, 16), np.float32)
    calib[0, :, 5] = 0.0
    assert bf(p(W), 16, 16, p(calib), 1, 4, 2, 1, None, C.byref(out)) == 4   # S is singular (Sec. 3.2)


def test_forward_rejects_null_layer(L):
    assert L.lqer_linear_forward(None, None, 4, 16, None, 16, None, 0, None) == 1
    assert L.lqer_linear_workspace_bytes(None, 4) == 0
    assert L.lqer_linear_path(None, 4) == 0
    assert L.lqer_layer_free(None) == 0


def test_newer_entry_points_reject_bad_arguments_on_the_host(L):
    out = C.c_void_p()
    bfd = L.lqer_build_factors_device
    assert bfd(None, 16, 16, None, 0, 0, 2, 0, None, None, C.byref(out)) == 1      # W missing
    assert bfd(None, 20, 16, None, 0, 0, 2, 0, None, None, C.byref(out)) == 2      # K % 16
    assert bfd(None, 16, 16, None, 0, 0, 2, 7, None, None, C.byref(out)) == 3      # mode
    assert bfd(None, 16, 16, None, 0, 0, 2, 0, None, None, None) == 1
    assert L.lqer_layer_set_activation_bits(None, 6) == 1
    assert L.lqer_linear_forward_requant(None, None, 4, 16, None, 16, None, None, 0, None, None) == 1
    assert L.lqer_linear_workspace_bytes_ex(None, 4, 2) == 0
    assert L.lqer_quantize_mx(None, 4, 32, 32, 6, 8, None, None, None) == 1        # 6-bit codes are a supported width
    assert L.lqer_linear_forward_shared(None, 2, None, 4, 16, None, None, None, 0, None) == 1
    assert L.lqer_linear_shared_workspace_bytes(None, 2, 4) == 0
    assert L.lqer_set_wait_limit(-1) == 2
    assert L.lqer_set_wait_limit(1 << 22) == 0                                     # the default
