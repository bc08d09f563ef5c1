"""ctypes face of liblqer.so: same names as the C ABI in include/lqer.h.

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  PyTorch supplies device memory and the current HIP stream.  There is
no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblqer.so")

LQER_OK = 0
STATUS_NAMES = {0: "LQER_OK", 1: "LQER_ERR_NULL", 2: "LQER_ERR_SHAPE", 3: "LQER_ERR_UNSUPPORTED",
                4: "LQER_ERR_SINGULAR_SCALE", 5: "LQER_ERR_WORKSPACE", 6: "LQER_ERR_HIP",
                7: "LQER_ERR_NO_CONVERGENCE", 8: "LQER_ERR_VALUE", 9: "LQER_ERR_NO_MEMORY"}

# every symbol include/lqer.h declares
EXPORTS = ("lqer_status_string", "lqer_quantize_mx", "lqer_build_factors", "lqer_build_factors_device",
           "lqer_layer_import",
           "lqer_layer_export", "lqer_layer_dims", "lqer_layer_set_activation_bits", "lqer_layer_free", "lqer_linear_workspace_bytes", "lqer_linear_workspace_bytes_ex",
           "lqer_linear_forward", "lqer_linear_forward_q", "lqer_linear_forward_ex", "lqer_linear_forward_requant", "lqer_linear_path",
           "lqer_linear_shared_workspace_bytes", "lqer_linear_forward_shared", "lqer_set_wait_limit",
           "lqer_linear_forward_static", "lqer_layer_import_w", "lqer_layer_weight_bits",
           "lqer_int_layer_import", "lqer_int_layer_export", "lqer_quantize_int8_token", "lqer_selftest_layouts")


class LqerError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")


class LaunchOpts(C.Structure):
    _fields_ = [("path", C.c_int), ("variant", C.c_int), ("stages", C.c_int)]


class Config(C.Structure):
    _fields_ = [("w_bits", C.c_int), ("h_bits", C.c_int), ("exp_bits", C.c_int), ("block", C.c_int)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime: import it first so that liblqer.so binds to the same
    # runtime instance (and the same streams and allocations) instead of loading a second one.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2402_02446_amd.build` "
                           "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    L.lqer_status_string.restype = C.c_char_p
    L.lqer_status_string.argtypes = [i32]
    L.lqer_quantize_mx.restype = i32
    L.lqer_quantize_mx.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp]
    L.lqer_build_factors.restype = i32
    L.lqer_build_factors.argtypes = [vp, i64, i64, vp, i64, i64, i32, i32, vp, C.POINTER(vp)]
    L.lqer_build_factors_device.restype = i32
    L.lqer_build_factors_device.argtypes = [vp, i64, i64, vp, i64, i64, i32, i32, vp, vp, C.POINTER(vp)]
    L.lqer_layer_import.restype = i32
    L.lqer_layer_import.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp, vp, C.POINTER(vp)]
    L.lqer_layer_import_w.restype = i32
    L.lqer_layer_import_w.argtypes = [i32, i64, i64, i32, vp, vp, vp, vp, vp, vp, C.POINTER(vp)]
    L.lqer_layer_weight_bits.restype = i32
    L.lqer_layer_weight_bits.argtypes = [vp]
    L.lqer_int_layer_import.restype = i32
    L.lqer_int_layer_import.argtypes = [i64, i64, i32, vp, vp, vp, vp, vp, vp, C.POINTER(vp)]
    L.lqer_int_layer_export.restype = i32
    L.lqer_int_layer_export.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.lqer_quantize_int8_token.restype = i32
    L.lqer_quantize_int8_token.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    L.lqer_layer_export.restype = i32
    L.lqer_layer_export.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.lqer_layer_dims.restype = i32
    L.lqer_layer_dims.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    L.lqer_layer_set_activation_bits.restype = i32
    L.lqer_layer_set_activation_bits.argtypes = [vp, i32]
    L.lqer_layer_free.restype = i32
    L.lqer_layer_free.argtypes = [vp]
    L.lqer_linear_workspace_bytes.restype = sz
    L.lqer_linear_workspace_bytes.argtypes = [vp, i64]
    L.lqer_linear_workspace_bytes_ex.restype = sz
    L.lqer_linear_workspace_bytes_ex.argtypes = [vp, i64, i32]
    L.lqer_linear_forward.restype = i32
    L.lqer_linear_forward.argtypes = [vp, vp, i64, i64, vp, i64, vp, sz, vp]
    L.lqer_linear_forward_q.restype = i32
    L.lqer_linear_forward_q.argtypes = [vp, vp, vp, i64, vp, i64, vp, sz, vp]
    L.lqer_linear_forward_ex.restype = i32
    L.lqer_linear_forward_ex.argtypes = [vp, vp, i64, i64, vp, i64, vp, sz, vp, C.POINTER(LaunchOpts)]
    L.lqer_linear_forward_requant.restype = i32
    L.lqer_linear_forward_requant.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp, sz, vp, vp]
    L.lqer_linear_shared_workspace_bytes.restype = sz
    L.lqer_linear_shared_workspace_bytes.argtypes = [C.POINTER(vp), i32, i64]
    L.lqer_linear_forward_shared.restype = i32
    L.lqer_linear_forward_shared.argtypes = [C.POINTER(vp), i32, vp, i64, i64, C.POINTER(vp), C.POINTER(i64), vp, sz, vp]
    L.lqer_set_wait_limit.restype = i32
    L.lqer_set_wait_limit.argtypes = [i32]
    L.lqer_linear_path.restype = i32
    L.lqer_linear_path.argtypes = [vp, i64]
    L.lqer_linear_forward_static.restype = i32
    L.lqer_linear_forward_static.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    _lib = L
    return L


def _check(status: int, where: str):
    if status != LQER_OK:
        raise LqerError(status, where)


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def lqer_status_string(status: int) -> str:
    return lib().lqer_status_string(int(status)).decode()


def lqer_quantize_mx(x, elem_bits: int = 8, exp_bits: int = 8):
    """x: CUDA fp32 [rows][cols] (row stride may exceed cols). Returns (codes, exps) CUDA tensors."""
    import torch
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else max(cols, x.stride(0))
    code_cols = cols if elem_bits >= 6 else cols // 2
    codes = torch.empty((rows, code_cols), dtype=torch.int8 if elem_bits >= 6 else torch.uint8, device=x.device)
    exps = torch.empty((rows, cols // 16), dtype=torch.uint8, device=x.device)
    _check(lib().lqer_quantize_mx(C.c_void_p(x.data_ptr()), rows, cols, ld, elem_bits, exp_bits,
                                  C.c_void_p(codes.data_ptr()), C.c_void_p(exps.data_ptr()), _stream()),
           "lqer_quantize_mx")
    return codes, exps


class Layer:
    """Owning wrapper of an lqer_layer handle."""

    def __init__(self, handle):
        self.handle = C.c_void_p(handle)
        K, N, k, kp = C.c_int64(), C.c_int64(), C.c_int(), C.c_int()
        _check(lib().lqer_layer_dims(self.handle, C.byref(K), C.byref(N), C.byref(k), C.byref(kp)),
               "lqer_layer_dims")
        self.K, self.N, self.k, self.kp = K.value, N.value, k.value, kp.value
        self.w_bits = int(lib().lqer_layer_weight_bits(self.handle))
        self._ws = None

    def set_activation_bits(self, bits: int):
        _check(lib().lqer_layer_set_activation_bits(self.handle, int(bits)), "lqer_layer_set_activation_bits")

    def free(self):
        if self.handle:
            lib().lqer_layer_free(self.handle)
            self.handle = C.c_void_p(None)
            self._ws = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def workspace(self, M: int, path: int = 0):
        """A cached torch allocation of lqer_linear_workspace_bytes_ex(M, path) bytes."""
        import torch
        need = lib().lqer_linear_workspace_bytes_ex(self.handle, M, path)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        return self._ws


def lqer_layer_import(K, N, k, Wc, We, Ac=None, Ae=None, Bc=None, Be=None) -> Layer:
    arrs = [None if a is None else np.ascontiguousarray(a) for a in (Wc, We, Ac, Ae, Bc, Be)]
    out = C.c_void_p()
    _check(lib().lqer_layer_import(K, N, k, *[_np_ptr(a) for a in arrs], C.byref(out)), "lqer_layer_import")
    return Layer(out.value)


def lqer_layer_import_w(w_bits, K, N, k, Wc, We, Ac=None, Ae=None, Bc=None, Be=None) -> Layer:
    """Import with the mantissa width of W_q given: 4 (Wc [N][K/2]) or 2 (Wc [N][K/4])."""
    arrs = [None if a is None else np.ascontiguousarray(a) for a in (Wc, We, Ac, Ae, Bc, Be)]
    if arrs[0].size != N * K * w_bits // 8:
        raise ValueError("Wc does not hold N * K codes of that width")
    out = C.c_void_p()
    _check(lib().lqer_layer_import_w(int(w_bits), K, N, k, *[_np_ptr(a) for a in arrs], C.byref(out)), "lqer_layer_import_w")
    return Layer(out.value)


def lqer_int_layer_import(K, N, k, Wc, Ws, Ac=None, As=None, Bc=None, Bs=None) -> Layer:
    """INT layer from canonical arrays; scales are float16 arrays."""
    arrs = [np.ascontiguousarray(Wc, dtype=np.uint8), np.ascontiguousarray(Ws, dtype=np.float16)]
    for a, dt in ((Ac, np.int8), (As, np.float16), (Bc, np.int8), (Bs, np.float16)):
        arrs.append(None if (a is None or k == 0) else np.ascontiguousarray(a, dtype=dt))
    out = C.c_void_p()
    _check(lib().lqer_int_layer_import(K, N, k, *[_np_ptr(a) for a in arrs], C.byref(out)), "lqer_int_layer_import")
    return Layer(out.value)


def lqer_int_layer_export(layer: Layer):
    K, N, kp = layer.K, layer.N, layer.kp
    Wc, Ws = np.zeros((N, K // 2), np.uint8), np.zeros((N, K // 128), np.float16)
    Ac, As = np.zeros((kp, K), np.int8), np.zeros((kp, K // 128), np.float16)
    Bc, Bs = np.zeros((N, kp), np.int8), np.zeros((N,), np.float16)
    ptrs = [_np_ptr(a) for a in ((Wc, Ws, Ac, As, Bc, Bs) if kp else (Wc, Ws))] + ([] if kp else [None] * 4)
    _check(lib().lqer_int_layer_export(layer.handle, *ptrs), "lqer_int_layer_export")
    return dict(Wc=Wc, Ws=Ws, Ac=Ac, As=As, Bc=Bc, Bs=Bs)


def lqer_quantize_int8_token(x):
    """x: CUDA fp32 [rows][cols].  Returns (codes int8 [rows][cols], scales float16 [rows]) CUDA tensors."""
    import torch
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else max(cols, x.stride(0))
    codes = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
    scales = torch.empty((rows,), dtype=torch.float16, device=x.device)
    _check(lib().lqer_quantize_int8_token(C.c_void_p(x.data_ptr()), rows, cols, ld, C.c_void_p(codes.data_ptr()),
                                          C.c_void_p(scales.data_ptr()), _stream()), "lqer_quantize_int8_token")
    return codes, scales


def lqer_layer_export(layer: Layer):
    K, N, kp = layer.K, layer.N, layer.kp
    Wc = np.zeros((N, K * layer.w_bits // 8), np.uint8)
    We = np.zeros((N, K // 16), np.uint8)
    Ac = np.zeros((kp, K), np.int8)
    Ae = np.zeros((kp, K // 16), np.uint8)
    Bc = np.zeros((N, kp), np.int8)
    Be = np.zeros((N, kp // 16), np.uint8)
    _check(lib().lqer_layer_export(layer.handle, *[_np_ptr(a) for a in (Wc, We, Ac, Ae, Bc, Be)]),
           "lqer_layer_export")
    return dict(Wc=Wc, We=We, Ac=Ac, Ae=Ae, Bc=Bc, Be=Be)


def lqer_build_factors(W, calib, k: int, mode: int = 1, cfg=None) -> Layer:
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    if calib is not None:
        calib = np.ascontiguousarray(calib, dtype=np.float32)
        ns, rows, kc = calib.shape
        if kc != K:
            raise ValueError("calib's last axis must be K")
    else:
        ns, rows = 0, 0
    c = None if cfg is None else C.byref(Config(*cfg))
    out = C.c_void_p()
    _check(lib().lqer_build_factors(_np_ptr(W), K, N, _np_ptr(calib), ns, rows, k, mode, c, C.byref(out)),
           "lqer_build_factors")
    return Layer(out.value)


def lqer_build_factors_device(W, calib, k: int, mode: int = 1, cfg=None) -> Layer:
    """W [K][N] and calib [n_samples][rows][K] are fp32 CUDA tensors; runs on torch's current stream."""
    import torch
    if not (W.is_cuda and W.dtype == torch.float32 and (calib is None or (calib.is_cuda and calib.dtype == torch.float32))):
        raise ValueError("W and calib must be fp32 CUDA tensors")
    W = W.contiguous()
    K, N = W.shape
    if calib is not None:
        calib = calib.contiguous()
        ns, rows, kc = calib.shape
        if kc != K:
            raise ValueError("calib's last axis must be K")
        cptr = C.c_void_p(calib.data_ptr())
    else:
        ns, rows, cptr = 0, 0, None
    c = None if cfg is None else C.byref(Config(*cfg))
    out = C.c_void_p()
    _check(lib().lqer_build_factors_device(C.c_void_p(W.data_ptr()), K, N, cptr, ns, rows, k, mode, c, _stream(), C.byref(out)),
           "lqer_build_factors_device")
    return Layer(out.value)


def lqer_linear_workspace_bytes(layer: Layer, M: int, path: int = 0) -> int:
    return int(lib().lqer_linear_workspace_bytes_ex(layer.handle, M, path))


def lqer_linear_path(layer: Layer, M: int) -> int:
    return int(lib().lqer_linear_path(layer.handle, M))


def lqer_linear_forward(layer: Layer, X, Y=None, workspace=None):
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, layer.N), dtype=torch.float32, device=X.device)
    ws = layer.workspace(M) if workspace is None else workspace
    ldx = X.stride(0) if M > 1 else max(layer.K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(layer.N, Y.stride(0))
    _check(lib().lqer_linear_forward(layer.handle, C.c_void_p(X.data_ptr()), M, ldx, C.c_void_p(Y.data_ptr()),
                                     ldy, C.c_void_p(ws.data_ptr()), ws.numel(), _stream()),
           "lqer_linear_forward")
    return Y


def lqer_linear_forward_static(layer: Layer, X, Y=None):
    """The forward pass on the library's own static scratch (no workspace argument)."""
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, layer.N), dtype=torch.float32, device=X.device)
    ldx = X.stride(0) if M > 1 else max(layer.K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(layer.N, Y.stride(0))
    _check(lib().lqer_linear_forward_static(layer.handle, C.c_void_p(X.data_ptr()), M, ldx, C.c_void_p(Y.data_ptr()),
                                            ldy, _stream()),
           "lqer_linear_forward_static")
    return Y


def lqer_linear_forward_q(layer: Layer, Xc, Xe, Y=None, workspace=None):
    import torch
    M = Xc.shape[0]
    if Y is None:
        Y = torch.empty((M, layer.N), dtype=torch.float32, device=Xc.device)
    ws = layer.workspace(M) if workspace is None else workspace
    ldy = Y.stride(0) if M > 1 else max(layer.N, Y.stride(0))
    _check(lib().lqer_linear_forward_q(layer.handle, C.c_void_p(Xc.data_ptr()), C.c_void_p(Xe.data_ptr()), M,
                                       C.c_void_p(Y.data_ptr()), ldy, C.c_void_p(ws.data_ptr()), ws.numel(),
                                       _stream()),
           "lqer_linear_forward_q")
    return Y


def lqer_linear_forward_ex(layer: Layer, X, Y=None, workspace=None, path=0, variant=0, stages=0):
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, layer.N), dtype=torch.float32, device=X.device)
    ws = layer.workspace(M, path) if workspace is None else workspace
    ldx = X.stride(0) if M > 1 else max(layer.K, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(layer.N, Y.stride(0))
    opts = LaunchOpts(path, variant, stages)
    _check(lib().lqer_linear_forward_ex(layer.handle, C.c_void_p(X.data_ptr()), M, ldx,
                                        C.c_void_p(Y.data_ptr()), ldy, C.c_void_p(ws.data_ptr()), ws.numel(),
                                        _stream(), C.byref(opts)),
           "lqer_linear_forward_ex")
    return Y


def lqer_linear_forward_requant(layer: Layer, X, workspace=None, path=0, variant=0):
    """Forward pass with Y leaving as MXINT8: returns (codes int8 [M][N], exps uint8 [M][N/16])."""
    import torch
    M = X.shape[0]
    codes = torch.empty((M, layer.N), dtype=torch.int8, device=X.device)
    exps = torch.empty((M, layer.N // 16), dtype=torch.uint8, device=X.device)
    ws = layer.workspace(M, path) if workspace is None else workspace
    ldx = X.stride(0) if M > 1 else max(layer.K, X.stride(0))
    opts = LaunchOpts(path, variant, 0)
    _check(lib().lqer_linear_forward_requant(layer.handle, C.c_void_p(X.data_ptr()), M, ldx,
                                             C.c_void_p(codes.data_ptr()), layer.N, C.c_void_p(exps.data_ptr()),
                                             C.c_void_p(ws.data_ptr()), ws.numel(), _stream(), C.byref(opts)),
           "lqer_linear_forward_requant")
    return codes, exps


def lqer_linear_shared_workspace_bytes(layers, M: int) -> int:
    arr = (C.c_void_p * len(layers))(*[l.handle for l in layers])
    return int(lib().lqer_linear_shared_workspace_bytes(arr, len(layers), M))


def lqer_linear_forward_shared(layers, X, Ys=None, workspace=None):
    """Several layers applied to the same X (quantized once): returns the list of their Y."""
    import torch
    M = X.shape[0]
    n = len(layers)
    if Ys is None:
        Ys = [torch.empty((M, l.N), dtype=torch.float32, device=X.device) for l in layers]
    arr = (C.c_void_p * n)(*[l.handle for l in layers])
    if workspace is None:
        need = lib().lqer_linear_shared_workspace_bytes(arr, n, M)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    ldx = X.stride(0) if M > 1 else max(layers[0].K, X.stride(0))
    yarr = (C.c_void_p * n)(*[C.c_void_p(y.data_ptr()) for y in Ys])
    ldys = (C.c_int64 * n)(*[(y.stride(0) if M > 1 else max(l.N, y.stride(0))) for y, l in zip(Ys, layers)])
    _check(lib().lqer_linear_forward_shared(arr, n, C.c_void_p(X.data_ptr()), M, ldx, yarr, ldys,
                                            C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream()),
           "lqer_linear_forward_shared")
    return Ys


def lqer_set_wait_limit(polls: int):
    _check(lib().lqer_set_wait_limit(int(polls)), "lqer_set_wait_limit")
