"""L2QER-INT: the scaled-integer variant of the layer (Table 2, rows "L2QER-INT"): oracle version.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Table 2 evaluates the method with INT4 weights in groups of 128 ("INT4, g128") and, in the
weight-activation setup, 8-bit activations ("W4A8, g128"); Sec. 2.1 gives the form of such formats: a weight
group is quantized with a scale factor, (W_q, s) = q(W), activations with a vector of per-token scalars, and an
inner product is a fixed-point inner product times an FP16 product of the two scalars.  The paper prints no
formula for q; the reading taken here is the plain symmetric one:

  weights (and A_k, B_k): groups of 128 consecutive elements along the contraction axis,
      s    = fp16(amax / qmax)   round to nearest even;  s = 1 for an all-zero group
      code = clamp(rne(v / s), -qmax, qmax)              qmax = 7 (4 bits) or 127 (8 bits)
      v^   = code * s
  activations: one scale per token row, s_t = fp16(amax_t / 127) with the division in fp32 (the precision the
      layer runs it in), code = clamp(rne(fp32(x) / fp32(s_t)), -127, 127) with that division in fp32 as well.

  T = X_q A_k is kept in full precision, Y = X_q W_q + T B_k as in Eq. 3 / Eq. 6.

The rank is padded to a multiple of 16 with zero columns / rows; B_k's contraction axis is the rank, at most
128 here, so every output column of B_k has exactly one scale.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import mxint
from .factors import calibrate_scale, error_factors, padded_rank

GROUP = 128


@dataclass
class IntLayer:
    K: int
    N: int
    k: int
    kp: int
    Wc: np.ndarray   # uint8   [N][K/2]    two's-complement nibbles, element 2i low
    Ws: np.ndarray   # float16 [N][K/128]
    Ac: np.ndarray   # int8    [kp][K]
    As: np.ndarray   # float16 [kp][K/128]
    Bc: np.ndarray   # int8    [N][kp]
    Bs: np.ndarray   # float16 [N]


def group_quantize(v, bits: int, axis: int = -1, group: int = GROUP):
    """Symmetric scaled-integer quantization in groups of `group` along `axis` (a shorter axis is one group).
    Returns (codes int8 like v, scales float16 with `axis` shrunk to the number of groups)."""
    v = np.asarray(v, dtype=np.float64)
    if not np.all(np.isfinite(v)):
        raise ValueError("quantizer requires finite inputs")
    v = np.moveaxis(v, axis, -1)
    n = v.shape[-1]
    g = min(group, n) if n else group
    if n % g:
        raise ValueError(f"length {n} along the group axis is not a multiple of {g}")
    blk = v.reshape(v.shape[:-1] + (n // g, g))
    qmax = (1 << (bits - 1)) - 1
    amax = np.abs(blk).max(axis=-1)
    with np.errstate(over="ignore"):
        s = (amax / qmax).astype(np.float16)                    # round to nearest even
    if not np.all(np.isfinite(s)):
        raise ValueError("a group scale exceeds the fp16 range")
    s = np.where(amax == 0.0, np.float16(1.0), s)
    if np.any(s == 0):
        raise ValueError("a group scale underflows fp16")
    q = np.rint(blk / s.astype(np.float64)[..., None])
    codes = np.clip(q, -qmax, qmax).astype(np.int8).reshape(v.shape)
    return (np.ascontiguousarray(np.moveaxis(codes, -1, axis)),
            np.ascontiguousarray(np.moveaxis(s.astype(np.float16), -1, axis)))


def group_dequantize(codes, scales, axis: int = -1, group: int = GROUP) -> np.ndarray:
    """v^ = code * s in fp64 (exact)."""
    c = np.moveaxis(np.asarray(codes).astype(np.float64), axis, -1)
    s = np.moveaxis(np.asarray(scales).astype(np.float64), axis, -1)
    n = c.shape[-1]
    g = min(group, n) if n else group
    out = (c.reshape(c.shape[:-1] + (n // g, g)) * s[..., None]).reshape(c.shape)
    return np.ascontiguousarray(np.moveaxis(out, -1, axis))


def quantize_tokens(X):
    """Per-token INT8: (codes int8 [M][K], scales float16 [M]); divisions in fp32 (see the head of this file)."""
    X = np.asarray(X, dtype=np.float32)
    if not np.all(np.isfinite(X)):
        raise ValueError("quantizer requires finite inputs")
    amax = np.abs(X).max(axis=1) if X.shape[1] else np.zeros(X.shape[0], np.float32)
    with np.errstate(over="ignore"):
        s = (amax.astype(np.float32) / np.float32(127.0)).astype(np.float16)
    if not np.all(np.isfinite(s)):
        raise ValueError("a token scale exceeds the fp16 range")
    s = np.where(amax == 0.0, np.float16(1.0), s)
    if np.any(s == 0):
        raise ValueError("a token scale underflows fp16")
    q = np.rint(X / s.astype(np.float32)[:, None])             # fp32 division, then round half to even
    return np.clip(q, -127, 127).astype(np.int8), s.astype(np.float16)


def build_factors_int(W, calib, k: int, mode: int = 1) -> IntLayer:
    """The offline step of Sec. 3 with the INT formats: W_q = q(W) (INT4, groups of 128 down each column),
    E_q = W - W_q, S from the calibration samples (App. A), rank-k split of S E_q (Eq. 4-5), A_k and B_k to INT8."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    if K % GROUP:
        raise ValueError("K must be a multiple of 128")
    kp = padded_rank(k)
    if not 0 <= k <= min(K, N) or kp > GROUP:
        raise ValueError("rank k must lie in [0, min(K, N, 128)]")
    wc, ws = group_quantize(W, 4, axis=0)
    E = W - group_dequantize(wc, ws, axis=0)
    s = calibrate_scale(calib) if mode == 1 else np.ones(K)
    Ap, Bp = np.zeros((K, kp)), np.zeros((kp, N))
    if k > 0:
        A, B, _ = error_factors(E, s, k)
        Ap[:, :k], Bp[:k] = A, B
    if kp == 0:
        return IntLayer(K=K, N=N, k=0, kp=0, Wc=mxint.pack_int4(np.ascontiguousarray(wc.T)), Ws=np.ascontiguousarray(ws.T),
                        Ac=np.zeros((0, K), np.int8), As=np.zeros((0, K // GROUP), np.float16),
                        Bc=np.zeros((N, 0), np.int8), Bs=np.ones(N, np.float16))
    ac, as_ = group_quantize(Ap, 8, axis=0)                    # [K][kp], [K/128][kp]
    bc, bs = group_quantize(Bp, 8, axis=0)                     # [kp][N], [1][N]
    return IntLayer(K=K, N=N, k=k, kp=kp,
                    Wc=mxint.pack_int4(np.ascontiguousarray(wc.T)), Ws=np.ascontiguousarray(ws.T),
                    Ac=np.ascontiguousarray(ac.T), As=np.ascontiguousarray(as_.T),
                    Bc=np.ascontiguousarray(bc.T), Bs=np.ascontiguousarray(bs.reshape(-1)))


def dequantize_layer(layer: IntLayer, cols=None):
    """(W^[K][n], A^[K][kp], B^[kp][n]) in fp64 for the output columns `cols` (all by default)."""
    cols = np.arange(layer.N) if cols is None else np.asarray(cols)
    W_hat = group_dequantize(mxint.unpack_int4(layer.Wc[cols]), layer.Ws[cols], axis=1).T
    A_hat = group_dequantize(layer.Ac, layer.As, axis=1).T if layer.kp else np.zeros((layer.K, 0))
    B_hat = (layer.Bc[cols].astype(np.float64) * layer.Bs[cols].astype(np.float64)[:, None]).T
    return W_hat, A_hat, B_hat


def forward(X, layer: IntLayer, cols=None) -> np.ndarray:
    """Y[:, cols] = X_q W_q + (X_q A_k) B_k with per-token INT8 activations, fp64."""
    xc, xs = quantize_tokens(X)
    X_hat = xc.astype(np.float64) * xs.astype(np.float64)[:, None]
    W_hat, A_hat, B_hat = dequantize_layer(layer, cols)
    return X_hat @ W_hat + (X_hat @ A_hat) @ B_hat


def forward_magnitudes(X, layer: IntLayer, cols=None):
    """Sums of absolute values behind every element of Y, as oracle.forward.forward_magnitudes: (main, tail, proj)."""
    xc, xs = quantize_tokens(X)
    X_hat = xc.astype(np.float64) * xs.astype(np.float64)[:, None]
    W_hat, A_hat, B_hat = dequantize_layer(layer, cols)
    X_abs, B_abs = np.abs(X_hat), np.abs(B_hat)
    return X_abs @ np.abs(W_hat), np.abs(X_hat @ A_hat) @ B_abs, (X_abs @ np.abs(A_hat)) @ B_abs


def average_weight_bits(m: int, n: int, k: int, w_bits: int = 4, group: int = GROUP) -> float:
    """Stored bits per element of W: codes plus one FP16 scale per group, plus the INT8 factors with theirs (App. D)."""
    total = m * n * (w_bits + 16.0 / group) + (m + n) * k * 8 + (m // group) * k * 16 + n * 16
    return total / (m * n)
