"""Inference pass of an LQER layer: oracle version.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

  X_q = q(X)            MXINT8, blocks of 16 along each token's channels (Sec. 4.1)
  T   = X_q A_k         kept in full precision, not re-quantized
  Y   = X_q W_q + T B_k                                   (Eq. 3, Eq. 6)

`forward` does this with three dense fp64 matmuls on the dequantized operands.
`forward_int_exact` is the same sum written the way Sec. 2.2 describes an
MXINT inner product: an integer dot product per block plus an exponent add.
"""
from __future__ import annotations

import numpy as np

from . import mxint
from .factors import PackedLayer, dequantize_layer, W_BITS, H_BITS


def quantize_activations(X, act_bits: int = H_BITS):
    """(codes[M][K] int8, exps[M][K/16] uint8) for activations X[M][K]; act_bits = 6 is the
    W4A6 setup of Table 2 (8-bit shared exponents for activations either way, Sec. 4.1)."""
    return mxint.mx_quantize(X, act_bits, axis=-1)


def forward_q(Xc, Xe, layer: PackedLayer, act_bits: int = H_BITS) -> np.ndarray:
    """Y from already-quantized activations, fp64."""
    X_hat = mxint.mx_dequantize(Xc, Xe, act_bits, axis=-1)
    W_hat, A_hat, B_hat = dequantize_layer(layer)
    T = X_hat @ A_hat
    return X_hat @ W_hat + T @ B_hat


def forward(X, layer: PackedLayer, act_bits: int = H_BITS) -> np.ndarray:
    """Y = X_q W_q + (X_q A_k) B_k for fp32 activations X[M][K], fp64 result."""
    Xc, Xe = quantize_activations(X, act_bits)
    return forward_q(Xc, Xe, layer, act_bits)


def forward_cols(X, layer: PackedLayer, cols, act_bits: int = H_BITS) -> np.ndarray:
    """Y[:, cols] of `forward` (Eq. 3, Eq. 6) for layers too wide to dequantize whole: only the
    selected output columns of W_q and B_k are expanded; A_k and T are the full ones."""
    cols = np.asarray(cols)
    Xc, Xe = quantize_activations(X, act_bits)
    X_hat = mxint.mx_dequantize(Xc, Xe, act_bits, axis=-1)
    W_sub = mxint.mx_dequantize(mxint.unpack_codes(layer.Wc[cols], layer.w_bits), layer.We[cols], layer.w_bits, axis=1).T   # [K][len(cols)]
    A_hat = mxint.mx_dequantize(layer.Ac, layer.Ae, H_BITS, axis=1).T                                     # [K][kp]
    B_sub = mxint.mx_dequantize(layer.Bc[cols], layer.Be[cols], H_BITS, axis=1).T                         # [kp][len(cols)]
    T = X_hat @ A_hat
    return X_hat @ W_sub + T @ B_sub


def forward_magnitudes(X, layer: PackedLayer, cols=None, act_bits: int = H_BITS):
    """The sums of absolute values behind every element of Y (Eq. 3, Eq. 6), for elementwise
    rounding bounds on an implementation that forms exact products and rounds only when adding:

      main[t][j]  = sum_i |X_q[t][i]| |W_q[i][j]|
      tail[t][j]  = sum_r |T[t][r]| |B_k[r][j]|             with T = X_q A_k
      proj[t][j]  = sum_r (sum_i |X_q[t][i]| |A_k[i][r]|) |B_k[r][j]|

    A sum of n exact terms added in any order in precision u differs from the exact sum by at most
    about n u times the sum of the terms' magnitudes (much less in practice); `main` bounds the main
    product that way, `proj` the rounding inside T carried through B_k, and `tail` both the second
    product and any rounding of T itself.  Returns (main, tail, proj), fp64, for the columns `cols`."""
    cols = np.arange(layer.N) if cols is None else np.asarray(cols)
    Xc, Xe = quantize_activations(X, act_bits)
    X_abs = np.abs(mxint.mx_dequantize(Xc, Xe, act_bits, axis=-1))
    X_hat = mxint.mx_dequantize(Xc, Xe, act_bits, axis=-1)
    W_abs = np.abs(mxint.mx_dequantize(mxint.unpack_codes(layer.Wc[cols], layer.w_bits), layer.We[cols], layer.w_bits, axis=1)).T
    A_hat = mxint.mx_dequantize(layer.Ac, layer.Ae, H_BITS, axis=1).T
    B_abs = np.abs(mxint.mx_dequantize(layer.Bc[cols], layer.Be[cols], H_BITS, axis=1)).T
    T = X_hat @ A_hat
    return X_abs @ W_abs, np.abs(T) @ B_abs, (X_abs @ np.abs(A_hat)) @ B_abs


def forward_int_exact(Xc, Xe, layer: PackedLayer) -> np.ndarray:
    """Same result through integer block dot products (Sec. 2.2).

    Main term:  sum over 16-blocks kb of 2^(ex + ew - 8) * sum_i Xc*Wc   (6 + 2 fraction bits)
    T:          sum over kb of 2^(ex + ea - 12) * sum_i Xc*Ac            (6 + 6 fraction bits)
    Tail:       sum_r T[:, r] * Bc[r] * 2^(eb - 6)
    Exponents are the unbiased ones.  fp64 accumulation of exact terms.
    """
    Xc = np.asarray(Xc).astype(np.int64)
    M, K = Xc.shape
    nb = K // mxint.BLOCK
    ex = np.asarray(Xe).astype(np.int64) - mxint.EXP_BIAS                    # [M][nb]
    Wc = mxint.unpack_codes(layer.Wc, layer.w_bits).astype(np.int64)         # [N][K]
    ew = layer.We.astype(np.int64) - mxint.EXP_BIAS                          # [N][nb]
    Ac = layer.Ac.astype(np.int64)
    ea = layer.Ae.astype(np.int64) - mxint.EXP_BIAS
    Xb = Xc.reshape(M, nb, mxint.BLOCK)
    Wb = Wc.reshape(layer.N, nb, mxint.BLOCK)
    Ab = Ac.reshape(layer.kp, nb, mxint.BLOCK)
    Y = np.zeros((M, layer.N), dtype=np.float64)
    T = np.zeros((M, layer.kp), dtype=np.float64)
    for kb in range(nb):
        dw = Xb[:, kb, :] @ Wb[:, kb, :].T                                   # int64 [M][N]
        Y += np.ldexp(dw.astype(np.float64),
                      ex[:, kb][:, None] + ew[:, kb][None, :] - (H_BITS - 2) - (layer.w_bits - 2))
        da = Xb[:, kb, :] @ Ab[:, kb, :].T
        T += np.ldexp(da.astype(np.float64),
                      ex[:, kb][:, None] + ea[:, kb][None, :] - 2 * (H_BITS - 2))
    B_hat = mxint.mx_dequantize(layer.Bc, layer.Be, H_BITS, axis=1).T        # [kp][N]
    return Y + T @ B_hat


def rel_frobenius(Y, Y_ref) -> float:
    """Parity metric for Y: ||Y - Y_ref||_F / ||Y_ref||_F."""
    Y = np.asarray(Y, np.float64)
    Y_ref = np.asarray(Y_ref, np.float64)
    den = np.linalg.norm(Y_ref)
    return float(np.linalg.norm(Y - Y_ref) / den) if den > 0 else float(np.linalg.norm(Y))
