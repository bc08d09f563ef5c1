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
    Wc = mxint.unpack_int4(layer.Wc).astype(np.int64)                        # [N][K]
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
                      ex[:, kb][:, None] + ew[:, kb][None, :] - (H_BITS - 2) - (W_BITS - 2))
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
