"""Offline construction of an LQER / L2QER layer: oracle version.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Steps, in the paper's order and notation (W is m x n = K x N, Y = X W):

  W_q = q(W)                       Sec. 3.1; MXINT4, blocks of 16 down each column (Sec. 4.1)
  E_q = W - W_q                    Eq. 1
  a_i = mean(|X_i|, axis=0);  a = max_i a_i;  s = a / sqrt(min(a) max(a))     App. A, Eq. 7-8
  S E_q = U' Sigma' V'^T           Eq. 4   (S = I gives Eq. 2, plain LQER)
  A'_k = S^-1 U'_k,  B'_k = Sigma'_k V'_k^T                                   Eq. 5
  A_k, B_k -> MXINT8, blocks of 16 down each column (Sec. 4.1), after zero
  padding the rank to a multiple of 16 so B_k's blocks (which run along k) are whole.

Canonical packed layer (contraction axis contiguous everywhere):
  Wc[N][K/2] nibble-packed int4, We[N][K/16]; Ac[kp][K] int8, Ae[kp][K/16];
  Bc[N][kp] int8, Be[N][kp/16].
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import mxint

W_BITS = 4
H_BITS = 8


@dataclass
class PackedLayer:
    K: int
    N: int
    k: int
    kp: int
    Wc: np.ndarray   # uint8 [N][K/2]
    We: np.ndarray   # uint8 [N][K/16]
    Ac: np.ndarray   # int8  [kp][K]
    Ae: np.ndarray   # uint8 [kp][K/16]
    Bc: np.ndarray   # int8  [N][kp]
    Be: np.ndarray   # uint8 [N][kp/16]
    w_bits: int = 4  # mantissa width of W_q: 4, or 2 (Wc is then [N][K/4], four codes per byte)


def padded_rank(k: int) -> int:
    return ((k + mxint.BLOCK - 1) // mxint.BLOCK) * mxint.BLOCK


def calibrate_scale(calib) -> np.ndarray:
    """S's diagonal from calibration samples (App. A, Eq. 7-8).

    `calib` is [n_samples][rows_per_sample][K].  Raises if a channel's magnitude
    is zero or not finite: the method needs S^-1 (Sec. 3.2).
    """
    x = np.abs(np.asarray(calib, dtype=np.float64))
    if x.ndim != 3:
        raise ValueError("calib must be [n_samples][rows][K]")
    a = x.mean(axis=1)            # a_i: per-sample mean magnitude of each channel
    abar = a.max(axis=0)          # maximum over samples
    if not np.all(np.isfinite(abar)) or np.any(abar <= 0.0):
        raise ValueError("singular activation scale: a calibrated channel is <= 0 or non-finite")
    return abar / np.sqrt(abar.min() * abar.max())


def quantize_weight(W, exp_bits: int = 8, w_bits: int = W_BITS):
    """W_q = q(W): returns (codes[K][N] int8, exps[K/16][N] uint8, dequantized fp64).
    w_bits = 2 is the W2A8 setup of Sec. 4.1 / Sec. 4.4."""
    W = np.asarray(W, dtype=np.float64)
    codes, exps = mxint.mx_quantize(W, w_bits, axis=0, exp_bits=exp_bits)
    return codes, exps, mxint.mx_dequantize(codes, exps, w_bits, axis=0)


def error_factors(E, s, k: int):
    """Rank-k split of the (scaled) quantization error, unquantized fp64.

    Returns (A[K][k], B[k][N], sigma[min(K,N)]) with A = S^-1 U_k and
    B = Sigma_k V_k^T for the SVD of S E (Eq. 4-5).
    """
    E = np.asarray(E, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    U, sig, Vt = np.linalg.svd(s[:, None] * E, full_matrices=False)
    A = U[:, :k] / s[:, None]
    B = sig[:k, None] * Vt[:k, :]
    return A, B, sig


def pack_layer(w_codes, w_exps, A, B, k: int, exp_bits: int = 8, w_bits: int = W_BITS) -> PackedLayer:
    """Quantize A, B to MXINT8 and lay every tensor out canonically."""
    K, N = w_codes.shape
    kp = padded_rank(k)
    Ap = np.zeros((K, kp), dtype=np.float64)
    Bp = np.zeros((kp, N), dtype=np.float64)
    Ap[:, :k] = A
    Bp[:k, :] = B
    a_codes, a_exps = mxint.mx_quantize(Ap, H_BITS, axis=0, exp_bits=exp_bits)      # blocks down K
    b_codes, b_exps = mxint.mx_quantize(Bp, H_BITS, axis=0, exp_bits=exp_bits)      # blocks down k
    return PackedLayer(
        K=K, N=N, k=k, kp=kp,
        w_bits=w_bits,
        Wc=mxint.pack_codes(np.ascontiguousarray(w_codes.T), w_bits),
        We=np.ascontiguousarray(w_exps.T),
        Ac=np.ascontiguousarray(a_codes.T),
        Ae=np.ascontiguousarray(a_exps.T),
        Bc=np.ascontiguousarray(b_codes.T),
        Be=np.ascontiguousarray(b_exps.T),
    )


def build_factors(W, calib, k: int, mode: int = 1, exp_bits: int = 8, w_bits: int = W_BITS) -> PackedLayer:
    """The whole offline step.  mode 0 = LQER (S = I), mode 1 = L2QER.
    exp_bits: width of the shared exponents of W_q, A_k and B_k (Sec. 4.1 uses 4).
    w_bits: mantissa width of W_q, 4 or 2 (the W2A8 setup, which Sec. 4.1 runs with k = 256)."""
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    if not 0 <= k <= min(K, N):
        raise ValueError("rank k must lie in [0, min(K, N)]")
    w_codes, w_exps, W_hat = quantize_weight(W, exp_bits, w_bits)
    E = W - W_hat
    s = calibrate_scale(calib) if mode == 1 else np.ones(K)
    if k > 0:
        A, B, _ = error_factors(E, s, k)
    else:
        A, B = np.zeros((K, 0)), np.zeros((0, N))
    return pack_layer(w_codes, w_exps, A, B, k, exp_bits, w_bits)


def dequantize_layer(layer: PackedLayer):
    """(W^[K][N], A^[K][kp], B^[kp][N]) in fp64 from the canonical bytes."""
    Wc = mxint.unpack_codes(layer.Wc, layer.w_bits)                         # [N][K]
    W_hat = mxint.mx_dequantize(Wc, layer.We, layer.w_bits, axis=1).T
    A_hat = mxint.mx_dequantize(layer.Ac, layer.Ae, H_BITS, axis=1).T
    B_hat = mxint.mx_dequantize(layer.Bc, layer.Be, H_BITS, axis=1).T
    return W_hat, A_hat, B_hat


def approximation_error(E, E_tilde) -> float:
    """e_a: mean absolute elementwise reconstruction error (App. B, Eq. 9)."""
    return float(np.mean(np.abs(np.asarray(E, np.float64) - np.asarray(E_tilde, np.float64))))


def extra_multiply_ratio(m: int, n: int, k: int) -> float:
    """High-precision multiplies the low-rank branch adds per token, relative
    to the m*n of the dense layer (Sec. 3.1)."""
    return (m + n) * k / (m * n)
