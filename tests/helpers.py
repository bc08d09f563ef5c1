"""Shared helpers for the parity tests: layers built by the oracle, uploaded through the C ABI."""
import numpy as np

from oracle import factors, forward, mxint
from paper_2402_02446_amd import synth

Y_TOL = 1e-3          # the bar: relative Frobenius error of Y against the fp64 oracle
Y_TOL_DERIVED = 2e-5  # what fp32 accumulation of exact products should achieve (about sqrt(K) * 2^-24)


def oracle_layer_small(K, N, k, seed=0, mode=1, outliers=4, gain=30.0, calib_rows=32):
    """Exact oracle construction (SVD) for sizes where that takes well under a second."""
    rng = np.random.default_rng(seed)
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, min(outliers, K))
    calib = np.stack([synth.gen_activations(rng, calib_rows, K, ch, gain)])
    return factors.build_factors(W, calib, k, mode), ch


def oracle_layer_big(K, N, k, seed=0, n_outlier=None, gain=50.0, chunk=512):
    """W_q by the oracle quantizer, A_k/B_k from random stand-ins quantized by the oracle.
    Used where an exact SVD would take minutes; the forward pass only needs the bytes."""
    rng = np.random.default_rng(seed)
    n_outlier = max(1, round(0.01 * K)) if n_outlier is None else n_outlier
    ch = synth.gen_outlier_channels(rng, K, n_outlier)
    Wc = np.empty((N, K // 2), np.uint8)
    We = np.empty((N, K // 16), np.uint8)
    for n0 in range(0, N, chunk):
        n1 = min(N, n0 + chunk)
        W = synth.gen_weight(rng, K, n1 - n0)
        c, e = mxint.mx_quantize(W, factors.W_BITS, axis=0)
        Wc[n0:n1] = mxint.pack_int4(np.ascontiguousarray(c.T))
        We[n0:n1] = e.T
    kp = factors.padded_rank(k)
    A, B = synth.gen_factor_standins(rng, K, N, k, ch, gain)
    Ap = np.zeros((K, kp)); Ap[:, :k] = A
    Bp = np.zeros((kp, N)); Bp[:k] = B
    ac, ae = mxint.mx_quantize(Ap, factors.H_BITS, axis=0)
    bc, be = mxint.mx_quantize(Bp, factors.H_BITS, axis=0)
    layer = factors.PackedLayer(K=K, N=N, k=k, kp=kp, Wc=Wc, We=We,
                                Ac=np.ascontiguousarray(ac.T), Ae=np.ascontiguousarray(ae.T),
                                Bc=np.ascontiguousarray(bc.T), Be=np.ascontiguousarray(be.T))
    return layer, ch


def upload(layer):
    from paper_2402_02446_amd import binding
    if layer.k == 0:
        return binding.lqer_layer_import(layer.K, layer.N, 0, layer.Wc, layer.We)
    return binding.lqer_layer_import(layer.K, layer.N, layer.k, layer.Wc, layer.We,
                                     layer.Ac, layer.Ae, layer.Bc, layer.Be)


def oracle_rows(X_rows, layer):
    """Oracle Y for a subset of token rows (rows are independent)."""
    return forward.forward(X_rows, layer)


def oracle_forward_cols(X, layer, cols):
    """Oracle Y[:, cols] computed column by column from the packed bytes (for very wide layers)."""
    Xc, Xe = forward.quantize_activations(X)
    X_hat = mxint.mx_dequantize(Xc, Xe, factors.H_BITS, axis=-1)
    Wsub = mxint.mx_dequantize(mxint.unpack_int4(layer.Wc[cols]), layer.We[cols], factors.W_BITS, axis=1)
    A_hat = mxint.mx_dequantize(layer.Ac, layer.Ae, factors.H_BITS, axis=1).T
    Bsub = mxint.mx_dequantize(layer.Bc[cols], layer.Be[cols], factors.H_BITS, axis=1)
    T = X_hat @ A_hat
    return X_hat @ Wsub.T + T @ Bsub.T
