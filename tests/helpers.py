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


def oracle_layer_big(K, N, k, seed=0, n_outlier=None, gain=50.0, chunk=512, w_bits=None):
    """W_q by the oracle quantizer, A_k/B_k from random stand-ins quantized by the oracle.
    Used where an exact SVD would take minutes; the forward pass only needs the bytes."""
    rng = np.random.default_rng(seed)
    n_outlier = max(1, round(0.01 * K)) if n_outlier is None else n_outlier
    ch = synth.gen_outlier_channels(rng, K, n_outlier)
    w_bits = factors.W_BITS if w_bits is None else w_bits
    Wc = np.empty((N, K * w_bits // 8), np.uint8)
    We = np.empty((N, K // 16), np.uint8)
    for n0 in range(0, N, chunk):
        n1 = min(N, n0 + chunk)
        W = synth.gen_weight(rng, K, n1 - n0)
        c, e = mxint.mx_quantize(W, w_bits, axis=0)
        Wc[n0:n1] = mxint.pack_codes(np.ascontiguousarray(c.T), w_bits)
        We[n0:n1] = e.T
    kp = factors.padded_rank(k)
    A, B = synth.gen_factor_standins(rng, K, N, k, ch, gain)
    Ap = np.zeros((K, kp)); Ap[:, :k] = A
    Bp = np.zeros((kp, N)); Bp[:k] = B
    ac, ae = mxint.mx_quantize(Ap, factors.H_BITS, axis=0)
    bc, be = mxint.mx_quantize(Bp, factors.H_BITS, axis=0)
    layer = factors.PackedLayer(K=K, N=N, k=k, kp=kp, w_bits=w_bits, Wc=Wc, We=We,
                                Ac=np.ascontiguousarray(ac.T), Ae=np.ascontiguousarray(ae.T),
                                Bc=np.ascontiguousarray(bc.T), Be=np.ascontiguousarray(be.T))
    return layer, ch


def upload(layer):
    from paper_2402_02446_amd import binding
    fac = (layer.Ac, layer.Ae, layer.Bc, layer.Be) if layer.k > 0 else ()
    if getattr(layer, "w_bits", 4) != 4:
        return binding.lqer_layer_import_w(layer.w_bits, layer.K, layer.N, layer.k, layer.Wc, layer.We, *fac)
    return binding.lqer_layer_import(layer.K, layer.N, layer.k, layer.Wc, layer.We, *fac)


# Elementwise bar beside the norm.  Every product that enters an accumulator is exact; what rounds is the fp32
# accumulation (unit roundoff u = 2^-24) over n = K + 2 kp terms, the fp32 accumulation inside T = X_q A_k
# (K terms) and the split of T into two bf16 terms, each cut off after 8 significant bits (relative 2^-14 at worst).  A sum of n terms added in fp32 in any
# order is within n u sum|terms| of the exact sum in the worst case and within a few sqrt(n) u sum|terms| with
# overwhelming probability; the tests assert, elementwise,
#   |Y - Y_ref| <= (C sqrt(n) + C0) u (main + tail) + 2^-14 tail + (C sqrt(K) + C0) u proj
# with the magnitude sums of oracle.forward.forward_magnitudes, C = 1/4 and C0 = 4 (the handful of roundings
# that do not shrink with K: the hand-over of partial sums, the final store).  For every size tested this is
# below the worst-case bound n u sum|terms|; the largest |error| / bound measured over the full-size workloads is 0.15.
ELEM_C = 0.25
ELEM_C0 = 4.0
U32 = 2.0 ** -24


def elementwise_bound(main, tail, proj, K, kp):
    n = K + 2 * kp
    return ((ELEM_C * np.sqrt(n) + ELEM_C0) * U32 * (main + tail) + 2.0 ** -14 * tail
            + (ELEM_C * np.sqrt(K) + ELEM_C0) * U32 * proj)


def assert_forward_matches(Y, X, layer, cols=None, act_bits=8, tol=Y_TOL_DERIVED):
    """Y (or its columns `cols`) for the token rows X against the oracle: relative Frobenius error within the
    stated bar and the derived one, every element within the rounding bound above, everything finite.
    Returns (relative Frobenius error, largest |error| / bound)."""
    Y = np.asarray(Y, np.float64)
    if cols is None:
        Yref = forward.forward(X, layer, act_bits=act_bits)
    else:
        Yref = forward.forward_cols(X, layer, cols, act_bits=act_bits)
    assert Y.shape == Yref.shape, (Y.shape, Yref.shape)
    assert np.all(np.isfinite(Y))
    err = forward.rel_frobenius(Y, Yref)
    assert err <= Y_TOL, err
    assert err <= tol, err
    main, tail, proj = forward.forward_magnitudes(X, layer, cols, act_bits=act_bits)
    bound = elementwise_bound(main, tail, proj, layer.K, layer.kp)
    diff = np.abs(Y - Yref)
    bad = diff > bound
    ratio = float((diff / np.maximum(bound, np.finfo(np.float64).tiny)).max()) if diff.size else 0.0
    assert not bad.any(), (f"{int(bad.sum())} elements outside the rounding bound, first at {np.argwhere(bad)[0].tolist()}, "
                           f"largest |error| / bound = {ratio:.3g}")
    return err, ratio


def tile_cover_samples(rng, M, N, row_band=32, col_band=32):
    """Row and column indices such that every row_band x col_band block of an M x N output holds one compared
    element (one random row per band of rows, one random column per band of columns, compared as a cross
    product), plus the corners: every output tile of every kernel shape, every wavefront's part of it and
    every 32 x 32 MFMA tile is then touched."""
    rows = [min(M - 1, b + int(rng.integers(0, row_band))) for b in range(0, M, row_band)]
    cols = [min(N - 1, b + int(rng.integers(0, col_band))) for b in range(0, N, col_band)]
    return np.unique(np.r_[0, M - 1, rows]), np.unique(np.r_[0, N - 1, cols])
