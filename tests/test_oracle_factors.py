"""Pins for the oracle's offline step (Sec. 3.1 Eq. 1-2, Sec. 3.2 Eq. 4-5,
App. A Eq. 7-8): Eckart-Young, exact recovery at full rank, the closed forms,
a brute-force Jacobi SVD, and the invariants of the S-scaled split."""
import os

import numpy as np
import pytest

from oracle import factors, mxint
from paper_2402_02446_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _small_problem(seed=0, K=64, N=48, outliers=4, gain=30.0):
    rng = np.random.default_rng(seed)
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, outliers)
    calib = np.stack([synth.gen_activations(rng, 32, K, ch, gain) for _ in range(3)])
    return W, calib


def _jacobi_singular_values(M):
    """One-sided Jacobi on the columns of M: plain rotations until orthogonal."""
    A = np.array(M, dtype=np.float64)
    n = A.shape[1]
    for _ in range(60):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                alpha = A[:, p] @ A[:, p]
                beta = A[:, q] @ A[:, q]
                gamma = A[:, p] @ A[:, q]
                if abs(gamma) <= 1e-300:
                    continue
                off = max(off, abs(gamma) / np.sqrt(alpha * beta))
                zeta = (beta - alpha) / (2.0 * gamma)
                t = np.sign(zeta) / (abs(zeta) + np.sqrt(1.0 + zeta * zeta)) if zeta != 0 else 1.0
                c = 1.0 / np.sqrt(1.0 + t * t)
                s = c * t
                ap = A[:, p].copy()
                A[:, p] = c * ap - s * A[:, q]
                A[:, q] = s * ap + c * A[:, q]
        if off < 1e-15:
            break
    return np.sort(np.linalg.norm(A, axis=0))[::-1]


def test_calibration_hand_example():
    # App. A: per-sample mean magnitude, max over samples, geometric-mean normalisation.
    calib = np.array([[[1.0, -2.0], [3.0, 6.0]], [[-5.0, 0.0], [1.0, 1.0]]])
    # a_1 = [2, 4], a_2 = [3, 0.5], abar = [3, 4], s = abar / sqrt(3*4)
    s = factors.calibrate_scale(calib)
    assert np.allclose(s, [3.0 / np.sqrt(12.0), 4.0 / np.sqrt(12.0)], rtol=0, atol=1e-15)


def test_calibration_brute_force():
    rng = np.random.default_rng(4)
    calib = rng.standard_normal((3, 5, 7))
    K = 7
    abar = [max(sum(abs(calib[i, r, c]) for r in range(5)) / 5 for i in range(3)) for c in range(K)]
    norm = (min(abar) * max(abar)) ** 0.5
    assert np.allclose(factors.calibrate_scale(calib), [a / norm for a in abar], rtol=1e-14)


def test_singular_scale_rejected():
    calib = np.ones((1, 4, 16))
    calib[:, :, 3] = 0.0
    with pytest.raises(ValueError):
        factors.calibrate_scale(calib)
    calib[:, :, 3] = np.inf
    with pytest.raises(ValueError):
        factors.calibrate_scale(calib)


def test_weight_quantization_error_is_small_and_columnwise():
    W, _ = _small_problem()
    codes, exps, W_hat = factors.quantize_weight(W)
    assert codes.shape == W.shape and exps.shape == (W.shape[0] // 16, W.shape[1])
    assert np.abs(codes).max() <= 7
    # blocks run down the columns: column j, rows 16b..16b+15 share exps[b, j]
    for j in (0, 17):
        for b in (0, 3):
            blk = W[16 * b:16 * b + 16, j]
            c, x = mxint.mx_quantize(blk, 4)
            assert np.array_equal(c, codes[16 * b:16 * b + 16, j]) and x[0] == exps[b, j]
    step = np.ldexp(1.0, exps.astype(np.int64) - 127 - 2)
    assert np.all(np.abs(W - W_hat) <= np.repeat(step, 16, axis=0))


@pytest.mark.parametrize("k", [1, 8, 20])
def test_eckart_young(k):
    W, calib = _small_problem()
    _, _, W_hat = factors.quantize_weight(W)
    E = W.astype(np.float64) - W_hat
    s = factors.calibrate_scale(calib)
    A, B, _ = factors.error_factors(E, s, k)
    SE = s[:, None] * E
    # singular values from a different routine: eigenvalues of the Gram matrix
    sig2 = np.sort(np.linalg.eigvalsh(SE.T @ SE))[::-1]
    res = np.linalg.norm(SE - s[:, None] * (A @ B)) ** 2
    assert np.isclose(res, sig2[k:].sum(), rtol=1e-9)
    assert np.isclose(res, np.linalg.norm(SE) ** 2 - sig2[:k].sum(), rtol=1e-9)
    # the split itself: S A has orthonormal columns, B's rows are orthogonal with norms sigma_i
    SA = s[:, None] * A
    assert np.allclose(SA.T @ SA, np.eye(k), atol=1e-12)
    BBt = B @ B.T
    assert np.allclose(BBt, np.diag(sig2[:k]), rtol=1e-8, atol=1e-12 * sig2[0])


def test_matches_bruteforce_jacobi():
    rng = np.random.default_rng(1)
    E = rng.standard_normal((32, 16)) * 1e-3
    s = np.exp(rng.standard_normal(32))
    _, _, sig = factors.error_factors(E, s, 4)
    assert np.allclose(sig, _jacobi_singular_values(s[:, None] * E), rtol=1e-10)


def test_rank_k_is_optimal_against_random_competitors():
    W, calib = _small_problem(seed=3)
    _, _, W_hat = factors.quantize_weight(W)
    E = W.astype(np.float64) - W_hat
    s = factors.calibrate_scale(calib)
    k = 6
    A, B, _ = factors.error_factors(E, s, k)
    best = np.linalg.norm(s[:, None] * (E - A @ B))
    rng = np.random.default_rng(0)
    for _ in range(20):
        P = rng.standard_normal((E.shape[0], k))
        Q, _ = np.linalg.qr(P)
        comp = Q @ (Q.T @ (s[:, None] * E))          # best approximation in a random k-dim column space
        assert best <= np.linalg.norm(s[:, None] * E - comp) + 1e-15


def test_full_rank_recovers_w_exactly():
    W, calib = _small_problem(K=48, N=32)
    _, _, W_hat = factors.quantize_weight(W)
    E = W.astype(np.float64) - W_hat
    for s in (np.ones(48), factors.calibrate_scale(calib)):
        A, B, _ = factors.error_factors(E, s, 32)
        assert np.linalg.norm(W - W_hat - A @ B) / np.linalg.norm(W) < 1e-12


def test_rank_one_closed_form():
    rng = np.random.default_rng(8)
    u = rng.standard_normal(32)
    v = rng.standard_normal(16)
    s = np.exp(rng.standard_normal(32))
    E = np.outer(u / s, v)                     # S E = u v^T has rank one
    A, B, sig = factors.error_factors(E, s, 1)
    assert np.allclose(A @ B, E, rtol=1e-12, atol=1e-15)
    assert np.isclose(sig[0], np.linalg.norm(u) * np.linalg.norm(v), rtol=1e-12)
    assert np.all(sig[1:] < 1e-12 * sig[0])


def test_scale_normalisation_is_irrelevant_to_the_product():
    W, calib = _small_problem(seed=5)
    _, _, W_hat = factors.quantize_weight(W)
    E = W.astype(np.float64) - W_hat
    s = factors.calibrate_scale(calib)
    A1, B1, _ = factors.error_factors(E, s, 5)
    A2, B2, _ = factors.error_factors(E, 37.5 * s, 5)
    assert np.allclose(A1 @ B1, A2 @ B2, rtol=1e-9, atol=1e-15)


def test_identity_scale_is_plain_truncated_svd_and_weighting_helps_in_weighted_norm():
    W, calib = _small_problem(seed=6)
    _, _, W_hat = factors.quantize_weight(W)
    E = W.astype(np.float64) - W_hat
    s = factors.calibrate_scale(calib)
    k = 8
    A0, B0, sig0 = factors.error_factors(E, np.ones(E.shape[0]), k)
    # S = I: A has orthonormal columns itself and the residual is E's own singular tail
    assert np.allclose(A0.T @ A0, np.eye(k), atol=1e-12)
    assert np.isclose(np.linalg.norm(E - A0 @ B0) ** 2, (sig0[k:] ** 2).sum(), rtol=1e-9)
    A1, B1, _ = factors.error_factors(E, s, k)
    w0 = np.linalg.norm(s[:, None] * (E - A0 @ B0))
    w1 = np.linalg.norm(s[:, None] * (E - A1 @ B1))
    u0 = np.linalg.norm(E - A0 @ B0)
    u1 = np.linalg.norm(E - A1 @ B1)
    assert w1 <= w0 * (1 + 1e-12)        # L2QER wins in the activation-weighted norm
    assert u0 <= u1 * (1 + 1e-12)        # plain LQER wins in the unweighted norm


def test_build_factors_layout_and_padding():
    W, calib = _small_problem()
    K, N = W.shape
    layer = factors.build_factors(W, calib, k=8, mode=1)
    assert (layer.K, layer.N, layer.k, layer.kp) == (K, N, 8, 16)
    assert layer.Wc.shape == (N, K // 2) and layer.We.shape == (N, K // 16)
    assert layer.Ac.shape == (16, K) and layer.Ae.shape == (16, K // 16)
    assert layer.Bc.shape == (N, 16) and layer.Be.shape == (N, 1)
    # padded ranks quantize to nothing
    assert not layer.Ac[8:].any() and not layer.Ae[8:].any() and not layer.Bc[:, 8:].any()
    W_hat, A_hat, B_hat = factors.dequantize_layer(layer)
    codes, exps, W_hat_direct = factors.quantize_weight(W)
    assert np.array_equal(W_hat, W_hat_direct)
    assert np.array_equal(mxint.unpack_int4(layer.Wc), codes.T)
    # the quantized correction still reduces the weighted error noticeably
    s = factors.calibrate_scale(calib)
    E = W.astype(np.float64) - W_hat
    assert np.linalg.norm(s[:, None] * (E - A_hat @ B_hat)) < 0.97 * np.linalg.norm(s[:, None] * E)
    # k = 0 is allowed and produces empty factors
    l0 = factors.build_factors(W, calib, k=0)
    assert l0.kp == 0 and l0.Ac.shape == (0, K) and l0.Bc.shape == (N, 0)
    with pytest.raises(ValueError):
        factors.build_factors(W, calib, k=min(K, N) + 1)


def test_extra_multiplies_closed_form():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_closed_forms.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, val, _ = [p.strip() for p in line.split("|")]
                vals[name] = float(val)
    pct_per_rank = 100.0 * factors.extra_multiply_ratio(12288, 49152, 1)
    assert round(pct_per_rank, 2) == vals["extra_multiply_percent_per_rank_opt175b_ffn"]
    assert factors.extra_multiply_ratio(10, 20, 3) == (10 + 20) * 3 / 200


def test_approximation_error_metric():
    E = np.array([[1.0, -2.0], [0.5, 0.0]])
    Et = np.array([[0.5, -1.0], [0.5, 1.0]])
    assert factors.approximation_error(E, Et) == (0.5 + 1.0 + 0.0 + 1.0) / 4


def test_four_bit_shared_exponents_in_the_offline_step():
    # Sec. 4.1: W_q, A_k, B_k with 4-bit shared exponents (one bias per tensor).  On weights of a few binades
    # the narrow exponent reaches every block: W_q is that of the 8-bit-exponent build, and so is E_q.
    rng = np.random.default_rng(5)
    W = synth.gen_weight(rng, 128, 96)
    ch = synth.gen_outlier_channels(rng, 128, 4)
    calib = np.stack([synth.gen_activations(rng, 32, 128, ch, 30.0)])
    a = factors.build_factors(W, calib, 8, 1)
    b = factors.build_factors(W, calib, 8, 1, exp_bits=4)
    assert np.array_equal(a.Wc, b.Wc) and np.array_equal(a.We, b.We)
    for e in (b.We, b.Ae, b.Be):
        assert int(e.max()) - int(e.min()) <= 15
    # the factors may lose low bits of their smallest blocks, never more than the error they correct
    s = factors.calibrate_scale(calib)
    W_hat, A8, B8 = factors.dequantize_layer(a)
    _, A4, B4 = factors.dequantize_layer(b)
    E = W.astype(np.float64) - W_hat
    r8 = np.linalg.norm(s[:, None] * (E - A8 @ B8))
    r4 = np.linalg.norm(s[:, None] * (E - A4 @ B4))
    assert r4 <= 1.02 * r8 and r4 < np.linalg.norm(s[:, None] * E)
    # full rank still recovers W up to the quantization of the factors
    W2 = synth.gen_weight(rng, 64, 48)
    full = factors.build_factors(W2, None, 48, 0, exp_bits=4)
    Wh, A, B = factors.dequantize_layer(full)
    assert np.linalg.norm(W2 - Wh - A @ B) < 0.05 * np.linalg.norm(W2 - Wh)
    # stored size (App. D): 4.25 bits per weight instead of 4.5, 8.25 instead of 8.5 per factor element
    assert mxint.lqer_average_weight_bits(4096, 4096, 32, 4, 8, 4, 4) == pytest.approx(4.25 + 8.25 * 32 * 8192 / 4096 ** 2)


def test_two_bit_weights_in_the_offline_step():
    # the W2A8 setup (Sec. 4.1, Sec. 4.4): W_q has 2-bit mantissas, four per byte; E_q = W - W_q is much larger than
    # with 4 bits, the split of S E_q still satisfies Eckart-Young, and a high rank recovers most of it
    rng = np.random.default_rng(21)
    K, N = 64, 48
    W = synth.gen_weight(rng, K, N)
    calib = np.abs(rng.standard_normal((2, 16, K))).astype(np.float32) + 0.1
    l2 = factors.build_factors(W, calib, 32, 1, w_bits=2)
    l4 = factors.build_factors(W, calib, 32, 1)
    assert l2.w_bits == 2 and l2.Wc.shape == (N, K // 4) and l4.Wc.shape == (N, K // 2)
    codes, exps, W_hat = factors.quantize_weight(W, w_bits=2)
    assert np.array_equal(mxint.unpack_int2(l2.Wc), codes.T) and np.array_equal(l2.We, exps.T)
    assert set(np.unique(codes).tolist()) <= {-1, 0, 1}
    W2, A2, B2 = factors.dequantize_layer(l2)
    W4, _, _ = factors.dequantize_layer(l4)
    assert np.array_equal(W2, W_hat)
    e2, e4 = np.linalg.norm(W - W2), np.linalg.norm(W - W4)
    assert e2 > 3 * e4
    s = factors.calibrate_scale(calib)
    E = W - W2
    A, B, sig = factors.error_factors(E, s, 32)
    resid = np.linalg.norm(s[:, None] * (E - A @ B)) ** 2
    assert abs(resid - (sig[32:] ** 2).sum()) <= 1e-10 * (sig ** 2).sum()
    # the quantized factors take back most of the weighted error
    assert np.linalg.norm(s[:, None] * (E - A2 @ B2)) < 0.5 * np.linalg.norm(s[:, None] * E)
