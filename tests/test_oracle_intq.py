"""Pins for the oracle's scaled-integer formats (Table 2 "L2QER-INT": INT4 g128 weights, INT8 per-token
activations; Sec. 2.1 for the form of such formats): exact-rational brute force, hand cases, the invariants of the
reading, the Table 2 bit count, and the forward pass against exact rationals from the bytes."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import factors, intq, mxint
from paper_2402_02446_amd import synth


def _rne(x: Fraction) -> int:
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def _fp16_rne(x: Fraction) -> Fraction:
    """x > 0 rounded to the nearest fp16 (ties to even), by search over the format: 11 significant bits,
    exponents -14..15, subnormals below."""
    e = 0
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    e = max(e, -14)
    ulp = Fraction(2) ** (e - 10)
    return _rne(x / ulp) * ulp


@pytest.mark.parametrize("bits", [4, 8])
def test_group_quantizer_by_exact_rationals(bits):
    rng = np.random.default_rng(3)
    v = (rng.standard_normal((6, 256)) * np.exp2(rng.integers(-6, 3, (6, 1)))).astype(np.float32)
    v[1, 5] = 0.02 * 7.5 / 7 * 7          # a few exact ties in code units
    v[2, :128] = 0.0                       # an all-zero group
    codes, scales = intq.group_quantize(v, bits)
    qmax = 2 ** (bits - 1) - 1
    for r in range(v.shape[0]):
        for g in range(2):
            blk = [Fraction(float(x)) for x in v[r, 128 * g:128 * (g + 1)]]
            amax = max(abs(x) for x in blk)
            s = Fraction(1) if amax == 0 else _fp16_rne(amax / qmax)
            assert Fraction(float(scales[r, g])) == s
            want = [max(-qmax, min(qmax, _rne(x / s))) for x in blk]
            assert codes[r, 128 * g:128 * (g + 1)].tolist() == want


def test_group_quantizer_hand_cases():
    # amax = 7 -> s = 1, codes are the rounded values; amax = 3.5 -> s = 0.5; ties go to the even code
    blk = np.zeros(128, np.float32)
    blk[:6] = [7.0, -3.0, 2.5, 3.5, -0.5, 0.49]
    c, s = intq.group_quantize(blk, 4)
    assert float(s[0]) == 1.0 and c[:6].tolist() == [7, -3, 2, 4, 0, 0]
    blk[:6] = [3.5, 0.25, 0.75, -1.25, 1.0, 0.0]
    c, s = intq.group_quantize(blk, 4)
    assert float(s[0]) == 0.5 and c[:6].tolist() == [7, 0, 2, -2, 2, 0]
    blk[:3] = [127.0, 1.5, -2.5]
    blk[3:6] = 0
    c, s = intq.group_quantize(blk, 8)
    assert float(s[0]) == 1.0 and c[:3].tolist() == [127, 2, -2]
    # 0.1 / 7 is no fp16 number: the stored scale is its nearest neighbour and the largest element still maps to 7
    blk[:] = 0
    blk[0] = 0.1
    c, s = intq.group_quantize(blk, 4)
    assert s.dtype == np.float16 and abs(float(s[0]) - 0.1 / 7) <= 2.0 ** -17 and c[0] == 7


@pytest.mark.parametrize("bits", [4, 8])
def test_group_quantizer_invariants(bits):
    rng = np.random.default_rng(5)
    v = (rng.standard_normal((40, 384)) * 0.02).astype(np.float32)
    c, s = intq.group_quantize(v, bits)
    qmax = 2 ** (bits - 1) - 1
    assert np.abs(c).max() <= qmax
    cn, sn = intq.group_quantize(-v, bits)
    assert np.array_equal(cn, -c) and np.array_equal(sn, s)                  # antisymmetry
    c8, s8 = intq.group_quantize(v * 8, bits)                                # powers of two move the scale only
    assert np.array_equal(c8, c) and np.array_equal(s8.astype(np.float64), s.astype(np.float64) * 8)
    v_hat = intq.group_dequantize(c, s)
    sd = np.repeat(s.astype(np.float64), 128, axis=1)
    unsat = np.abs(np.rint(v / sd)) <= qmax
    assert np.all(np.abs(v - v_hat)[unsat] <= 0.5 * sd[unsat] * (1 + 1e-12))  # half a step unless clamped
    assert np.all(np.abs(v - v_hat) <= sd * (1 + 2.0 ** -10))                # the fp16 rounding of s can clamp the largest by < 1 step
    # the element that sets the scale gets the largest code (the scale is amax / qmax up to fp16 rounding)
    big = np.abs(v.reshape(40, 3, 128)).argmax(axis=2)
    cc = np.abs(c.reshape(40, 3, 128))
    assert np.all(np.take_along_axis(cc, big[..., None], axis=2) == qmax)
    # axis argument = transpose
    c0, s0 = intq.group_quantize(v.T, bits, axis=0)
    assert np.array_equal(c0.T, c) and np.array_equal(s0.T, s)


def test_token_quantizer_by_fp32_steps():
    # per-token INT8 with the divisions in fp32: every step retyped with numpy scalars, row by row
    rng = np.random.default_rng(8)
    ch = synth.gen_outlier_channels(rng, 256, 3)
    X = synth.gen_activations(rng, 9, 256, ch, 50.0)
    X[4] = 0.0
    c, s = intq.quantize_tokens(X)
    assert c.dtype == np.int8 and s.dtype == np.float16
    for t in range(X.shape[0]):
        amax = np.float32(np.abs(X[t]).max())
        st = np.float16(1.0) if amax == 0 else np.float16(np.float32(amax / np.float32(127.0)))
        assert s[t] == st
        for j in range(0, 256, 17):
            q = np.float32(X[t, j]) / np.float32(st)
            assert int(c[t, j]) == int(max(-127, min(127, np.rint(q))))
    assert np.all(np.abs(c).max(axis=1)[[0, 1, 2, 3, 5]] >= 126) and not c[4].any()
    cn, sn = intq.quantize_tokens(-X)
    assert np.array_equal(cn, -c) and np.array_equal(sn, s)


def test_table2_bits_of_int4_g128():
    # Table 2 lists 4.1 average weight bits for INT4 g128: 4 + 16 / 128
    assert intq.average_weight_bits(4096, 4096, 0) == pytest.approx(4.125 + 16 / 4096)
    assert round(4 + 16 / 128, 1) == 4.1
    # with rank-32 INT8 factors the LLaMA-7B-sized layer stores 0.13 bits more per weight
    assert intq.average_weight_bits(4096, 4096, 32) - intq.average_weight_bits(4096, 4096, 0) == pytest.approx(0.127, abs=2e-3)


def _layer(seed=0, K=256, N=48, k=8, mode=1):
    rng = np.random.default_rng(seed)
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, 4)
    calib = np.stack([synth.gen_activations(rng, 32, K, ch, 30.0)])
    X = synth.gen_activations(rng, 5, K, ch, 30.0)
    return W, calib, X, intq.build_factors_int(W, calib, k, mode)


def test_offline_step_layout_and_optimality():
    W, calib, X, layer = _layer(seed=1, k=20)
    K, N = W.shape
    assert layer.kp == 32 and layer.Wc.shape == (N, K // 2) and layer.Ws.shape == (N, K // 128)
    assert layer.Ac.shape == (32, K) and layer.As.shape == (32, K // 128) and layer.Bc.shape == (N, 32) and layer.Bs.shape == (N,)
    assert not layer.Ac[20:].any() and not layer.Bc[:, 20:].any()
    wc, ws = intq.group_quantize(W, 4, axis=0)
    assert np.array_equal(mxint.unpack_int4(layer.Wc), wc.T) and np.array_equal(layer.Ws, ws.T)
    W_hat, A_hat, B_hat = intq.dequantize_layer(layer)
    assert np.array_equal(W_hat, intq.group_dequantize(wc, ws, axis=0))
    # the quantized factors come within a few percent of the Eckart-Young optimum of S E_q (Eq. 4-5) in the weighted norm
    s = factors.calibrate_scale(calib)
    E = W.astype(np.float64) - W_hat
    sig = np.linalg.svd(s[:, None] * E, compute_uv=False)
    best = np.sqrt((sig[20:] ** 2).sum())
    got = np.linalg.norm(s[:, None] * (E - A_hat @ B_hat))
    assert best <= got * (1 + 1e-12) and got <= 1.02 * best
    # rank zero: empty factors, the forward pass is the plain quantized product
    l0 = intq.build_factors_int(W, calib, 0)
    assert l0.kp == 0 and l0.Ac.shape == (0, K)
    xc, xs = intq.quantize_tokens(X)
    assert np.allclose(intq.forward(X, l0), (xc * xs.astype(np.float64)[:, None]) @ W_hat, rtol=1e-13)


def test_forward_by_exact_rationals_and_identities():
    W, calib, X, layer = _layer(seed=2, K=128, N=5, k=3)
    Y = intq.forward(X, layer)
    xc, xs = intq.quantize_tokens(X)
    Wc = mxint.unpack_int4(layer.Wc)
    F = lambda a: Fraction(float(a))
    for t in range(X.shape[0]):
        xh = [int(xc[t, i]) * F(xs[t]) for i in range(layer.K)]
        T = [sum(xh[i] * int(layer.Ac[r, i]) * F(layer.As[r, i // 128]) for i in range(layer.K)) for r in range(layer.kp)]
        for j in range(layer.N):
            y = sum(xh[i] * int(Wc[j, i]) * F(layer.Ws[j, i // 128]) for i in range(layer.K))
            y += sum(T[r] * int(layer.Bc[j, r]) * F(layer.Bs[j]) for r in range(layer.kp))
            assert abs(float(y) - Y[t, j]) <= 1e-13 * max(1.0, abs(float(y)))
    # Eq. 3: one product with the fused weight; column subsets select; magnitudes dominate
    W_hat, A_hat, B_hat = intq.dequantize_layer(layer)
    X_hat = xc * xs.astype(np.float64)[:, None]
    assert np.allclose(Y, X_hat @ (W_hat + A_hat @ B_hat), rtol=1e-12, atol=1e-15)
    cols = np.array([4, 0, 2])
    assert np.allclose(intq.forward(X, layer, cols), Y[:, cols], rtol=1e-13)
    main, tail, proj = intq.forward_magnitudes(X, layer)
    assert np.all(main + tail >= np.abs(Y) * (1 - 1e-12)) and np.all(proj >= tail * (1 - 1e-12))
    m2, t2, p2 = intq.forward_magnitudes(X, layer, cols)
    assert np.array_equal(m2, main[:, cols]) and np.array_equal(t2, tail[:, cols])


def test_ordering_of_table1_holds_for_the_int_formats():
    # qualitative, as for MXINT: output error of plain INT4 g128 >= LQER-INT >= L2QER-INT on outlier-heavy inputs
    rng = np.random.default_rng(4)
    K, N = 512, 256
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, 8)
    calib = np.stack([synth.gen_activations(rng, 128, K, ch, 30.0)])
    X = synth.gen_activations(rng, 16, K, ch, 30.0)
    ref = X.astype(np.float64) @ W.astype(np.float64)
    errs = [np.linalg.norm(intq.forward(X, intq.build_factors_int(W, calib, k, mode)) - ref)
            for k, mode in ((0, 1), (16, 0), (16, 1))]
    assert errs[0] >= errs[1] >= errs[2] and errs[2] < 0.95 * errs[0]
