"""Pins for the oracle's inference pass (Eq. 3, Eq. 6; Sec. 2.2 for the
integer form): the fused-weight identity, an exact rational brute force, the
integer-exact form, degenerate cases and the qualitative ordering of Table 1."""
from fractions import Fraction

import numpy as np

from oracle import factors, forward, mxint
from paper_2402_02446_amd import synth


def _layer(seed=0, K=64, N=48, k=8, mode=1):
    rng = np.random.default_rng(seed)
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, 4)
    calib = np.stack([synth.gen_activations(rng, 32, K, ch, 30.0)])
    X = synth.gen_activations(rng, 5, K, ch, 30.0)
    return W, calib, X, factors.build_factors(W, calib, k, mode)


def test_equals_single_matmul_with_fused_weight():
    # Eq. 3: X W_q + (X A_k) B_k = X (W_q + A_k B_k)
    _, _, X, layer = _layer()
    W_hat, A_hat, B_hat = factors.dequantize_layer(layer)
    Xc, Xe = forward.quantize_activations(X)
    X_hat = mxint.mx_dequantize(Xc, Xe, 8)
    Y = forward.forward(X, layer)
    assert np.allclose(Y, X_hat @ (W_hat + A_hat @ B_hat), rtol=1e-12, atol=1e-15)


def test_rational_brute_force_tiny():
    # 2 x 32 x 3 with kp = 16, every product and sum in exact rationals from the bytes.
    rng = np.random.default_rng(2)
    K, N, M = 32, 3, 2
    W = synth.gen_weight(rng, K, N)
    calib = rng.standard_normal((1, 8, K)).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[:, 5] *= 40
    layer = factors.build_factors(W, calib, k=2, mode=1)
    Xc, Xe = forward.quantize_activations(X)
    Wc = mxint.unpack_int4(layer.Wc)
    two = Fraction(2)

    def xh(t, i):
        return int(Xc[t, i]) * two ** (int(Xe[t, i // 16]) - 127 - 6)

    def wh(i, j):
        return int(Wc[j, i]) * two ** (int(layer.We[j, i // 16]) - 127 - 2)

    def ah(i, r):
        return int(layer.Ac[r, i]) * two ** (int(layer.Ae[r, i // 16]) - 127 - 6)

    def bh(r, j):
        return int(layer.Bc[j, r]) * two ** (int(layer.Be[j, r // 16]) - 127 - 6)

    Y = forward.forward(X, layer)
    for t in range(M):
        T = [sum(xh(t, i) * ah(i, r) for i in range(K)) for r in range(layer.kp)]
        for j in range(N):
            y = sum(xh(t, i) * wh(i, j) for i in range(K)) + sum(T[r] * bh(r, j) for r in range(layer.kp))
            assert abs(float(y) - Y[t, j]) <= 1e-13 * max(1.0, abs(float(y)))


def test_integer_form_agrees():
    _, _, X, layer = _layer(seed=4, K=128, N=32, k=16)
    Xc, Xe = forward.quantize_activations(X)
    Y = forward.forward_q(Xc, Xe, layer)
    Yi = forward.forward_int_exact(Xc, Xe, layer)
    assert np.allclose(Y, Yi, rtol=1e-13, atol=1e-18)


def test_uniform_exponent_case_is_exact_in_any_order():
    # One exponent everywhere, K <= 512, no correction: every partial sum is an
    # integer multiple of one power of two below 2^24, so fp32 summation in any
    # order gives the same bits as the fp64 oracle.
    rng = np.random.default_rng(6)
    K, N, M = 256, 32, 4
    Wc = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    layer = factors.PackedLayer(K=K, N=N, k=0, kp=0, Wc=mxint.pack_int4(Wc),
                                We=np.full((N, K // 16), 125, np.uint8),
                                Ac=np.zeros((0, K), np.int8), Ae=np.zeros((0, K // 16), np.uint8),
                                Bc=np.zeros((N, 0), np.int8), Be=np.zeros((N, 0), np.uint8))
    Xc = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    Xe = np.full((M, K // 16), 129, np.uint8)
    Y = forward.forward_q(Xc, Xe, layer)
    Yi = forward.forward_int_exact(Xc, Xe, layer)
    assert np.array_equal(Y, Yi)
    ints = Xc.astype(np.int64) @ Wc.astype(np.int64).T
    assert np.abs(ints).max() < 2 ** 24
    assert np.array_equal(Y, ints * 2.0 ** ((129 - 127 - 6) + (125 - 127 - 2)))
    assert np.array_equal(Y.astype(np.float32).astype(np.float64), Y)


def test_rank_zero_and_single_token():
    W, calib, X, _ = _layer(seed=7)
    l0 = factors.build_factors(W, calib, 0)
    W_hat, _, _ = factors.dequantize_layer(l0)
    Xc, Xe = forward.quantize_activations(X)
    X_hat = mxint.mx_dequantize(Xc, Xe, 8)
    assert np.allclose(forward.forward(X, l0), X_hat @ W_hat, rtol=1e-13)
    # M = 1 is a matrix-vector product; rows are independent
    _, _, _, layer = _layer(seed=7)
    Yall = forward.forward(X, layer)
    assert np.array_equal(forward.forward(X[2:3], layer), Yall[2:3])


def test_table1_ordering_on_outlier_heavy_inputs():
    # Table 1's ablation, qualitatively: output error of plain MXINT >= LQER >= L2QER
    wl = synth.WORKLOADS["cfg1"]
    d = synth.draw(wl)
    X = d.X[16]
    ref = X.astype(np.float64) @ d.W.astype(np.float64)
    errs = []
    for k, mode in ((0, 1), (wl.k, 0), (wl.k, 1)):
        layer = factors.build_factors(d.W, d.calib, k, mode)
        errs.append(np.linalg.norm(forward.forward(X, layer) - ref))
    assert errs[0] >= errs[1] >= errs[2]
    assert errs[2] < 0.9 * errs[0]


def test_column_subset_form_equals_the_full_one():
    # forward_cols is the checker for layers too wide to dequantize whole: every column, a strict
    # subset in scrambled order with a repeat, and the 6-bit activation width, against forward()
    _, _, X, layer = _layer(seed=11, K=96, N=80, k=20)
    Y = forward.forward(X, layer)
    assert np.array_equal(forward.forward_cols(X, layer, np.arange(layer.N)), Y)
    cols = np.array([79, 0, 33, 32, 31, 5, 5, 64])
    sub = forward.forward_cols(X, layer, cols)
    assert sub.shape == (X.shape[0], len(cols))
    assert np.allclose(sub, Y[:, cols], rtol=1e-13, atol=1e-18)
    assert np.allclose(forward.forward_cols(X, layer, cols, act_bits=6), forward.forward(X, layer, act_bits=6)[:, cols],
                       rtol=1e-13, atol=1e-18)
    # and against exact rationals on two elements, straight from the bytes
    Xc, Xe = forward.quantize_activations(X)
    Wc = mxint.unpack_int4(layer.Wc)
    two = Fraction(2)
    for (t, jj) in ((0, 0), (4, 3)):
        j = int(cols[jj])
        xh = [int(Xc[t, i]) * two ** (int(Xe[t, i // 16]) - 133) for i in range(layer.K)]
        T = [sum(xh[i] * int(layer.Ac[r, i]) * two ** (int(layer.Ae[r, i // 16]) - 133) for i in range(layer.K))
             for r in range(layer.kp)]
        y = sum(xh[i] * int(Wc[j, i]) * two ** (int(layer.We[j, i // 16]) - 129) for i in range(layer.K))
        y += sum(T[r] * int(layer.Bc[j, r]) * two ** (int(layer.Be[j, r // 16]) - 133) for r in range(layer.kp))
        assert abs(float(y) - sub[t, jj]) <= 1e-13 * max(1.0, abs(float(y)))


def test_magnitude_sums():
    # forward_magnitudes feeds the elementwise rounding bound of the GPU tests.  Pins: exact rationals on one
    # element; with every operand non-negative the sums are the result itself (main + tail = Y, proj = tail);
    # in general main + tail >= |Y| and proj >= tail (triangle inequality); column subsets select.
    _, _, X, layer = _layer(seed=12, K=64, N=24, k=16)
    main, tail, proj = forward.forward_magnitudes(X, layer)
    Y = forward.forward(X, layer)
    assert np.all(main + tail >= np.abs(Y) * (1 - 1e-12))
    assert np.all(proj >= tail * (1 - 1e-12))
    cols = np.array([3, 20, 7])
    m2, t2, p2 = forward.forward_magnitudes(X, layer, cols)
    assert np.array_equal(m2, main[:, cols]) and np.array_equal(t2, tail[:, cols]) and np.array_equal(p2, proj[:, cols])
    Xc, Xe = forward.quantize_activations(X)
    Wc = mxint.unpack_int4(layer.Wc)
    two = Fraction(2)
    t, j = 2, 7
    xh = [int(Xc[t, i]) * two ** (int(Xe[t, i // 16]) - 133) for i in range(layer.K)]
    ah = [[int(layer.Ac[r, i]) * two ** (int(layer.Ae[r, i // 16]) - 133) for i in range(layer.K)] for r in range(layer.kp)]
    bh = [int(layer.Bc[j, r]) * two ** (int(layer.Be[j, r // 16]) - 133) for r in range(layer.kp)]
    want_main = sum(abs(xh[i]) * abs(int(Wc[j, i])) * two ** (int(layer.We[j, i // 16]) - 129) for i in range(layer.K))
    want_tail = sum(abs(sum(xh[i] * ah[r][i] for i in range(layer.K))) * abs(bh[r]) for r in range(layer.kp))
    want_proj = sum(sum(abs(xh[i]) * abs(ah[r][i]) for i in range(layer.K)) * abs(bh[r]) for r in range(layer.kp))
    for got, want in ((main[t, j], want_main), (tail[t, j], want_tail), (proj[t, j], want_proj)):
        assert abs(float(want) - got) <= 1e-13 * float(want)
    # non-negative operands: the magnitudes are the values
    pos = factors.PackedLayer(K=layer.K, N=layer.N, k=layer.k, kp=layer.kp,
                              Wc=mxint.pack_int4(np.abs(Wc).astype(np.int8)), We=layer.We,
                              Ac=np.abs(layer.Ac), Ae=layer.Ae, Bc=np.abs(layer.Bc), Be=layer.Be)
    Xp = np.abs(X)
    main, tail, proj = forward.forward_magnitudes(Xp, pos)
    assert np.allclose(main + tail, forward.forward(Xp, pos), rtol=1e-13)
    assert np.allclose(proj, tail, rtol=1e-13)


def test_two_bit_weights_in_the_forward_pass():
    # w_bits = 2 through every form of the forward pass: dense, column subset, integer blocks, magnitudes;
    # and exact rationals straight from the bytes on one element
    rng = np.random.default_rng(13)
    K, N, M = 64, 40, 3
    W = synth.gen_weight(rng, K, N)
    calib = np.abs(rng.standard_normal((1, 8, K))).astype(np.float32) + 0.1
    X = rng.standard_normal((M, K)).astype(np.float32)
    layer = factors.build_factors(W, calib, 24, 1, w_bits=2)
    Y = forward.forward(X, layer)
    cols = np.array([39, 0, 7])
    assert np.allclose(forward.forward_cols(X, layer, cols), Y[:, cols], rtol=1e-13, atol=1e-18)
    Xc, Xe = forward.quantize_activations(X)
    assert np.allclose(forward.forward_int_exact(Xc, Xe, layer), Y, rtol=1e-13, atol=1e-18)
    main, tail, proj = forward.forward_magnitudes(X, layer)
    assert np.all(main + tail >= np.abs(Y) * (1 - 1e-12))
    Wc = mxint.unpack_int2(layer.Wc)
    two = Fraction(2)
    t, j = 1, 7
    xh = [int(Xc[t, i]) * two ** (int(Xe[t, i // 16]) - 133) for i in range(K)]
    T = [sum(xh[i] * int(layer.Ac[r, i]) * two ** (int(layer.Ae[r, i // 16]) - 133) for i in range(K)) for r in range(layer.kp)]
    y = sum(xh[i] * int(Wc[j, i]) * two ** (int(layer.We[j, i // 16]) - 127) for i in range(K))       # no fraction bits
    y += sum(T[r] * int(layer.Bc[j, r]) * two ** (int(layer.Be[j, r // 16]) - 133) for r in range(layer.kp))
    assert abs(float(y) - Y[t, j]) <= 1e-13 * max(1.0, abs(float(y)))
