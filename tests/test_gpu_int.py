"""GPU parity of the scaled-integer variant (Table 2 "L2QER-INT": INT4 g128 weights with FP16 scales, INT8 g128 factors,
INT8 per-token activations) against the fp64 oracle: the per-token quantizer bit for bit, canonical arrays round-trip,
the forward pass on ragged token and column counts and ranks from none to 128, the offline step, the static scratch,
the LLaMA-7B-shaped layers at full size, and the 4096 x 4096 layer at 65536 tokens."""
import numpy as np
import pytest

from oracle import factors, intq
from paper_2402_02446_amd import synth
from helpers import ELEM_C, ELEM_C0, U32, Y_TOL, Y_TOL_DERIVED, tile_cover_samples

pytestmark = pytest.mark.gpu


def _standin_layer(K, N, k, seed=0, n_outlier=None, gain=50.0):
    """W_q by the oracle quantizer; A_k, B_k from random stand-ins quantized by the oracle (no SVD at these sizes)."""
    rng = np.random.default_rng(seed)
    ch = synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)) if n_outlier is None else n_outlier)
    wc, ws = intq.group_quantize(synth.gen_weight(rng, K, N), 4, axis=0)
    kp = factors.padded_rank(k)
    A, B = synth.gen_factor_standins(rng, K, N, k, ch, gain)
    Ap = np.zeros((K, kp)); Ap[:, :k] = A
    Bp = np.zeros((kp, N)); Bp[:k] = B
    from oracle import mxint
    if kp:
        ac, as_ = intq.group_quantize(Ap, 8, axis=0)
        bc, bs = intq.group_quantize(Bp, 8, axis=0)
        fac = dict(Ac=np.ascontiguousarray(ac.T), As=np.ascontiguousarray(as_.T), Bc=np.ascontiguousarray(bc.T),
                   Bs=np.ascontiguousarray(bs.reshape(-1)))
    else:
        fac = dict(Ac=np.zeros((0, K), np.int8), As=np.zeros((0, K // 128), np.float16), Bc=np.zeros((N, 0), np.int8),
                   Bs=np.ones(N, np.float16))
    return intq.IntLayer(K=K, N=N, k=k, kp=kp, Wc=mxint.pack_int4(np.ascontiguousarray(wc.T)), Ws=np.ascontiguousarray(ws.T), **fac), ch


def _upload(layer):
    from paper_2402_02446_amd import binding
    return binding.lqer_int_layer_import(layer.K, layer.N, layer.k, layer.Wc, layer.Ws, layer.Ac, layer.As, layer.Bc, layer.Bs)


def _check(Y, X, layer, cols=None):
    """Norm and elementwise bars as for the MXINT layer: exact integer group sums, fp32 scaling and accumulation
    over K / 128 groups, T in fp32 split into two truncated bf16 terms."""
    Y = np.asarray(Y, np.float64)
    Yref = intq.forward(X, layer, cols)
    assert Y.shape == Yref.shape and np.all(np.isfinite(Y))
    den = np.linalg.norm(Yref)
    err = float(np.linalg.norm(Y - Yref) / den) if den > 0 else float(np.linalg.norm(Y))
    assert err <= Y_TOL and err <= Y_TOL_DERIVED, err
    main, tail, proj = intq.forward_magnitudes(X, layer, cols)
    n = layer.K // 128 + 2 * layer.kp
    bound = ((ELEM_C * np.sqrt(n) + ELEM_C0) * U32 * (main + tail) + 2.0 ** -14 * tail
             + (ELEM_C * np.sqrt(layer.K // 128) + ELEM_C0) * U32 * proj)
    diff = np.abs(Y - Yref)
    ratio = float((diff / np.maximum(bound, np.finfo(np.float64).tiny)).max())
    assert not (diff > bound).any(), f"largest |error| / bound = {ratio:.3g} at {np.argwhere(diff > bound)[0].tolist()}"
    return err, ratio


def test_token_quantizer_bit_for_bit():
    import torch
    from paper_2402_02446_amd import binding
    rng = np.random.default_rng(1)
    for rows, cols in ((1, 128), (37, 1000), (300, 4096), (5, 11008)):
        ch = synth.gen_outlier_channels(rng, cols, max(1, cols // 100))
        X = synth.gen_activations(rng, rows, cols, ch, 50.0)
        X[rows // 2] *= np.float32(1e-3)
        if rows > 2:
            X[1] = 0.0                                          # an all-zero token: scale 1, codes 0
        # exact ties in code units on one row: x = (n + 0.5) * s with s a power of two
        X[0, :64] = (np.arange(64, dtype=np.float32) - 32.5) * np.float32(0.25)
        X[0, 64] = np.float32(127 * 0.25)
        X[0, 65:] = np.clip(X[0, 65:], -30, 30)
        codes, scales = binding.lqer_quantize_int8_token(torch.from_numpy(X).cuda())
        torch.cuda.synchronize()
        oc, osc = intq.quantize_tokens(X)
        assert np.array_equal(scales.cpu().numpy().view(np.uint16), osc.view(np.uint16))
        assert np.array_equal(codes.cpu().numpy(), oc)
    # strided rows
    xb = torch.full((9, 600), 7.0e30, dtype=torch.float32, device="cuda")
    X = synth.gen_activations(rng, 9, 512, np.array([3]), 30.0)
    xb[:, :512] = torch.from_numpy(X).cuda()
    codes, scales = binding.lqer_quantize_int8_token(xb[:, :512])
    oc, osc = intq.quantize_tokens(X)
    assert np.array_equal(codes.cpu().numpy(), oc) and np.array_equal(scales.cpu().numpy().view(np.uint16), osc.view(np.uint16))


@pytest.mark.parametrize("K,N,k", [(128, 40, 0), (256, 100, 8), (1024, 272, 64), (2304, 528, 33), (512, 1100, 128), (4096, 64, 16)])
@pytest.mark.parametrize("M", [1, 5, 16, 100, 128, 129, 300])
def test_forward_shapes(K, N, k, M):
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = _standin_layer(K, N, k, seed=K + k, n_outlier=4)
    h = _upload(layer)
    assert binding.lqer_linear_path(h, M) == 3
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
    ld = (N + 3) // 4 * 4
    buf = torch.full((M, ld), float("nan"), dtype=torch.float32, device="cuda")
    binding.lqer_linear_forward(h, torch.from_numpy(X).cuda(), Y=buf[:, :N])
    torch.cuda.synchronize()
    assert torch.isnan(buf[:, N:]).all()                       # nothing is written behind a row
    _check(buf[:, :N].cpu().numpy(), X, layer)
    h.free()


def test_round_trip_errors_and_other_entry_points():
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = _standin_layer(256, 100, 20, seed=3, n_outlier=4)
    h = _upload(layer)
    ex = binding.lqer_int_layer_export(h)
    for name in ("Wc", "Ac", "Bc"):
        assert np.array_equal(ex[name], getattr(layer, name)), name
    for name in ("Ws", "As", "Bs"):
        assert np.array_equal(ex[name].view(np.uint16), getattr(layer, name).view(np.uint16)), name
    X = torch.from_numpy(synth.gen_activations(np.random.default_rng(0), 7, 256, ch, 30.0)).cuda()
    want = binding.lqer_linear_forward(h, X).clone()
    # same bits on every run, and from the static scratch
    for _ in range(3):
        assert torch.equal(binding.lqer_linear_forward(h, X), want)
    assert torch.equal(binding.lqer_linear_forward_static(h, X), want)
    # the entry points of the MXINT formats refuse the layer
    for call in (lambda: binding.lqer_linear_forward_ex(h, X, path=2), lambda: binding.lqer_linear_forward_requant(h, X),
                 lambda: binding.lqer_layer_export(h), lambda: h.set_activation_bits(6),
                 lambda: binding.lqer_linear_forward_q(h, torch.zeros((7, 256), dtype=torch.int8, device="cuda"),
                                                       torch.zeros((7, 16), dtype=torch.uint8, device="cuda"))):
        with pytest.raises(binding.LqerError) as e:
            call()
        assert e.value.status == 3
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_linear_forward(h, X, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 5
    with pytest.raises(binding.LqerError) as e:           # beyond the static scratch (32 MiB): refused, nothing launched
        binding.lqer_linear_forward_static(h, torch.zeros((140000, 256), dtype=torch.float32, device="cuda"))
    assert e.value.status == 5
    assert binding.lqer_linear_forward(h, X[:0]).shape == (0, 100)
    h.free()
    # excluded values and shapes
    bad = layer.Wc.copy(); bad[0, 0] = 0x08
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_int_layer_import(256, 100, 0, bad, layer.Ws)
    assert e.value.status == 8
    zs = layer.Ws.copy(); zs[0, 0] = 0
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_int_layer_import(256, 100, 0, layer.Wc, zs)
    assert e.value.status == 8
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_int_layer_import(192, 100, 0, layer.Wc, layer.Ws)       # K % 128
    assert e.value.status == 2


@pytest.mark.parametrize("K,N,k,mode", [(256, 192, 20, 1), (512, 384, 64, 1), (384, 200, 8, 0)])
def test_offline_step(K, N, k, mode):
    # lqer_build_factors with {4, 8, 16, 128}: W_q and its FP16 scales bit for bit the oracle's; the weighted residual of
    # the quantized factors where the oracle's is; forward pass of the built layer against the oracle on its own arrays
    import torch
    from paper_2402_02446_amd import binding
    rng = np.random.default_rng(K + k)
    W = synth.gen_weight(rng, K, N)
    ch = synth.gen_outlier_channels(rng, K, 4)
    calib = np.stack([synth.gen_activations(rng, 32, K, ch, 30.0) for _ in range(2)])
    want = intq.build_factors_int(W, calib, k, mode)
    h = binding.lqer_build_factors(W, calib if mode else None, k, mode, cfg=(4, 8, 16, 128))
    ex = binding.lqer_int_layer_export(h)
    assert np.array_equal(ex["Wc"], want.Wc) and np.array_equal(ex["Ws"].view(np.uint16), want.Ws.view(np.uint16))
    got = intq.IntLayer(K=K, N=N, k=k, kp=h.kp, **ex)
    s = factors.calibrate_scale(calib) if mode else np.ones(K)
    W_hat, A_o, B_o = intq.dequantize_layer(want)
    _, A_g, B_g = intq.dequantize_layer(got)
    E = W.astype(np.float64) - W_hat
    total = np.linalg.norm(s[:, None] * E)
    r_o = np.linalg.norm(s[:, None] * (E - A_o @ B_o))
    r_g = np.linalg.norm(s[:, None] * (E - A_g @ B_g))
    assert abs(r_g - r_o) <= 0.01 * total, (r_g, r_o, total)
    X = synth.gen_activations(rng, 40, K, ch, 30.0)
    _check(binding.lqer_linear_forward(h, torch.from_numpy(X).cuda()).cpu().numpy(), X, got)
    h.free()


@pytest.mark.parametrize("K,N,k,M", [(1024, 272, 64, 5), (2304, 528, 33, 100), (4096, 640, 128, 16), (4096, 1100, 0, 129)])
def test_few_tokens_split_over_k_same_bits_every_run(K, N, k, M):
    # with few output tiles the projection and the main product split K over planes of workgroups that a small kernel adds
    # in plane order: the result has the same bits on every run, also through the static-scratch entry
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = _standin_layer(K, N, k, seed=3 * K + N)
    h = _upload(layer)
    X = torch.from_numpy(synth.gen_activations(np.random.default_rng(K + M), M, K, ch, 40.0)).cuda()
    Y0 = binding.lqer_linear_forward(h, X)
    _check(Y0.cpu().numpy(), X.cpu().numpy(), layer)
    for _ in range(3):
        assert torch.equal(binding.lqer_linear_forward(h, X), Y0)
    Ys = torch.full_like(Y0, float("nan"))
    binding.lqer_linear_forward_static(h, X, Y=Ys)
    assert torch.equal(Ys, Y0)
    h.free()


@pytest.mark.parametrize("K,N,k,M", [(4096, 4096, 32, 16), (4096, 11008, 32, 16), (11008, 4096, 32, 16),
                                     (4096, 11008, 32, 2048), (11008, 4096, 32, 2048)])
def test_7b_shaped_layers_every_tile(K, N, k, M):
    # the LLaMA-7B-shaped layers with Table 2's k = 32, decode and prefill: every token row (M = 16) or one of every band
    # of 32 against one column of every group of 32 - every output tile, wavefront part and MFMA tile is touched
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = _standin_layer(K, N, k, seed=K + N)
    h = _upload(layer)
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 50.0)
    Y = binding.lqer_linear_forward(h, torch.from_numpy(X).cuda())
    assert bool(torch.isfinite(Y).all())
    rows, cols = tile_cover_samples(np.random.default_rng(2), M, N)
    if M <= 16:
        rows = np.arange(M)
    Ys = Y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    err, ratio = _check(Ys, X[rows], layer, cols)
    print(f"{K}x{N} M={M}: rel. Frobenius error {err:.3g}, largest |error| / bound {ratio:.3g}")
    h.free()


def test_int_layer_at_65536_tokens_every_tile():
    # the 4096 x 4096 layer at the decoder block's 65536 tokens, the configuration the benchmark times for this variant:
    # one row of every band of 32 token rows against one column of every group of 32 columns (every output tile, every
    # wavefront's part of it and every MFMA tile holds a compared element), norm and elementwise; the per-token
    # quantizer's codes and scales on the same rows, bit for bit; everything else finite.
    import torch
    from paper_2402_02446_amd import binding
    K = N = 4096
    k, M = 32, 65536
    layer, ch = _standin_layer(K, N, k, seed=5)
    h = _upload(layer)
    rng = np.random.default_rng(9)
    X = torch.empty((M, K), dtype=torch.float32, device="cuda")
    rows, cols = tile_cover_samples(rng, M, N)
    rows = np.unique(np.r_[rows, 127, 128, 255, 256, 32767, 32768, M - 129, M - 128])
    keep = {}
    for r0 in range(0, M, 8192):                             # generated in slabs: the host never holds all of X
        slab = synth.gen_activations(np.random.default_rng(r0 + 3), 8192, K, ch, 50.0)
        X[r0:r0 + 8192] = torch.from_numpy(slab).cuda()
        for r in rows[(rows >= r0) & (rows < r0 + 8192)]:
            keep[int(r)] = slab[r - r0].copy()
    Xs = np.stack([keep[int(r)] for r in rows])
    Y = binding.lqer_linear_forward(h, X)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    Ys = Y[idx][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert bool(torch.isfinite(Y).all())
    err, ratio = _check(Ys, Xs, layer, cols)
    print(f"INT {K}x{N} at {M} tokens: {len(rows)} x {len(cols)} samples, rel. Frobenius error {err:.3g}, largest |error| / bound {ratio:.3g}")
    del Y
    codes, scales = binding.lqer_quantize_int8_token(X)
    torch.cuda.synchronize()
    oc, os_ = intq.quantize_tokens(Xs)
    assert np.array_equal(codes[idx].cpu().numpy(), oc)
    assert np.array_equal(scales[idx].cpu().numpy().view(np.uint16), os_.view(np.uint16))
    h.free()
