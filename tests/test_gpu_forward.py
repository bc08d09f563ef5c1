"""GPU parity of lqer_linear_forward against the fp64 oracle (Eq. 3, Eq. 6): relative Frobenius
error of Y within the stated 1e-3 bar (and within what fp32 accumulation of exact products
should give), bitwise equality where the arithmetic is exact in any order, both kernels, every
tile shape, ragged sizes, and the full LLaMA-shaped workloads on sampled rows."""
import numpy as np
import pytest

from oracle import factors, forward, mxint
from paper_2402_02446_amd import synth
from helpers import Y_TOL, assert_forward_matches, oracle_layer_big, oracle_layer_small, tile_cover_samples, upload

pytestmark = pytest.mark.gpu


def _gpu_forward(h, X, **kw):
    import torch
    from paper_2402_02446_amd import binding
    Xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
    Y = binding.lqer_linear_forward_ex(h, Xd, **kw) if kw else binding.lqer_linear_forward(h, Xd)
    torch.cuda.synchronize()
    return Y.cpu().numpy()



def test_cfg1_exact_factors():
    wl = synth.WORKLOADS["cfg1"]
    d = synth.draw(wl)
    layer = factors.build_factors(d.W, d.calib, wl.k, 1)
    h = upload(layer)
    X = d.X[16]
    assert_forward_matches(_gpu_forward(h, X), X, layer)
    h.free()


@pytest.mark.parametrize("M", [1, 2, 4, 5, 15, 16, 17, 32])
def test_streaming_kernel_row_counts(M):
    layer, ch = oracle_layer_small(512, 256, 24, seed=M)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(M), M, 512, ch, 30.0)
    assert_forward_matches(_gpu_forward(h, X, path=1), X, layer)
    h.free()


STREAM_VARIANTS = [11441, 11421, 12241, 12242, 12181, 12141, 11181, 11101, 11281, 11241,
                   21181, 21141, 22181, 21101, 22421, 21441]


@pytest.mark.parametrize("K,N,k", [(48, 40, 0), (272, 100, 8), (1024, 272, 64), (2304, 528, 33), (4096, 64, 16)])
@pytest.mark.parametrize("M", [3, 5, 20, 40, 64])
@pytest.mark.parametrize("variant", STREAM_VARIANTS)
def test_streaming_kernel_shapes(K, N, k, M, variant):
    # variant = 10000 KSP + 1000 G + 100 NWC + 10 (NWK % 16) + DT; a shape whose activation stages do
    # not fit the 160 KB of LDS must be refused, every other one must match the oracle
    from paper_2402_02446_amd import binding
    nwk = (variant // 10) % 10 or 16
    rows = 4 if M <= 4 else (16 if M <= 16 else (32 if M <= 32 else 64))
    mb = rows // 32 or 1                                     # token blocks of 32 per wavefront
    kt = (K + 255) // 256
    ksp = variant // 10000
    stages = 1 if (variant % 10 == 1 and kt <= nwk * ksp) else 2
    g, nwc = (variant // 1000) % 10, (variant // 100) % 10
    lds = 9216 * mb + max(stages * nwk * rows * 512,
                          nwk * nwc * g * mb * 4096 + (nwc * g * 4096 if ksp == 2 else 0))
    if mb == 2 and ksp == 2:
        lds = 1 << 20                                        # pairs of workgroups take at most 32 tokens
    layer, ch = oracle_layer_small(K, N, k, seed=K + k)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(1), M, K, ch, 30.0)
    if lds > 160 * 1024:
        with pytest.raises(binding.LqerError):
            _gpu_forward(h, X, path=1, variant=variant)
    else:
        assert_forward_matches(_gpu_forward(h, X, path=1, variant=variant), X, layer)
    h.free()


# variant = 100 * mode + tile shape; mode 2 cuts output tiles along K between workgroups wherever the
# tiles do not fill whole rounds of the chip (along tile boundaries where the chip holds two or more workgroups
# per remaining tile, otherwise in equal shares of the remaining K tiles), mode 3 always in equal shares,
# mode 1 never cuts, mode 0 decides by estimate
@pytest.mark.parametrize("variant", [1, 3, 4, 7, 8, 11, 12, 13, 101, 111, 112, 204, 211, 212, 304, 311, 312])
@pytest.mark.parametrize("M,K,N,k", [(16, 512, 512, 8), (300, 272, 200, 0), (513, 1024, 528, 64), (100, 2304, 40, 33),
                                     (700, 4352, 1100, 16)])
def test_tiled_kernel_shapes(variant, M, K, N, k):
    layer, ch = oracle_layer_small(K, N, k, seed=M + variant)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(2), M, K, ch, 30.0)
    assert_forward_matches(_gpu_forward(h, X, path=2, variant=variant), X, layer)
    h.free()


@pytest.mark.parametrize("path", [1, 2])
def test_uniform_exponent_case_is_bitwise_exact(path):
    # Every partial sum is an integer multiple of one power of two below 2^24: any fp32 order is exact.
    rng = np.random.default_rng(6)
    K, N, M = 512, 96, 16
    Wc = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    layer = factors.PackedLayer(K=K, N=N, k=0, kp=0, Wc=mxint.pack_int4(Wc),
                                We=np.full((N, K // 16), 125, np.uint8),
                                Ac=np.zeros((0, K), np.int8), Ae=np.zeros((0, K // 16), np.uint8),
                                Bc=np.zeros((N, 0), np.int8), Be=np.zeros((N, 0), np.uint8))
    codes = rng.integers(-100, 101, size=(M, K)).astype(np.float64)
    codes[:, ::16] = 127.0                                   # pins every block's exponent to 0
    X = (codes / 64.0).astype(np.float32)
    Yref = forward.forward(X, layer)
    assert np.abs(Yref * 2 ** 10).max() < 2 ** 24
    Y = _gpu_forward(upload(layer), X, path=path)
    assert np.array_equal(Y.astype(np.float64), Yref)


def test_wide_exponent_spread():
    # block exponents spread over 2^+-40 on both operands; still exact products, fp32 accumulation
    rng = np.random.default_rng(8)
    K, N, M = 512, 64, 16
    W = (rng.standard_normal((K, N)) * np.exp2(rng.integers(-40, 40, (K // 16, 1, N)).repeat(16, 0).reshape(K, N))).astype(np.float32)
    X = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-40, 40, (M, K // 16)).repeat(16, 1))).astype(np.float32)
    calib = np.abs(rng.standard_normal((1, 16, K))).astype(np.float32) + 0.1
    layer = factors.build_factors(W, calib, 16, 1)
    h = upload(layer)
    for path in (1, 2):
        assert_forward_matches(_gpu_forward(h, X, path=path), X, layer)
    h.free()


def test_prequantized_entry_point_and_stage_split():
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(1024, 272, 32, seed=9)
    h = upload(layer)
    for M in (7, 200):
        X = synth.gen_activations(np.random.default_rng(M), M, 1024, ch, 30.0)
        Xd = torch.from_numpy(X).cuda()
        Y = binding.lqer_linear_forward(h, Xd)
        Xc, Xe = binding.lqer_quantize_mx(Xd, 8)
        Yq = binding.lqer_linear_forward_q(h, Xc, Xe)
        Y1 = torch.zeros_like(Y)
        binding.lqer_linear_forward_ex(h, Xd, Y=Y1, stages=1)
        binding.lqer_linear_forward_ex(h, Xd, Y=Y1, stages=2)
        torch.cuda.synchronize()
        assert torch.equal(Y, Yq) and torch.equal(Y, Y1)
        assert_forward_matches(Y.cpu().numpy(), X, layer)
    h.free()


def test_strided_x_and_y():
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(512, 100, 8, seed=4)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(3), 9, 512, ch, 30.0)
    xb = torch.full((9, 600), 7.0e30, dtype=torch.float32, device="cuda")
    xb[:, :512] = torch.from_numpy(X).cuda()
    yb = torch.full((9, 128), -5.0, dtype=torch.float32, device="cuda")
    binding.lqer_linear_forward(h, xb[:, :512], Y=yb[:, :100])
    torch.cuda.synchronize()
    out = yb.cpu().numpy()
    assert np.all(out[:, 100:] == -5.0)                    # nothing written outside Y
    assert_forward_matches(out[:, :100], X, layer)
    h.free()


def test_argument_errors_on_device():
    import torch
    from paper_2402_02446_amd import binding
    layer, _ = oracle_layer_small(64, 32, 8)
    h = upload(layer)
    X = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_linear_forward(h, X, workspace=small)
    assert e.value.status == 5
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_linear_forward_ex(h, torch.zeros((100, 64), device="cuda"), path=1)   # too many rows
    assert e.value.status == 2
    Y = binding.lqer_linear_forward(h, X[:0])
    assert Y.shape == (0, 32)
    h.free()


# ---- the LLaMA-shaped workloads at full size, in the launch configuration the benchmark times ----

def test_cfg2_decode_full():
    wl = synth.WORKLOADS["cfg2"]
    layer, ch = oracle_layer_big(wl.K, wl.N, wl.k, seed=0, n_outlier=wl.n_outlier, gain=wl.gain)
    h = upload(layer)
    for M in wl.Ms:
        X = synth.gen_activations(np.random.default_rng(M), M, wl.K, ch, wl.gain)
        assert_forward_matches(_gpu_forward(h, X), X, layer)
    h.free()


@pytest.mark.parametrize("name", ["cfg3_up", "cfg3_down"])
def test_cfg3_prefill_whole_output(name):
    # the 7B-shaped MLP layers at M = 2048 in the launch configuration the benchmark times (automatic path
    # and shape, tiles cut along K): the whole 2048 x N output against the oracle, norm and every element
    wl = synth.WORKLOADS[name]
    layer, ch = oracle_layer_big(wl.K, wl.N, wl.k, seed=1, n_outlier=wl.n_outlier, gain=wl.gain)
    h = upload(layer)
    M = wl.Ms[0]
    X = synth.gen_activations(np.random.default_rng(11), M, wl.K, ch, wl.gain)
    Y = _gpu_forward(h, X)
    err, ratio = assert_forward_matches(Y, X, layer)
    print(f"{name}: rel. Frobenius error {err:.3g}, largest |error| / elementwise bound {ratio:.3g}")
    h.free()


@pytest.mark.parametrize("K,N,k", [(4096, 4096, 32), (4096, 11008, 64), (11008, 4096, 16)])
def test_cfg5_block_shapes_at_65536_tokens_every_tile(K, N, k):
    # the decoder-block workload (batch 32 x sequence 2048 = 65536 tokens) at its full size, in the launch
    # configuration the benchmark times.  Compared with the oracle: one row of every band of 32 token rows
    # against one column of every group of 32 columns (so every output tile, every wavefront's part of it and
    # every MFMA tile holds a compared element), norm and elementwise; the stand-alone quantizer's codes and
    # exponent bytes on the same rows, bit for bit; everything else finite.
    import torch
    from paper_2402_02446_amd import binding
    M = 65536
    d = synth.random_packed_layer(np.random.default_rng(K + k), K, N, k)
    layer = factors.PackedLayer(**d)
    h = upload(layer)
    rng = np.random.default_rng(7)
    ch = synth.gen_outlier_channels(rng, K, round(0.01 * K))
    X = torch.empty((M, K), dtype=torch.float32, device="cuda")
    rows, cols = tile_cover_samples(rng, M, N)
    rows = np.unique(np.r_[rows, 127, 128, 255, 256, 32767, 32768, M - 129, M - 128])
    keep = {}
    for r0 in range(0, M, 8192):                             # generated in slabs: the host never holds all of X
        slab = synth.gen_activations(np.random.default_rng(r0 + 1), 8192, K, ch, 50.0)
        X[r0:r0 + 8192] = torch.from_numpy(slab).cuda()
        for r in rows[(rows >= r0) & (rows < r0 + 8192)]:
            keep[int(r)] = slab[r - r0].copy()
    Xs = np.stack([keep[int(r)] for r in rows])
    Y = binding.lqer_linear_forward(h, X)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).cuda()
    Ys = Y[idx][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert bool(torch.isfinite(Y).all())
    err, ratio = assert_forward_matches(Ys, Xs, layer, cols)
    print(f"{K}x{N}: {len(rows)} x {len(cols)} samples, rel. Frobenius error {err:.3g}, largest |error| / bound {ratio:.3g}")
    del Y
    codes, exps = binding.lqer_quantize_mx(X, 8)
    torch.cuda.synchronize()
    oc, oe = mxint.mx_quantize(Xs, 8, axis=-1)
    assert np.array_equal(codes[idx].cpu().numpy(), oc) and np.array_equal(exps[idx].cpu().numpy(), oe)
    h.free()


@pytest.mark.parametrize("M,K,N,k", [(3, 1024, 272, 32), (16, 4096, 64, 16), (20, 2304, 528, 33), (64, 512, 16384, 8),
                                     (300, 1024, 528, 64)])
def test_six_bit_activations(M, K, N, k):
    # the W4A6 setup (Table 2): X is quantized to MXINT6 (8-bit shared exponent, Sec. 4.1); every kind of
    # activation staging is covered - bf16 cells (M = 3), MXINT cells (16, 20, 64) and the tiled kernel's rows
    import torch
    from paper_2402_02446_amd import binding
    if N > 4096:
        d = synth.random_packed_layer(np.random.default_rng(N), K, N, k)
        layer = factors.PackedLayer(**d)
        ch = synth.gen_outlier_channels(np.random.default_rng(1), K, 4)
    else:
        layer, ch = oracle_layer_small(K, N, k, seed=M + k)
    h = upload(layer)
    h.set_activation_bits(6)
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
    want = forward.forward(X, layer, act_bits=6)
    Xd = torch.from_numpy(X).cuda()
    Y = binding.lqer_linear_forward(h, Xd)
    assert_forward_matches(Y.cpu().numpy(), X, layer, act_bits=6)
    # far from the 8-bit result: the width really is in effect
    assert forward.rel_frobenius(Y.cpu().numpy(), forward.forward(X, layer)) > 1e-3
    # already-quantized 6-bit codes give the same bits
    Xc, Xe = binding.lqer_quantize_mx(Xd, 6)
    oc, oe = mxint.mx_quantize(X, 6, axis=-1)
    assert np.array_equal(Xc.cpu().numpy(), oc) and np.array_equal(Xe.cpu().numpy(), oe)
    Yq = binding.lqer_linear_forward_q(h, Xc, Xe)
    assert torch.equal(Y, Yq)
    with pytest.raises(binding.LqerError):
        h.set_activation_bits(5)
    h.free()


@pytest.mark.parametrize("M,K,N,k,bits", [(33000, 272, 64, 33, 8), (32776, 528, 40, 0, 8), (40000, 1040, 112, 100, 6)])
def test_many_tokens_ragged_rows_and_columns(M, K, N, k, bits):
    # launches of 2048 workgroups and more take the row-wise form of the projection kernel (whole rows per wavefront,
    # block maxima across the four lanes of a quad, operands turned through LDS): ragged last row group, K that ends
    # inside a 256-wide tile, ranks in more than four groups, 6-bit activations; the whole output against the oracle
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(K, N, k, seed=M)
    h = upload(layer)
    if bits == 6:
        h.set_activation_bits(6)
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
    Xd = torch.from_numpy(X).cuda()
    Y = binding.lqer_linear_forward(h, Xd)
    assert_forward_matches(Y.cpu().numpy(), X, layer, act_bits=bits)
    Xc, Xe = binding.lqer_quantize_mx(Xd, bits)
    assert torch.equal(binding.lqer_linear_forward_q(h, Xc, Xe), Y)           # the lane-per-block form gives the same bits
    h.free()


@pytest.mark.parametrize("M,K,N,k,path,variant", [
    (1, 1024, 272, 32, 1, 11181), (16, 4096, 64, 16, 1, 11181), (20, 2304, 528, 33, 1, 11241), (5, 1024, 4096, 8, 1, 12241),
    (40, 512, 16384, 8, 1, 11421), (300, 1024, 528, 64, 2, 111), (300, 1024, 528, 64, 2, 112), (513, 4352, 1104, 16, 2, 211),
    (700, 2304, 272, 33, 2, 204), (100, 272, 48, 0, 2, 104)])
def test_output_as_mxint8(M, K, N, k, path, variant):
    # The result leaves as MXINT8 (blocks of 16 along N) from the epilogue of the main kernel: codes and
    # exponent bytes must be exactly what the oracle's quantizer makes of the fp32 Y the same kernel shape stores
    import torch
    from paper_2402_02446_amd import binding
    if N > 2048:
        layer = factors.PackedLayer(**synth.random_packed_layer(np.random.default_rng(N), K, N, k))
        ch = synth.gen_outlier_channels(np.random.default_rng(1), K, 4)
    else:
        layer, ch = oracle_layer_small(K, N, k, seed=M + k)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
    Xd = torch.from_numpy(X).cuda()
    Y = binding.lqer_linear_forward_ex(h, Xd, path=path, variant=variant).cpu().numpy()
    codes, exps = binding.lqer_linear_forward_requant(h, Xd, path=path, variant=variant)
    torch.cuda.synchronize()
    oc, oe = mxint.mx_quantize(Y, 8, axis=-1)
    assert np.array_equal(exps.cpu().numpy(), oe)
    assert np.array_equal(codes.cpu().numpy(), oc)
    # and the dequantized output is the oracle's Y to within the 8-bit step of each block
    Yq = mxint.mx_dequantize(codes.cpu().numpy(), exps.cpu().numpy(), 8, axis=-1)
    assert forward.rel_frobenius(Yq, forward.forward(X, layer)) < 2.0 ** -6
    h.free()


def test_output_as_mxint8_automatic_shape_and_errors():
    import torch
    from paper_2402_02446_amd import binding
    # a layer whose automatic streaming shape runs pairs of workgroups: the MXINT8 output must avoid them
    layer, ch = oracle_layer_big(4096, 4096, 32, seed=3)
    h = upload(layer)
    for M in (1, 16, 32):
        X = synth.gen_activations(np.random.default_rng(M), M, 4096, ch, 50.0)
        Xd = torch.from_numpy(X).cuda()
        codes, exps = binding.lqer_linear_forward_requant(h, Xd)
        Yq = mxint.mx_dequantize(codes.cpu().numpy(), exps.cpu().numpy(), 8, axis=-1)
        assert forward.rel_frobenius(Yq, forward.forward(X, layer)) < 2.0 ** -6
        with pytest.raises(binding.LqerError):
            binding.lqer_linear_forward_requant(h, Xd, path=1, variant=21181 if M <= 16 else 21141)
    h.free()
    odd, ch = oracle_layer_small(512, 40, 8, seed=1)             # N is no multiple of 16: no MXINT8 blocks along N
    h = upload(odd)
    Xd = torch.from_numpy(synth.gen_activations(np.random.default_rng(0), 4, 512, ch, 30.0)).cuda()
    with pytest.raises((binding.LqerError, RuntimeError)):
        binding.lqer_linear_forward_requant(h, Xd)
    h.free()


def test_layers_sharing_their_activations():
    # q/k/v or gate/up of a block see the same X_q (Sec. 4.1: one quantizer per activation tensor; Eq. 3 per layer):
    # the shared call quantizes X once and must give every layer the bits its own forward pass gives, and the
    # oracle's Y within the bound.  Ranks differ between the layers (one has none), token counts cover the tiled
    # kernel with and without split tiles and the streaming kernel (where the call is one pass per layer).
    import torch
    from paper_2402_02446_amd import binding
    K = 2304
    specs = [(528, 33, 21), (1000, 8, 22), (272, 0, 23), (4128, 64, 24)]
    layers, hs = [], []
    ch = None
    for (N, k, seed) in specs:
        layer, ch = (oracle_layer_small if N < 2000 else oracle_layer_big)(K, N, k, seed=seed)
        layers.append(layer)
        hs.append(upload(layer))
    for M in (300, 130, 70, 16):
        X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
        Xd = torch.from_numpy(X).cuda()
        alone = [binding.lqer_linear_forward(h, Xd).clone() for h in hs]
        torch.cuda.synchronize()
        for order in ([0, 1, 2, 3], [2, 3, 0], [3]):
            group = [hs[i] for i in order]
            Ys = [torch.full((M, layers[i].N), float("nan"), dtype=torch.float32, device="cuda") for i in order]
            binding.lqer_linear_forward_shared(group, Xd, Ys=Ys)
            torch.cuda.synchronize()
            for i, Y in zip(order, Ys):
                assert torch.equal(Y, alone[i]), (M, order, i)
        for i in (0, 3):
            assert forward.rel_frobenius(alone[i].cpu().numpy(), forward.forward(X, layers[i])) < Y_TOL
    # the shared call allocates nothing and uses one stream: captured in a HIP graph, every replay reproduces it
    M = 300
    group = [hs[0], hs[1], hs[3]]
    Xg = torch.from_numpy(synth.gen_activations(np.random.default_rng(5), M, K, ch, 30.0)).cuda()
    want = [binding.lqer_linear_forward(h, Xg).clone() for h in group]
    ws = torch.empty(binding.lqer_linear_shared_workspace_bytes(group, M), dtype=torch.uint8, device="cuda")
    Ys = [torch.empty_like(w) for w in want]
    binding.lqer_linear_forward_shared(group, Xg, Ys=Ys, workspace=ws)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.lqer_linear_forward_shared(group, Xg, Ys=Ys, workspace=ws)
    for rep in range(3):
        for Y in Ys:
            Y.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for Y, w in zip(Ys, want):
            assert torch.equal(Y, w), rep
    # layers of different K cannot share activations
    other, _ = oracle_layer_small(512, 64, 8, seed=1)
    ho = upload(other)
    with pytest.raises(binding.LqerError):
        binding.lqer_linear_forward_shared([hs[0], ho], torch.zeros((4, K), device="cuda"))
    ho.free()
    for h in hs:
        h.free()


def test_split_tiles_in_hip_graph_and_on_two_streams():
    # The flags of the hand-over are cleared by the projection kernel of every call, so replays of a captured
    # forward pass and two calls in flight on two streams (distinct workspaces) all reproduce the eager result.
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(2304, 528, 33, seed=21)
    h = upload(layer)
    M = 300
    X = torch.from_numpy(synth.gen_activations(np.random.default_rng(1), M, 2304, ch, 30.0)).cuda()
    X2 = torch.from_numpy(synth.gen_activations(np.random.default_rng(2), M, 2304, ch, 30.0)).cuda()
    for variant in (211, 212):
        want = binding.lqer_linear_forward_ex(h, X, path=2, variant=variant).clone()
        want2 = binding.lqer_linear_forward_ex(h, X2, path=2, variant=variant).clone()
        torch.cuda.synchronize()
        Xg, Yg = X.clone(), torch.empty_like(want)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            binding.lqer_linear_forward_ex(h, Xg, Y=Yg, path=2, variant=variant)
        for rep, (src, w) in enumerate([(X, want), (X2, want2), (X, want)]):
            Xg.copy_(src)
            Yg.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Yg, w), f"replay {rep} differs (variant {variant})"
            _ = binding.lqer_linear_forward_ex(h, X2, path=2, variant=variant)
        # two streams, two workspaces
        nbytes = binding.lqer_linear_workspace_bytes(h, M, 2)
        wsa = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        wsb = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        Ya, Yb = torch.empty_like(want), torch.empty_like(want)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for _ in range(5):
            with torch.cuda.stream(sa):
                binding.lqer_linear_forward_ex(h, X, Y=Ya, workspace=wsa, path=2, variant=variant)
            with torch.cuda.stream(sb):
                binding.lqer_linear_forward_ex(h, X2, Y=Yb, workspace=wsb, path=2, variant=variant)
        torch.cuda.synchronize()
        assert torch.equal(Ya, want) and torch.equal(Yb, want2)
    h.free()


@pytest.mark.parametrize("M,K,N,k,path,variant", [(5, 1024, 272, 32, 1, 0), (16, 2304, 528, 33, 1, 12241), (40, 512, 16384, 8, 1, 0),
                                                  (300, 1024, 528, 64, 2, 111), (300, 2304, 272, 33, 2, 212)])
def test_both_forms_of_weight_exponents_on_the_device(M, K, N, k, path, variant):
    # The device copy keeps W_q's exponents as nibbles when the layer spans at most 16 exponent values and as
    # bytes otherwise; the same layer is run in both forms (one far-off exponent byte on a block of zero
    # codes forces bytes without changing a single product) and must give the same bits, and export must
    # return the canonical bytes either way.
    import torch
    from paper_2402_02446_amd import binding
    if N > 2048:
        layer = factors.PackedLayer(**synth.random_packed_layer(np.random.default_rng(N), K, N, k))
        ch = synth.gen_outlier_channels(np.random.default_rng(1), K, 4)
    else:
        layer, ch = oracle_layer_small(K, N, k, seed=M + k)
    assert int(layer.We.max()) - int(layer.We.min()) <= 15
    wide = factors.PackedLayer(K=layer.K, N=layer.N, k=layer.k, kp=layer.kp, Wc=layer.Wc.copy(), We=layer.We.copy(),
                               Ac=layer.Ac, Ae=layer.Ae, Bc=layer.Bc, Be=layer.Be)
    wide.Wc[3, 8:16] = 0                                       # block 1 of column 3: all codes zero ...
    wide.We[3, 1] = 40                                         # ... so its exponent byte is free
    narrow = factors.PackedLayer(K=layer.K, N=layer.N, k=layer.k, kp=layer.kp, Wc=wide.Wc, We=layer.We,
                                 Ac=layer.Ac, Ae=layer.Ae, Bc=layer.Bc, Be=layer.Be)
    X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 30.0)
    Xd = torch.from_numpy(X).cuda()
    outs = []
    for lay in (narrow, wide):
        h = upload(lay)
        outs.append(binding.lqer_linear_forward_ex(h, Xd, path=path, variant=variant).clone())
        ex = binding.lqer_layer_export(h)
        assert np.array_equal(ex["Wc"], lay.Wc) and np.array_equal(ex["We"], lay.We)
        h.free()
    assert torch.equal(outs[0], outs[1])
    assert_forward_matches(outs[0].cpu().numpy(), X, narrow)


def test_split_is_refused_for_shapes_without_it():
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(1024, 272, 8, seed=2)
    h = upload(layer)
    X = synth.gen_activations(np.random.default_rng(2), 300, 1024, ch, 30.0)
    for variant in (201, 203, 207, 208, 213, 301, 411):
        with pytest.raises(binding.LqerError):
            _gpu_forward(h, X, path=2, variant=variant)
    h.free()


@pytest.mark.parametrize("variant", [211, 212, 204])
def test_split_tiles_give_the_same_bits_every_run(variant):
    # Output tiles cut along K: the pieces are added in K order by one workgroup, whatever the order
    # in which the others finish, so repeated runs agree bit for bit (and with the oracle within tolerance)
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(4096, 4096, 32, seed=5)
    h = upload(layer)
    M = 300
    Xn = synth.gen_activations(np.random.default_rng(M), M, 4096, ch, 50.0)
    X = torch.from_numpy(Xn).cuda()
    first = binding.lqer_linear_forward_ex(h, X, path=2, variant=variant).clone()
    assert_forward_matches(first.cpu().numpy(), Xn, layer)
    for _ in range(10):
        Y = torch.full_like(first, 3.0)
        binding.lqer_linear_forward_ex(h, X, Y=Y, path=2, variant=variant)
        assert torch.equal(Y, first)
    h.free()


@pytest.mark.parametrize("variant", [211, 212, 204, 311, 312, 304])
def test_split_along_tile_boundaries_and_in_equal_shares(variant):
    # 13 x 4 tiles of 128 x 512 (13 x 8, 13 x 16 for the smaller shapes) with 11 K tiles each: the chip holds
    # several workgroups per tile, so mode 2 cuts every tile into the same number of pieces (ragged: 11 K tiles
    # in pieces of 3 or 6, with empty units behind the last one) and mode 3 into equal shares that cross tiles.
    # Both against the oracle, and the same bits on a second run.
    import torch
    from paper_2402_02446_amd import binding
    K, N, k, M = 2816, 2048, 40, 1664
    layer, ch = oracle_layer_big(K, N, k, seed=variant)
    h = upload(layer)
    Xn = synth.gen_activations(np.random.default_rng(variant), M, K, ch, 50.0)
    X = torch.from_numpy(Xn).cuda()
    first = binding.lqer_linear_forward_ex(h, X, path=2, variant=variant).clone()
    assert_forward_matches(first.cpu().numpy(), Xn, layer)
    Y = torch.full_like(first, float("nan"))
    binding.lqer_linear_forward_ex(h, X, Y=Y, path=2, variant=variant)
    assert torch.equal(Y, first)
    h.free()


def test_a_wait_that_gives_up_ends_the_kernel_and_stores_nan():
    # The bounded wait of the work split, forced from the host: with a limit of zero polls every workgroup that
    # waits for another one's partial sums gives up at once.  The kernel must still end normally, every tile
    # that was cut must come out as NaN (never as a wrong number), tiles computed whole must be right, and with
    # the default limit back the same call must give the full result again.
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(4096, 4096, 32, seed=9)
    h = upload(layer)
    M = 300
    X = torch.from_numpy(synth.gen_activations(np.random.default_rng(M), M, 4096, ch, 50.0)).cuda()
    want = binding.lqer_linear_forward_ex(h, X, path=2, variant=211).clone()      # 24 tiles, all cut
    whole = binding.lqer_linear_forward_ex(h, X, path=2, variant=111).clone()
    torch.cuda.synchronize()
    assert torch.isfinite(want).all()
    try:
        binding.lqer_set_wait_limit(0)
        Y = binding.lqer_linear_forward_ex(h, X, path=2, variant=211)
        torch.cuda.synchronize()                                                # returns: the kernel ended
        assert torch.isnan(Y).all()
        Yw = binding.lqer_linear_forward_ex(h, X, path=2, variant=111)            # no cut tiles, no waits
        torch.cuda.synchronize()
        assert torch.equal(Yw, whole)
    finally:
        binding.lqer_set_wait_limit(1 << 22)
    Y = binding.lqer_linear_forward_ex(h, X, path=2, variant=211)
    torch.cuda.synchronize()
    assert torch.equal(Y, want)
    h.free()


def test_cfg4_70b_shape_every_tile():
    # LLaMA-2-70B-shaped MLP (8192 x 28672, k = 64) at M = 1, 16 (streaming kernel) and 4096 (tiled), in the
    # launch configuration the benchmark times: seeded packed bytes; the oracle on every row (M <= 16) or one
    # row of every band of 32 (M = 4096), against one column of every group of 32 columns plus the tile edges -
    # every output tile, every wavefront's part of it and every MFMA tile holds a compared element
    import torch
    from paper_2402_02446_amd import binding
    K, N, k = 8192, 28672, 64
    rng = np.random.default_rng(4)
    d = synth.random_packed_layer(rng, K, N, k)
    layer = factors.PackedLayer(**d)
    h = upload(layer)
    ch = synth.gen_outlier_channels(rng, K, round(0.01 * K))
    for M in (1, 16, 4096):
        X = synth.gen_activations(np.random.default_rng(M), M, K, ch, 50.0)
        assert binding.lqer_linear_path(h, M) == (1 if M <= 32 else 2)
        Y = _gpu_forward(h, X)
        assert np.all(np.isfinite(Y))
        rows, cols = tile_cover_samples(rng, M, N)
        cols = np.unique(np.r_[cols, 31, 32, 127, 128, 255, 256, 511, 512, N - 33])
        if M <= 16:
            rows = np.arange(M)
        else:
            rows = np.unique(np.r_[rows, 127, 128, 2047, 2048])
        err, ratio = assert_forward_matches(Y[np.ix_(rows, cols)], X[rows], layer, cols)
        print(f"M={M}: {len(rows)} x {len(cols)} samples, rel. Frobenius error {err:.3g}, largest |error| / bound {ratio:.3g}")
    h.free()


def test_paired_workgroups_give_the_same_bits_every_run():
    # Narrow layers run two workgroups per column block that both add into Y with fp32 atomics; with
    # exactly two addends on top of zero the sum does not depend on the order of arrival.
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(4096, 4096, 32, seed=3)
    h = upload(layer)
    for M in (1, 16, 32):
        X = torch.from_numpy(synth.gen_activations(np.random.default_rng(M), M, 4096, ch, 50.0)).cuda()
        first = binding.lqer_linear_forward(h, X).clone()
        for _ in range(20):
            Y = torch.full_like(first, 3.0)               # stale contents must not leak into the sum
            binding.lqer_linear_forward(h, X, Y=Y)
            assert torch.equal(Y, first)
    h.free()


def test_forward_in_hip_graph_replays():
    # The forward pass allocates nothing and uses only the caller's stream, so it can be captured in a
    # HIP graph (the benchmark times it that way).  Every replay must reproduce the eager result,
    # with eager work and synchronisations between the replays.
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_small(1024, 272, 32, seed=12)
    h = upload(layer)
    for M in (5, 200):
        X = torch.from_numpy(synth.gen_activations(np.random.default_rng(M), M, 1024, ch, 30.0)).cuda()
        X2 = torch.from_numpy(synth.gen_activations(np.random.default_rng(M + 1), M, 1024, ch, 30.0)).cuda()
        Y_eager = binding.lqer_linear_forward(h, X).clone()
        Y2_eager = binding.lqer_linear_forward(h, X2).clone()
        torch.cuda.synchronize()
        Xg = X.clone()
        Yg = torch.empty_like(Y_eager)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            binding.lqer_linear_forward(h, Xg, Y=Yg)
        for rep, (src, want) in enumerate([(X, Y_eager), (X2, Y2_eager), (X, Y_eager)]):
            Xg.copy_(src)
            Yg.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Yg, want), f"replay {rep} differs from the eager result (M={M})"
            _ = binding.lqer_linear_forward(h, X2)       # eager work between replays
            torch.cuda.synchronize()
        del g
    h.free()


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_shapes_on_the_automatic_path(seed):
    # Shapes nobody picked by hand: token counts on both sides of every dispatch boundary, K any multiple of 16,
    # N any size (ragged column groups), ranks from none to the limit; the automatic path and shape, against the
    # oracle, and the pre-quantized entry point giving the same bits.
    import torch
    from paper_2402_02446_amd import binding
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.choice([1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 129, 200, 257, 400]))
    K = 16 * int(rng.integers(1, 160))
    N = int(rng.integers(1, 1400))
    k = int(rng.integers(0, min(64, K, N) + 1))
    layer, ch = oracle_layer_big(K, N, k, seed=seed, n_outlier=max(1, K // 100))
    h = upload(layer)
    X = synth.gen_activations(rng, M, K, ch, 50.0)
    ld = (N + 3) // 4 * 4                                     # the row stride of Y must be a multiple of 4
    buf = torch.full((M, ld), float("nan"), dtype=torch.float32, device="cuda")
    binding.lqer_linear_forward(h, torch.from_numpy(X).cuda(), Y=buf[:, :N])
    Y = buf[:, :N].cpu().numpy()
    assert torch.isnan(buf[:, N:]).all()                      # nothing is written behind a row
    assert_forward_matches(Y, X, layer)
    Xc, Xe = forward.quantize_activations(X, 8)
    bufq = torch.empty_like(buf)
    binding.lqer_linear_forward_q(h, torch.from_numpy(Xc).cuda(), torch.from_numpy(Xe).cuda(), Y=bufq[:, :N])
    assert np.array_equal(bufq[:, :N].cpu().numpy(), Y), (M, K, N, k)
    h.free()
