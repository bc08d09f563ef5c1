"""lqer_linear_forward_static: the forward pass on the library's own static scratch, for callers that cannot
allocate device memory.  Checked through the C ABI against lqer_linear_forward (same kernels, so the same bits
wherever that call does not cut tiles between workgroups) and against the oracle, on two calls in a row, the
second with a smaller input, for the streaming and the tiled kernel; sizes beyond the scratch are refused."""
import numpy as np
import pytest

from paper_2402_02446_amd import synth
from helpers import assert_forward_matches, oracle_layer_big, upload

pytestmark = pytest.mark.gpu


def _both(h, layer, X, tiled):
    import torch
    from paper_2402_02446_amd import binding
    Xd = torch.from_numpy(X).cuda()
    Y = torch.full((X.shape[0], layer.N), float("nan"), dtype=torch.float32, device="cuda")
    binding.lqer_linear_forward_static(h, Xd, Y=Y)
    # the existing entry point; for the tiled kernel in the launch that never cuts tiles (variant 100), which is
    # what the static scratch - it has no slots for partial tiles - runs
    want = binding.lqer_linear_forward_ex(h, Xd, path=2, variant=100) if tiled else binding.lqer_linear_forward(h, Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y, want)
    assert_forward_matches(Y.cpu().numpy(), X, layer)
    if tiled:                                                  # the plain call may cut tiles: same result within the bound
        assert_forward_matches(binding.lqer_linear_forward(h, Xd).cpu().numpy(), X, layer)


def test_static_scratch_two_calls_second_smaller():
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(2304, 1040, 40, seed=31)
    h = upload(layer)
    for M in (30, 5):                                          # streaming kernel: 32-row cells, then 16-row cells
        assert binding.lqer_linear_path(h, M) == 1
        _both(h, layer, synth.gen_activations(np.random.default_rng(M), M, 2304, ch, 50.0), tiled=False)
    for M in (700, 130):                                       # tiled kernel, ragged last tile both times
        assert binding.lqer_linear_path(h, M) == 2
        _both(h, layer, synth.gen_activations(np.random.default_rng(M), M, 2304, ch, 50.0), tiled=True)
    # back to few tokens after the tiled calls: whatever they left in the scratch must not matter
    _both(h, layer, synth.gen_activations(np.random.default_rng(3), 3, 2304, ch, 50.0), tiled=False)
    h.free()


def test_static_scratch_refuses_sizes_beyond_it():
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(2304, 64, 0, seed=32)
    h = upload(layer)
    M = 8192                                                   # 8192 x (2304 + 128) bf16 = 40 MB > 32 MiB
    X = torch.zeros((M, 2304), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.LqerError) as e:
        binding.lqer_linear_forward_static(h, X)
    assert e.value.status == 5
    Y = binding.lqer_linear_forward_static(h, X[:0])           # no tokens: nothing to do
    assert Y.shape == (0, 64)
    h.free()


def test_static_scratch_under_graph_capture():
    # the callers the entry point is for: after one call outside any capture (which looks up the scratch's address),
    # the call is captured in a HIP graph and every replay - with eager work and synchronisations in between -
    # reproduces the eager result
    import torch
    from paper_2402_02446_amd import binding
    layer, ch = oracle_layer_big(1024, 528, 24, seed=33)
    h = upload(layer)
    for M in (7, 200):
        X = torch.from_numpy(synth.gen_activations(np.random.default_rng(M), M, 1024, ch, 50.0)).cuda()
        X2 = torch.from_numpy(synth.gen_activations(np.random.default_rng(M + 1), M, 1024, ch, 50.0)).cuda()
        want = binding.lqer_linear_forward_static(h, X).clone()
        want2 = binding.lqer_linear_forward_static(h, X2).clone()
        torch.cuda.synchronize()
        Xg, Yg = X.clone(), torch.empty_like(want)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            binding.lqer_linear_forward_static(h, Xg, Y=Yg)
        for rep, (src, w) in enumerate([(X, want), (X2, want2), (X, want)]):
            Xg.copy_(src)
            Yg.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Yg, w), f"replay {rep} differs (M={M})"
            _ = binding.lqer_linear_forward_static(h, X2)          # eager work on the same scratch between replays
            torch.cuda.synchronize()
        del g
    h.free()
