"""GPU parity of lqer_quantize_mx against the oracle: bit-exact codes and exponent bytes
(Sec. 2.2, Sec. 4.1)."""
import numpy as np
import pytest

from oracle import mxint
from paper_2402_02446_amd import synth

pytestmark = pytest.mark.gpu


def _run(x_np, bits, ld=None):
    import torch
    from paper_2402_02446_amd import binding
    rows, cols = x_np.shape
    if ld is None:
        x = torch.from_numpy(x_np).cuda()
    else:
        buf = torch.zeros((rows, ld), dtype=torch.float32, device="cuda")
        buf[:, :cols] = torch.from_numpy(x_np).cuda()
        buf[:, cols:] = 1.0e30                     # must never be read
        x = buf[:, :cols]
    codes, exps = binding.lqer_quantize_mx(x, bits)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), exps.cpu().numpy()


def _check(x_np, bits, ld=None):
    codes, exps = _run(x_np, bits, ld)
    oc, oe = mxint.mx_quantize(x_np, bits, axis=-1)
    if bits == 4:
        oc = mxint.pack_int4(oc)
    assert np.array_equal(exps, oe)
    assert np.array_equal(codes.view(np.uint8), oc.view(np.uint8))


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_adversarial_blocks(bits):
    rng = np.random.default_rng(0)
    blocks = synth.adversarial_blocks(rng, 4096)            # ties, saturation, zeros, subnormals, huge
    _check(blocks.reshape(256, 256), bits)


@pytest.mark.parametrize("bits", [8, 6, 4])
@pytest.mark.parametrize("shape", [(1, 16), (3, 48), (16, 512), (17, 4096), (257, 1040)])
def test_shapes_and_ragged_tails(bits, shape):
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(shape) * np.exp2(rng.integers(-12, 12, (shape[0], 1)))).astype(np.float32)
    _check(x, bits)


def test_strided_rows():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((37, 272)).astype(np.float32)
    _check(x, 8, ld=300)


def test_empty_is_a_noop():
    import torch
    from paper_2402_02446_amd import binding
    x = torch.zeros((0, 64), dtype=torch.float32, device="cuda")
    codes, exps = binding.lqer_quantize_mx(x, 8)
    assert codes.shape == (0, 64) and exps.shape == (0, 4)


def test_outlier_activations_full_width():
    # the activation recipe of the LLaMA-shaped workloads: 1 % of channels scaled by 50
    wl = synth.WORKLOADS["cfg3_up"]
    rng = np.random.default_rng(5)
    ch = synth.gen_outlier_channels(rng, wl.K, wl.n_outlier)
    x = synth.gen_activations(rng, 2048, wl.K, ch, wl.gain)
    _check(x, 8)
