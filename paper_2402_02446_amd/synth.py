"""Seeded synthetic inputs for the LQER linear layer.

Pure numpy random draws: this module holds none of the method's arithmetic
(no quantizer, no SVD, no matmul).  It serves the oracle-side tests and the
HIP-side harness alike, as data.

The draws stand in for what the paper uses and this build does not have:
trained OPT/LLaMA weights, a SlimPajama calibration subset, and real LLM
activations whose few outlier channels are much larger than the rest
(Sec. 1, Sec. 3.2, Sec. 4.1).

Recipe (fixed draw order W -> outlier channel set -> calibration rows -> X):
  W      ~ N(0, 0.02^2), fp32, shape K x N (in x out, Y = X W)
  chans  = `n_outlier` distinct channel indices, uniform without replacement
  calib  ~ N(0, 1), fp32, [n_samples][rows][K], outlier channels scaled by `gain`
  X      ~ N(0, 1), fp32, [M][K], same channels scaled by `gain`
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    K: int
    N: int
    Ms: tuple            # token counts this workload is run at
    k: int               # rank of the correction
    n_outlier: int       # number of outlier channels
    gain: float          # their scale factor
    calib_rows: int = 128
    calib_samples: int = 1
    seed: int = 0
    notes: str = ""


def _pct(K: int) -> int:
    return max(1, round(0.01 * K))


# The five configurations of the benchmark plan, by name.
WORKLOADS = {
    "cfg1": Workload("cfg1", 512, 512, (16,), 8, 8, 30.0),
    "cfg2": Workload("cfg2", 4096, 4096, (1, 16), 32, _pct(4096), 50.0),
    "cfg3_up": Workload("cfg3_up", 4096, 11008, (2048,), 32, _pct(4096), 50.0),
    "cfg3_down": Workload("cfg3_down", 11008, 4096, (2048,), 32, _pct(11008), 50.0),
    "cfg4": Workload("cfg4", 8192, 28672, (1, 16, 4096), 64, _pct(8192), 50.0),
}

# cfg5: the seven linears of one LLaMA-7B decoder block at M = 32 * 2048 tokens.
CFG5_LINEARS = (("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                ("gate", 4096, 11008), ("up", 4096, 11008), ("down", 11008, 4096))
CFG5_M = 32 * 2048


@dataclass
class Draw:
    W: np.ndarray
    channels: np.ndarray
    calib: np.ndarray
    X: dict = field(default_factory=dict)     # M -> X[M][K]


def gen_weight(rng: np.random.Generator, K: int, N: int, std: float = 0.02) -> np.ndarray:
    return (rng.standard_normal((K, N), dtype=np.float32) * np.float32(std)).astype(np.float32)


def gen_outlier_channels(rng: np.random.Generator, K: int, n_outlier: int) -> np.ndarray:
    return np.sort(rng.choice(K, size=n_outlier, replace=False))


def gen_activations(rng: np.random.Generator, rows: int, K: int, channels: np.ndarray,
                    gain: float) -> np.ndarray:
    x = rng.standard_normal((rows, K), dtype=np.float32)
    x[:, channels] *= np.float32(gain)
    return x


def draw(wl: Workload, Ms=None, with_weight: bool = True) -> Draw:
    """All inputs of one workload, in the fixed draw order."""
    rng = np.random.default_rng(wl.seed)
    W = gen_weight(rng, wl.K, wl.N) if with_weight else None
    ch = gen_outlier_channels(rng, wl.K, wl.n_outlier)
    calib = np.stack([gen_activations(rng, wl.calib_rows, wl.K, ch, wl.gain)
                      for _ in range(wl.calib_samples)])
    d = Draw(W=W, channels=ch, calib=calib)
    for M in (wl.Ms if Ms is None else Ms):
        d.X[M] = gen_activations(rng, M, wl.K, ch, wl.gain)
    return d


def gen_factor_standins(rng: np.random.Generator, K: int, N: int, k: int, channels: np.ndarray,
                        gain: float, err_scale: float = 0.02 / 16.0):
    """Random stand-ins for A_k (K x k) and B_k (k x N) at sizes where an exact
    SVD is too slow for a test: orthogonal-looking columns divided by an
    S-like channel weight, and rows with a decaying magnitude profile of the
    size a 4-bit quantization error of W would have.  Only draws and scaling
    of draws; the quantization of these factors is done by whoever uses them.
    """
    A = rng.standard_normal((K, k)) / np.sqrt(K)
    A[channels, :] /= gain
    decay = 1.0 / np.sqrt(1.0 + np.arange(k))
    B = rng.standard_normal((k, N)) * (err_scale * np.sqrt(K) * decay)[:, None]
    return A, B


def adversarial_blocks(rng: np.random.Generator, n_blocks: int) -> np.ndarray:
    """fp32 rows of 16 built to stress a block quantizer: exact ties, values
    that round up to the saturation limit, zeros, subnormals, huge and tiny
    magnitudes, mixed signs.  Returns [n_blocks][16] fp32."""
    out = np.zeros((n_blocks, 16), dtype=np.float32)
    for i in range(n_blocks):
        kind = i % 8
        e = int(rng.integers(-100, 100))
        base = np.float32(2.0) ** np.float32(e)
        if kind == 0:      # all zero
            pass
        elif kind == 1:    # ties at .5 in code units
            q = rng.integers(-126, 127, size=16).astype(np.float32) + np.float32(0.5)
            out[i] = q * base / np.float32(64.0)
            out[i, 0] = np.float32(1.5) * base      # pins the exponent to e
        elif kind == 2:    # just below the next power of two: rounds to 128 -> saturates
            out[i] = np.float32(rng.standard_normal(16)) * base * np.float32(0.3)
            out[i, 3] = np.nextafter(np.float32(2.0) * base, np.float32(0.0))
            out[i, 7] = -np.nextafter(np.float32(2.0) * base, np.float32(0.0))
        elif kind == 3:    # subnormal inputs
            out[i] = (rng.integers(-2000, 2000, size=16).astype(np.float32)
                      * np.float32(1.401298464324817e-45))
        elif kind == 4:    # near the top of the fp32 range
            out[i] = np.float32(rng.uniform(-1, 1, 16)) * np.float32(3.0e38)
        elif kind == 5:    # one outlier dominates
            out[i] = np.float32(rng.standard_normal(16))
            out[i, int(rng.integers(0, 16))] *= np.float32(1.0e4)
        elif kind == 6:    # smallest normals and mixed subnormals
            out[i] = np.float32(rng.uniform(-4, 4, 16)) * np.float32(1.1754943508222875e-38)
        else:              # ordinary Gaussian at a random binade
            out[i] = np.float32(rng.standard_normal(16)) * base
    return out


def random_packed_layer(rng: np.random.Generator, K: int, N: int, k: int, w_bits: int = 4):
    """Random canonical bytes with the statistics of a quantized Gaussian layer, for timing runs
    at sizes where quantizing real draws on the host would dominate the run: 4-bit codes drawn
    uniformly from [-7, 7] (2-bit: from {-1, 0, 1}, four per byte) with exponent bytes near 2^-6, int8 factor
    codes with exponents near 2^-8 (A_k) and 2^-10 (B_k).  Returns a dict of the six canonical arrays plus kp
    (and w_bits when it is not 4)."""
    kp = ((k + 15) // 16) * 16
    if w_bits == 4:
        nib = rng.integers(0, 15, size=(N, K), dtype=np.uint8)        # 15 values: the codes -7 .. 7
        nib[nib >= 8] += 1                                            # 8..14 -> 9..15 (codes -7..-1); nibble 8 (-8) never occurs
        Wc = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    else:
        pair = rng.integers(0, 3, size=(N, K), dtype=np.uint8)        # 0, 1, 2 -> bit pairs 00, 01, 11 (codes 0, 1, -1)
        pair[pair == 2] = 3
        Wc = (pair[:, 0::4] | (pair[:, 1::4] << 2) | (pair[:, 2::4] << 4) | (pair[:, 3::4] << 6)).astype(np.uint8)
    We = rng.integers(119, 123, size=(N, K // 16), dtype=np.uint8)
    Ac = rng.integers(-127, 128, size=(kp, K)).astype(np.int8)
    Ae = rng.integers(117, 121, size=(kp, K // 16), dtype=np.uint8)
    Bc = rng.integers(-127, 128, size=(N, kp)).astype(np.int8)
    Be = rng.integers(115, 119, size=(N, max(kp // 16, 0)), dtype=np.uint8)
    if kp > k:
        Ac[k:] = 0
        Ae[k:] = 0
        Bc[:, k:] = 0
    d = dict(K=K, N=N, k=k, kp=kp, Wc=Wc, We=We, Ac=Ac, Ae=Ae, Bc=Bc, Be=Be)
    if w_bits != 4:
        d["w_bits"] = w_bits
    return d


def random_int_layer(rng: np.random.Generator, K: int, N: int, k: int):
    """Random canonical arrays of the scaled-integer variant (INT4 codes in groups of 128 with FP16 scales, INT8
    factors) with the statistics of a quantized Gaussian layer, for timing runs: codes uniform in [-7, 7], weight
    scales near 0.06 / 7, factor scales near 2^-8 / 127 (A_k) and 2^-4 / 127 (B_k).  Returns a dict of the six arrays plus kp."""
    kp = ((k + 15) // 16) * 16
    nib = rng.integers(0, 15, size=(N, K), dtype=np.uint8)
    nib[nib >= 8] += 1
    Wc = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    Ws = (rng.uniform(0.05, 0.07, size=(N, K // 128)) / 7.0).astype(np.float16)
    Ac = rng.integers(-127, 128, size=(kp, K)).astype(np.int8)
    As = (rng.uniform(0.8, 1.2, size=(kp, K // 128)) * 2.0 ** -8 / 127.0).astype(np.float16)
    Bc = rng.integers(-127, 128, size=(N, kp)).astype(np.int8)
    Bs = (rng.uniform(0.8, 1.2, size=(N,)) * 2.0 ** -4 / 127.0).astype(np.float16)
    if kp > k:
        Ac[k:] = 0
        Bc[:, k:] = 0
    return dict(K=K, N=N, k=k, kp=kp, Wc=Wc, Ws=Ws, Ac=Ac, As=As, Bc=Bc, Bs=Bs)
