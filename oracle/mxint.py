"""MXINT block format: oracle quantizer, dequantizer and canonical byte layouts.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sec. 2.2 describes MXINT as a block of fixed-point mantissas sharing one
exponent; Sec. 4.1 fixes the block at 16 elements ([1,16] for activations,
[16,1] for W_q, A_k, B_k, i.e. always along the contraction axis) and the
mantissa widths (4 for W_q - 2 in the W2A8 setup of Sec. 4.4 -, 8 for X, A_k, B_k).  The paper gives no formula,
so the reading taken here is:

  amax  = max |v_i| over the block
  e     = floor(log2 amax), clamped to [-127, 127];  e = -127 when amax == 0
  ebyte = e + 127                                    (one byte per block)
  scale = 2^(e - (b - 2))          1 sign bit, 1 integer bit, b-2 fraction bits
  c_i   = clamp(round_half_even(v_i / scale), -(2^(b-1) - 1), +(2^(b-1) - 1))
  dq    : v^_i = c_i * scale

Rounding that reaches 2^(b-1) saturates; the exponent is never bumped.
All arithmetic is fp64; every step above is exact in fp64 for fp32 inputs.

Sec. 4.1 gives W_q, A_k and B_k 4-bit shared exponents (activations keep 8 bits)
and states no bias for them.  Reading taken for exp_bits = 4: one bias per tensor,
chosen so that the tensor's largest block keeps its own exponent,

  top   = max over the tensor's blocks of e
  floor = max(top - 15, -127)
  e'    = max(e, floor)                              stored as the nibble e' - floor

and a block below the floor is quantized with e' (its codes shrink towards zero:
the narrow exponent cannot reach it).  Everything else is as above with e' for e.
"""
from __future__ import annotations

import numpy as np

BLOCK = 16
EXP_BIAS = 127
E_MIN = -127
E_MAX = 127


def code_limit(bits: int) -> int:
    """Largest code magnitude of a b-bit symmetric mantissa."""
    return (1 << (bits - 1)) - 1


def _to_blocks(v: np.ndarray, axis: int) -> np.ndarray:
    """Move `axis` last and split it into blocks of 16: shape (..., n/16, 16)."""
    v = np.moveaxis(v, axis, -1)
    n = v.shape[-1]
    if n % BLOCK != 0:
        raise ValueError(f"length {n} along the block axis is not a multiple of {BLOCK}")
    return v.reshape(v.shape[:-1] + (n // BLOCK, BLOCK))


def block_exponent(amax: np.ndarray) -> np.ndarray:
    """Unbiased shared exponent e = floor(log2 amax) clamped to [-127,127]; -127 for 0."""
    amax = np.asarray(amax, dtype=np.float64)
    _, ex = np.frexp(amax)               # amax = m * 2^ex with m in [0.5, 1)
    e = np.where(amax > 0.0, ex - 1, E_MIN)
    return np.clip(e, E_MIN, E_MAX).astype(np.int64)


def mx_quantize(v, bits: int, axis: int = -1, exp_bits: int = 8):
    """Quantize `v` to MXINT with `bits`-bit mantissas in blocks of 16 along `axis`.

    Returns (codes, exps): codes is int8 with the shape of `v`; exps is uint8
    (biased by 127) with `axis` shrunk by 16.  With exp_bits = 4 the bytes of one
    call span at most 16 consecutive values (see the head of this file);
    exp4_bias() and pack_exp4() turn them into the stored nibbles.
    """
    v = np.asarray(v, dtype=np.float64)
    if not np.all(np.isfinite(v)):
        raise ValueError("MXINT quantizer requires finite inputs")
    if exp_bits not in (4, 8):
        raise ValueError("shared exponents are 4 or 8 bits wide")
    blk = _to_blocks(v, axis)
    amax = np.max(np.abs(blk), axis=-1)
    e = block_exponent(amax)
    if exp_bits == 4 and e.size:
        e = np.maximum(e, max(int(e.max()) - 15, E_MIN))
    shift = e - (bits - 2)                                   # log2(scale)
    q = np.rint(np.ldexp(blk, (-shift)[..., None]))          # v / scale, exact, then RNE
    lim = code_limit(bits)
    codes = np.clip(q, -lim, lim).astype(np.int8)
    codes = codes.reshape(codes.shape[:-2] + (codes.shape[-2] * BLOCK,))
    codes = np.moveaxis(codes, -1, axis)
    exps = np.moveaxis((e + EXP_BIAS).astype(np.uint8), -1, axis)
    return np.ascontiguousarray(codes), np.ascontiguousarray(exps)


def mx_dequantize(codes, exps, bits: int, axis: int = -1) -> np.ndarray:
    """v^ = code * 2^(e - (bits-2)) in fp64 (exact)."""
    c = _to_blocks(np.asarray(codes).astype(np.float64), axis)
    e = np.moveaxis(np.asarray(exps).astype(np.int64), axis, -1) - EXP_BIAS
    out = np.ldexp(c, (e - (bits - 2))[..., None])
    out = out.reshape(out.shape[:-2] + (out.shape[-2] * BLOCK,))
    return np.ascontiguousarray(np.moveaxis(out, -1, axis))


# --------------------------------------------------------------------------
# canonical byte layouts (contraction axis contiguous for every tensor)
# --------------------------------------------------------------------------

def pack_int4(codes: np.ndarray) -> np.ndarray:
    """[..., n] int8 codes in [-7,7] -> [..., n/2] uint8.

    Element 2i sits in the low nibble, element 2i+1 in the high nibble, both as
    two's-complement nibbles.
    """
    c = np.asarray(codes).astype(np.int16)
    if c.shape[-1] % 2:
        raise ValueError("need an even number of 4-bit codes")
    lo = c[..., 0::2] & 0xF
    hi = c[..., 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    """Inverse of pack_int4: [..., n/2] uint8 -> [..., n] int8."""
    p = np.asarray(packed).astype(np.int16)
    lo = p & 0xF
    hi = (p >> 4) & 0xF
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int16)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    out = np.where(out >= 8, out - 16, out)
    return out.astype(np.int8)


def pack_int2(codes: np.ndarray) -> np.ndarray:
    """[..., n] int8 codes in [-1,1] (2-bit mantissas) -> [..., n/4] uint8: element 4i in bits 0-1,
    4i+1 in bits 2-3, 4i+2 in bits 4-5, 4i+3 in bits 6-7, each as a two's-complement pair of bits."""
    c = np.asarray(codes).astype(np.int16)
    if c.shape[-1] % 4:
        raise ValueError("need a multiple of four 2-bit codes")
    out = np.zeros(c.shape[:-1] + (c.shape[-1] // 4,), dtype=np.int16)
    for j in range(4):
        out |= (c[..., j::4] & 0x3) << (2 * j)
    return out.astype(np.uint8)


def unpack_int2(packed: np.ndarray) -> np.ndarray:
    """Inverse of pack_int2: [..., n/4] uint8 -> [..., n] int8."""
    p = np.asarray(packed).astype(np.int16)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 4,), dtype=np.int16)
    for j in range(4):
        out[..., j::4] = (p >> (2 * j)) & 0x3
    out = np.where(out >= 2, out - 4, out)
    return out.astype(np.int8)


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Canonical bytes of `bits`-bit weight codes: nibbles (4) or bit pairs (2)."""
    return pack_int4(codes) if bits == 4 else pack_int2(codes)


def unpack_codes(packed: np.ndarray, bits: int) -> np.ndarray:
    return unpack_int4(packed) if bits == 4 else unpack_int2(packed)


def exp4_bias(exps) -> int:
    """The byte a zero nibble stands for in a tensor whose exponent bytes span at
    most 16 values: its largest byte minus 15 (not below 0)."""
    e = np.asarray(exps)
    top = int(e.max()) if e.size else 0
    if e.size and top - int(e.min()) > 15:
        raise ValueError("exponent bytes span more than 16 values")
    return max(top - 15, 0)


def pack_exp4(exps):
    """[..., n] exponent bytes of one tensor -> ([..., n/2] uint8, bias): block 2i
    in the low nibble, block 2i+1 in the high nibble, each byte minus the bias."""
    e = np.asarray(exps).astype(np.int16)
    if e.shape[-1] % 2:
        raise ValueError("need an even number of exponents")
    bias = exp4_bias(e)
    n = e - bias
    return (n[..., 0::2] | (n[..., 1::2] << 4)).astype(np.uint8), bias


def unpack_exp4(packed, bias: int) -> np.ndarray:
    """Inverse of pack_exp4."""
    p = np.asarray(packed).astype(np.int16)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int16)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = (p >> 4) & 0xF
    return (out + bias).astype(np.uint8)


def average_bits(mant_bits: int, exp_bits: int, block: int = BLOCK) -> float:
    """Average bits per element of one MXINT tensor (App. D): one shared
    exponent spread over `block` mantissas."""
    return mant_bits + exp_bits / block


def lqer_average_weight_bits(m: int, n: int, k: int, w_bits: int, lr_bits: int,
                             w_exp_bits: int, lr_exp_bits: int) -> float:
    """Average stored bits per element of W for W_q plus A_k, B_k (App. D)."""
    total = m * n * average_bits(w_bits, w_exp_bits) + (m + n) * k * average_bits(lr_bits, lr_exp_bits)
    return total / (m * n)
