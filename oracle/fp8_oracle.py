"""CPU oracle for the FP8-E4M3 rollout perturbation.  TEST INFRASTRUCTURE ONLY.

The rollout side of the method runs in FP8 E4M3 (Sec. 2.1; App. "FP8 rollout").  The synthetic
workloads model its effect on the logits as a per-row symmetric quantisation in the sense of Eq. 1 —
scale s = max|X| / q_max, round, rescale — with the E4M3 value grid (q_max = 448) in place of the
integer grid.  This file states that operation from the format's definition:

  E4M3 "fn" (OCP 8-bit floating point): 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits;
  exponent field 0 holds subnormals m/8 * 2^-6; there are no infinities and S.1111.111 is NaN, so the
  largest finite magnitude is 1.75 * 2^8 = 448.  Conversion rounds to nearest, ties to the even
  mantissa, and saturates at +-448.

Arithmetic that decides a code is fixed to fp32 on both sides (the precision the GPU kernel uses):
s = fp32(max|z|) / fp32(448), q = fp32(z) / s, both correctly rounded fp32 divisions.  Shares no code
with the HIP path.  Pins: tests/test_fp8_oracle.py.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table() -> np.ndarray:
    """The value of each of the 256 codes (NaN for the two NaN codes), as float64: the grid that stands in for the
    integer grid of Eq. 1 when the rollout engine runs in FP8 (Sec. 2.1), from the published E4M3 "fn" format."""
    out = np.empty(256)
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 0xF, code & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = (m / 8.0) * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        out[code] = -v if s else v
    return out


def e4m3_encode(q) -> np.ndarray:
    """Codes of the E4M3 values nearest to q (ties to even, saturating): the rounding step of Eq. 1 on that grid.  q is
    taken as fp32 values."""
    q = np.asarray(q, dtype=np.float32).astype(np.float64)
    sign = np.signbit(q)
    a = np.minimum(np.abs(q), E4M3_MAX)
    _, ex = np.frexp(a)                       # a = f * 2^ex, f in [0.5, 1)
    e = np.maximum(ex - 1, -6)                # binade of a; everything below 2^-6 shares the subnormal spacing
    step = np.exp2((e - 3).astype(np.float64))
    k = np.rint(a / step)                     # exact scaling by a power of two; rint rounds ties to even
    val = k * step
    _, ex2 = np.frexp(val)
    e2 = np.maximum(ex2 - 1, -6)
    mant = np.rint(val / np.exp2((e2 - 3).astype(np.float64))).astype(np.int64)
    normal = val >= 2.0 ** -6
    code = np.where(normal, ((e2 + 7) << 3) | (mant - 8), mant)
    return (code | (sign.astype(np.int64) << 7)).astype(np.uint8)


def quantize_rows(z):
    """Per-row quantisation, Eq. 1 with symmetric per-row scaling (Sec. 2.1): (codes [R, V] uint8, scale [R] fp32) with
    s = max|z| / 448 (1 for an all-zero row)."""
    z = np.asarray(z, dtype=np.float32)
    amax = np.abs(z).max(axis=1).astype(np.float32)
    s = (amax / np.float32(E4M3_MAX)).astype(np.float32)
    s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    q = (z / s[:, None]).astype(np.float32)
    return e4m3_encode(q), s


def dequantize_rows(codes, scale):
    """The de-quantisation of Eq. 1: s * value(code) as fp32 (one correctly rounded fp32 multiplication)."""
    table = e4m3_decode_table().astype(np.float32)
    return (table[np.asarray(codes)] * np.asarray(scale, dtype=np.float32)[:, None]).astype(np.float32)


def rollout_logprob(z, y, valid=None):
    """log pi_roll of Alg. 1 ("Sampler-Trainer ratio") for a rollout engine whose logits went through Eq. 1: log-softmax
    of the quantise-dequantise round trip of each row, at token y (fp64 from the fp32 z_r)."""
    z = np.asarray(z, dtype=np.float32)
    R = z.shape[0]
    valid = np.ones(R, dtype=bool) if valid is None else np.asarray(valid).astype(bool)
    codes, s = quantize_rows(z)
    zr = dequantize_rows(codes, s).astype(np.float64)
    out = np.zeros(R)
    for n in range(R):
        if valid[n]:
            m = zr[n].max()
            out[n] = zr[n, int(y[n])] - (m + np.log(np.exp(zr[n] - m).sum()))
    return out
