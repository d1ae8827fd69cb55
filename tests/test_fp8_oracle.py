"""Pins of the FP8-E4M3 oracle: the format definition, torch's own float8_e4m3fn conversion (a library
routine), brute-force nearest-value search, and the workload generator's torch recipe.  CPU only."""
import math

import numpy as np
import torch

import oracle.fp8_oracle as F
from paper_2605_13907_amd import workloads as W


def test_decode_table_matches_format_and_torch():
    t = F.e4m3_decode_table()
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0 and t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6
    assert t[0x38] == 1.0 and t[0x00] == 0.0 and t[0x40] == 2.0
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ok = ~np.isnan(ref)
    assert np.array_equal(t[ok], ref[ok]) and np.array_equal(np.isnan(t), np.isnan(ref))
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                     # codes are ordered like their values


def test_encode_round_trip_ties_saturation():
    t = F.e4m3_decode_table()
    finite = np.array([c for c in range(256) if not np.isnan(t[c])], dtype=np.uint8)
    assert np.array_equal(F.e4m3_encode(t[finite]), finite)                   # representable values are fixed points
    # ties go to the even mantissa: 17 is halfway between 16 (m=0) and 18 (m=1) -> 16; 19 -> 20; 2^-10 -> 0
    enc = lambda x: t[F.e4m3_encode(np.array([x]))][0]
    assert enc(17.0) == 16.0 and enc(19.0) == 20.0 and enc(21.0) == 20.0 and enc(23.0) == 24.0
    assert enc(2.0 ** -10) == 0.0 and enc(3 * 2.0 ** -10) == 2.0 ** -8 and enc(-17.0) == -16.0
    assert enc(15.5) == 16.0 and enc(464.0) == 448.0 and enc(1e9) == 448.0 and enc(-1e9) == -448.0
    assert F.e4m3_encode(np.array([-0.0]))[0] == 0x80


def test_encode_is_nearest_by_brute_force():
    t = F.e4m3_decode_table()
    vals = np.array([v for v in t if not np.isnan(v)])
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.normal(0, 150, 3000), rng.normal(0, 1, 3000), rng.normal(0, 0.01, 1000)]).astype(np.float32)
    got = t[F.e4m3_encode(xs)]
    for x, g in zip(xs.astype(np.float64), got):
        xc = min(448.0, max(-448.0, x))
        best = np.abs(vals - xc).min()
        assert abs(g - xc) == best, (x, g)


def test_encode_matches_torch_cast():
    rng = np.random.default_rng(2)
    xs = np.concatenate([rng.normal(0, 200, 20000), rng.normal(0, 2, 20000), rng.normal(0, 0.02, 5000),
                         np.arange(-460, 460, 0.25)]).astype(np.float32)
    ref = torch.from_numpy(xs).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = F.e4m3_encode(xs)
    same = got == ref
    # the only admissible difference is the sign bit of a zero result
    assert np.all(same | ((got & 0x7F) == 0) & ((ref & 0x7F) == 0))


def test_quantize_rows_scale_and_extremes():
    rng = np.random.default_rng(3)
    z = rng.normal(0, 3, size=(6, 200)).astype(np.float32)
    z[4] = 0.0
    z[5, 7] = -50.0
    codes, s = F.quantize_rows(z)
    assert s.dtype == np.float32 and s[4] == 1.0 and np.all(codes[4] == 0)
    for n in (0, 1, 2, 3, 5):
        j = np.abs(z[n]).argmax()
        assert codes[n, j] == (0x7E if z[n, j] > 0 else 0xFE)                 # the row abs-max maps to +-448
        assert s[n] == np.float32(np.abs(z[n]).max()) / np.float32(448.0)
    zr = F.dequantize_rows(codes, s)
    big = np.abs(z) > np.abs(z).max(axis=1, keepdims=True) * (2.0 ** -6 / 448.0) * 8
    rel = np.abs(zr - z)[big] / np.abs(z)[big]
    assert rel.max() <= 2.0 ** -4 + 1e-6                                       # half a mantissa step of 2^-3


def test_rollout_logprob_matches_generator_recipe():
    """The oracle's round trip and the workload generator's torch recipe (clamp, cast to float8_e4m3fn, scale,
    log_softmax) are two independent routes to the same log-probabilities."""
    shape = W.config(2).scaled(vocab=1000, len_div=128, seed=13)
    b = W.generate(shape, "cpu")
    z = b.logits.float().numpy()
    got = F.rollout_logprob(z, b.token_ids.numpy())
    np.testing.assert_allclose(got, b.logp_roll.double().numpy(), atol=5e-6)
    zr_torch = W.fp8_rollout_logits(b.logits.float()).numpy()
    codes, s = F.quantize_rows(z)
    assert np.array_equal(F.dequantize_rows(codes, s), zr_torch)


def test_reciprocal_division_scheme_is_correctly_rounded():
    """The arithmetic the GPU kernels use for z / s, replayed on the CPU with exact rationals and fp32
    roundings: r = RN(1/s); q0 = RN(x r); q1 = RN(q0 + RN(x - q0 s) r); q = RN(q1 + RN(x - q1 s) r).
    q1 is a faithful quotient, so its residual is exactly representable, and q equals the correctly rounded
    quotient for divisors whose significand is not all ones (Markstein's theorem).  The single-correction
    variant is NOT always correct (q0 can be more than one ulp off): this test also shows such a case."""
    from fractions import Fraction

    def rn(fr):                      # round a rational to the nearest fp32, ties to even
        f = np.float32(float(fr))    # float(Fraction) is correctly rounded to fp64; then fp64 -> fp32
        cands = [np.nextafter(f, np.float32(-np.inf)), f, np.nextafter(f, np.float32(np.inf))]
        best = min(cands, key=lambda c: (abs(Fraction(float(c)) - fr), int(np.float32(c).view(np.uint32)) & 1))
        return np.float32(best)

    F = lambda v: Fraction(float(v))
    rng = np.random.default_rng(5)
    first_residual_inexact = 0
    cases = [(np.float32(-52187192.0), np.float32(130199.8359375))]       # q0 is 1.03 ulp off here
    for _ in range(3000):
        s = np.float32(10.0 ** rng.uniform(-6, 6) * rng.uniform(1, 2))
        cases.append((np.float32(rng.uniform(-448, 448) * float(s)), s))
    for x, s in cases:
        if (s.view(np.uint32) & 0x7FFFFF) == 0x7FFFFF:
            continue
        fs, fx = F(s), F(x)
        r = rn(1 / fs)
        q0 = rn(fx * F(r))
        e0 = rn(fx - F(q0) * fs)
        first_residual_inexact += F(e0) != fx - F(q0) * fs
        q1 = rn(F(q0) + F(e0) * F(r))
        e1 = rn(fx - F(q1) * fs)
        assert F(e1) == fx - F(q1) * fs, (x, s)                  # residual of the faithful quotient: exact
        q = rn(F(q1) + F(e1) * F(r))
        assert q == rn(fx / fs), (x, s)
    assert first_residual_inexact >= 1
