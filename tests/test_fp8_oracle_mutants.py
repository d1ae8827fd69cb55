"""Are the pins of the FP8-E4M3 oracle sharp?  Each case plants one plausible mistake (a wrong bias, a missing
saturation, ties rounded up, a reciprocal instead of a division, a wrong sign) in a *copy* of the oracle's source, on
the CPU, and requires that at least one of its pins fails on the broken copy.  The real oracle is never modified."""
import os
import types

import pytest

from tests import test_fp8_oracle as pins

SRC_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "fp8_oracle.py")
SRC = open(SRC_PATH).read()

MUTANTS = [
    ("v = (m / 8.0) * 2.0 ** -6", "v = (m / 8.0) * 2.0 ** -7"),
    ("v = (1.0 + m / 8.0) * 2.0 ** (e - 7)", "v = (1.0 + m / 8.0) * 2.0 ** (e - 8)"),
    ("v = (1.0 + m / 8.0) * 2.0 ** (e - 7)", "v = (1.0 + m / 16.0) * 2.0 ** (e - 7)"),
    ("if e == 15 and m == 7:", "if e == 15:"),
    ("a = np.minimum(np.abs(q), E4M3_MAX)", "a = np.abs(q)"),
    ("a = np.minimum(np.abs(q), E4M3_MAX)", "a = np.minimum(np.abs(q), 240.0)"),
    ("e = np.maximum(ex - 1, -6)                # binade", "e = np.maximum(ex - 1, -7)                # binade"),
    ("k = np.rint(a / step)", "k = np.floor(a / step + 0.5)"),
    ("k = np.rint(a / step)", "k = np.floor(a / step)"),
    ("step = np.exp2((e - 3).astype(np.float64))", "step = np.exp2((e - 2).astype(np.float64))"),
    ("code = np.where(normal, ((e2 + 7) << 3) | (mant - 8), mant)", "code = np.where(normal, ((e2 + 8) << 3) | (mant - 8), mant)"),
    ("return (code | (sign.astype(np.int64) << 7)).astype(np.uint8)", "return code.astype(np.uint8)"),
    ("s = (amax / np.float32(E4M3_MAX)).astype(np.float32)", "s = (amax / np.float32(240.0)).astype(np.float32)"),
    ("amax = np.abs(z).max(axis=1).astype(np.float32)", "amax = z.max(axis=1).astype(np.float32)"),
    ("s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)", "s = s.astype(np.float32)"),
    ("q = (z / s[:, None]).astype(np.float32)", "q = (z * (np.float32(1.0) / s)[:, None]).astype(np.float32)"),
    ("return (table[np.asarray(codes)] * np.asarray(scale, dtype=np.float32)[:, None]).astype(np.float32)",
     "return (table[np.asarray(codes)] / np.asarray(scale, dtype=np.float32)[:, None]).astype(np.float32)"),
    ("out[n] = zr[n, int(y[n])] - (m + np.log(np.exp(zr[n] - m).sum()))",
     "out[n] = zr[n, int(y[n])] - np.log(np.exp(zr[n] - m).sum())"),
    ("zr = dequantize_rows(codes, s).astype(np.float64)", "zr = z.astype(np.float64)"),
]

PINS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


def broken_module(old, new):
    assert SRC.count(old) >= 1, f"mutation target not found: {old!r}"
    mod = types.ModuleType("fp8_oracle_mutant")
    exec(compile(SRC.replace(old, new, 1), "fp8_oracle_mutant", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("old,new", MUTANTS, ids=[f"m{i}" for i in range(len(MUTANTS))])
def test_some_pin_catches_the_planted_mistake(old, new, monkeypatch):
    monkeypatch.setattr(pins, "F", broken_module(old, new))
    caught = []
    for pin in PINS:
        try:
            with __import__("warnings").catch_warnings():
                __import__("warnings").simplefilter("ignore")
                pin()
        except Exception as e:                      # an assertion, or the mistake blowing up inside numpy
            caught.append(pin.__name__)
    assert caught, f"no pin noticed: {old!r} -> {new!r}"


def test_the_real_oracle_passes_every_pin():
    for pin in PINS:
        pin()
