"""The hidden-state read-out oracle against its pins, and the pins against planted mistakes.  CPU only."""
import os
import types

import pytest

import oracle.lm_head_oracle as L
from tests import lm_head_pins

SRC_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "lm_head_oracle.py")
SRC = open(SRC_PATH).read()

# One plausible mistake each, planted in a copy of the oracle's source; at least one pin must notice.
MUTANTS = [
    ("return h @ w.T", "return h @ w[:, ::-1].T"),
    ("return h @ w.T", "return (w @ h.T).T if h.shape[1] != w.shape[0] else h @ w"),
    ("        row = z[n] * inv_temperature\n        m = row.max()\n        lse[n]", "        row = z[n]\n        m = row.max()\n        lse[n]"),
    ("lse[n] = m + np.log(np.exp(row - m).sum())", "lse[n] = np.log(np.exp(row - m).sum())"),
    ("logp[n] = row[y[n]] - lse[n]", "logp[n] = row[y[n]] + lse[n]"),
    ("logp[n] = row[y[n]] - lse[n]", "logp[n] = z[n, y[n]] - lse[n]"),
    ("prob[int(y[n])] -= 1.0", "prob[int(y[n])] += 1.0"),
    ("prob[int(y[n])] -= 1.0", "pass"),
    ("dz[n] = (g[n] * inv_temperature) * prob", "dz[n] = g[n] * prob"),
    ("dz[n] = (g[n] * inv_temperature) * prob", "dz[n] = -(g[n] * inv_temperature) * prob"),
    ("d_hidden = dz @ _f64(weight)", "d_hidden = dz @ _f64(weight)[::-1]"),
    ("d_weight = dz.T @ _f64(hidden)", "d_weight = dz.T @ _f64(hidden)[::-1]"),
    ("d_weight = dz.T @ _f64(hidden)", "d_weight = np.abs(dz).T @ _f64(hidden)"),
]


@pytest.mark.parametrize("pin", lm_head_pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(L)


def _load(src):
    mod = types.ModuleType("lm_head_mutant")
    exec(compile(src, "lm_head_mutant.py", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("old,new", MUTANTS, ids=[f"m{i:02d}" for i in range(len(MUTANTS))])
def test_pins_catch(old, new):
    assert SRC.count(old) == 1, f"mutation site not found exactly once: {old!r}"
    mutant = _load(SRC.replace(old, new))
    caught = []
    for pin in lm_head_pins.ALL_PINS:
        try:
            pin(mutant)
        except Exception as exc:
            caught.append((pin.__name__, type(exc).__name__))
    assert caught, f"no pin noticed: {old!r} -> {new!r}"
