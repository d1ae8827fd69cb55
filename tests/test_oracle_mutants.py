"""Are the oracle's pins sharp?  Each case plants one plausible mistake (a dropped term, a wrong sign,
a swapped operand, a wrong normalisation) in a *copy* of the oracle's source, on the CPU, and requires
that at least one pin fails on the broken copy.  The real oracle is never modified."""
import os
import types

import pytest

from tests import oracle_pins

SRC_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "ais_oracle.py")
SRC = open(SRC_PATH).read()

MUTANTS = [
    # O1
    ("lse[n] = m + np.log(np.exp(row - m).sum())", "lse[n] = np.log(np.exp(row - m).sum())"),
    ("logp[n] = row[y[n]] - lse[n]", "logp[n] = row[y[n]] + lse[n]"),
    ("row = z[n] * inv_temperature", "row = z[n]"),
    # O2
    ("d = _f64(logp_train) - _f64(logp_roll)", "d = _f64(logp_roll) - _f64(logp_train)"),
    ("wbar = np.minimum(rho, C)", "wbar = np.maximum(rho, C)"),
    ("wbar = np.minimum(rho, C)", "wbar = rho"),
    # O3
    ("g = r.reshape(-1, group_size)", "g = r.reshape(group_size, -1).T"),
    ("adv = g - g.mean(axis=1, keepdims=True)", "adv = g - np.median(g, axis=1, keepdims=True)"),
    ("adv = np.where(den > 0.0, adv / np.where(den > 0.0, den, 1.0), 0.0)", "adv = adv / (den + 1e-3)"),
    # O4
    ("var_w = ((w - mean_w) ** 2).mean()", "var_w = ((w - mean_w) ** 2).sum() / (w.size - 1)"),
    ("cv2 = (np.sqrt(var_w) / mean_w) ** 2", "cv2 = np.sqrt(var_w) / mean_w"),
    ("cv2 = (np.sqrt(var_w) / mean_w) ** 2", "cv2 = (var_w / mean_w) ** 2"),
    ("if mean_w > 0.0 else 0.0", "if mean_w > 0.0 else 1.0"),
    ("if mean_w > 0.0 else 0.0", "if mean_w > 1e-50 else 0.0"),
    ("alpha_ess = (1.0 + cv2) ** -0.5", "alpha_ess = (1.0 + cv2) ** -1.0"),
    ("dbar = np.abs(d[valid]).mean()", "dbar = np.abs(d[valid].mean())"),
    ("dbar = np.abs(d[valid]).mean()", "dbar = np.abs(rho[valid] - 1).mean()"),
    ("alpha_mis = min(1.0, dbar / p.delta)", "alpha_mis = min(1.0, dbar * p.delta)"),
    ("dsigma = std_aw / (std_a + p.eps_std) if", "dsigma = std_a / (std_aw + p.eps_std) if"),
    ("dsigma = std_aw / (std_a + p.eps_std) if std_a + p.eps_std > 0.0 else 0.0", "dsigma = std_aw / std_a if std_a else 0.0"),
    ("if std_a + p.eps_std > 0.0 else 0.0", "if std_a + p.eps_std > 0.0 else 1e9"),
    ("alpha_var = max(0.0, (dsigma - p.gamma) / p.gamma)", "alpha_var = max(0.0, dsigma - p.gamma)"),
    ("alpha_ess - p.beta_var * alpha_var", "alpha_ess + p.beta_var * alpha_var"),
    ("alpha_ess - p.beta_var * alpha_var", "alpha_ess - alpha_var"),
    (" * alpha_mis   # Eq. 17", "   # Eq. 17"),
    ("count = np.array([int(valid[cu[i]:cu[i + 1]].sum()) for i in range(B)]",
     "count = np.array([int(cu[i + 1] - cu[i]) for i in range(B)]"),
    ("a = _f64(adv)[seq][valid]                       # A broadcast to its tokens",
     "a = _f64(adv)[seq[::-1]][valid]"),
    ('out["kl_roll_train"] = float((-d[valid]).mean())', 'out["kl_roll_train"] = float((d[valid]).mean())'),
    ('out["kl_roll_train"] = float((-d[valid]).mean())', 'out["kl_roll_train"] = float(np.abs(d[valid]).mean())'),
    ("np.abs(np.exp(logp_train[valid]) - np.exp(_f64(logp_roll)[valid])).mean()",
     "np.abs(logp_train[valid] - _f64(logp_roll)[valid]).mean()"),
    # O5
    ("wt = 1.0 + alpha * (_f64(wbar) - 1.0)", "wt = 1.0 + alpha * _f64(wbar)"),
    ("wt = 1.0 + alpha * (_f64(wbar) - 1.0)", "wt = alpha + (1.0 - alpha) * _f64(wbar)"),
    # O6
    ("logp_at_rollout = logp if logp_old is None else _f64(logp_old)", "logp_at_rollout = logp"),
    ("diag = diagnostics(logp if logp_old is None else logp_old, logp_roll", "diag = diagnostics(logp, logp_roll"),
    ("active = (unclipped <= clipped)", "active = (unclipped >= clipped)"),
    ("s = np.minimum(unclipped, clipped)", "s = np.maximum(unclipped, clipped)"),
    ("clipped = np.clip(rho_on, 1.0 - p.clip_eps, 1.0 + p.clip_eps) * a",
     "clipped = np.clip(rho_on, 1.0 - p.clip_eps, 1.0) * a"),
    ("dobj = wtilde * a * rho_on * active", "dobj = wtilde * a * active"),
    ("dobj = dobj - p.beta_kl * (1.0 - np.exp(q))", "dobj = dobj + p.beta_kl * (1.0 - np.exp(q))"),
    ("obj = obj - p.beta_kl * (np.exp(q) - q - 1.0)", "obj = obj - p.beta_kl * (np.exp(q) - 1.0)"),
    ("1.0 / (B * cnt), 0.0)", "1.0 / cnt, 0.0)"),
    ("1.0 / (B * cnt), 0.0)", "1.0 / (B * np.maximum(1, np.diff(cu))[seq]), 0.0)"),
    ("loss -= float(", "loss += float("),
    # O7
    ("prob[int(y[n])] -= 1.0", "prob[int(y[n])] += 1.0"),
    ("prob[int(y[n])] -= 1.0", "pass"),
    ("prob = np.exp(z[n] * inv_temperature - lse[n])", "prob = np.exp(z[n] - lse[n])"),
    ("dz[n] = (g[n] * inv_temperature) * prob", "dz[n] = g[n] * prob"),
    ("dz[n] = (g[n] * inv_temperature) * prob", "dz[n] = -(g[n] * inv_temperature) * prob"),
]


def _load(src):
    mod = types.ModuleType("oracle_mutant")
    mod.__dict__["__name__"] = "oracle_mutant"
    import sys
    sys.modules["oracle_mutant"] = mod          # dataclasses looks the module up by name
    exec(compile(src, "oracle_mutant.py", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("old,new", MUTANTS, ids=[f"m{i:02d}" for i in range(len(MUTANTS))])
def test_pins_catch(old, new):
    assert SRC.count(old) == 1, f"mutation site not found exactly once: {old!r}"
    mutant = _load(SRC.replace(old, new))
    caught = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(mutant)
        except Exception as exc:   # an assertion, or the mistake crashing the computation
            caught.append((pin.__name__, type(exc).__name__))
    assert caught, f"no pin noticed: {old!r} -> {new!r}"
