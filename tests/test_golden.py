"""Values printed in the paper (tests/golden/) against the oracle's defaults and the workloads."""
import os

import oracle.ais_oracle as O
from paper_2605_13907_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split()
            out[k] = float(v)
    return out


def test_oracle_defaults_are_the_papers():
    g = read_golden("hyperparameters.txt")
    p = O.Params()
    assert (p.C, p.delta, p.gamma, p.eps_std, p.clip_eps) == (g["C"], g["delta"], g["gamma"], g["eps_std"], g["clip_eps"])
    assert p.adv_mode == 0 and p.alpha_override < 0 and p.beta_kl == 0.0 and p.inv_temperature == 1.0


def test_workloads_use_the_papers_group_size():
    g = read_golden("hyperparameters.txt")
    for k in (2, 3, 4, 5):
        assert W.config(k).group_size == int(g["group_size"])
