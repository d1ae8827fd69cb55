"""The whole-batch comparison machinery (tests/full_size.py) on the CPU: its worker tasks must accept a correct
device output and must catch a planted error.  The "device output" here is the oracle's own gradient rounded to
bf16, so nothing of the HIP path is involved; the mistakes are planted in that stand-in."""
import numpy as np
import torch

import oracle.ais_oracle as O
from paper_2605_13907_amd import workloads as W
from tests import full_size as F


def _bf16_bits(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_worker_tasks_accept_the_truth_and_catch_planted_errors(tmp_path):
    shape = W.config(2).scaled(vocab=3000, len_div=256, seed=5)
    batch = W.generate(shape, "cpu")
    z_bits = batch.logits.view(torch.int16).numpy().view(np.uint16)
    y, valid, cu = batch.token_ids.numpy(), batch.valid.numpy(), batch.cu_rows.numpy()
    R = batch.n_rows
    ref = O.ais_grpo(F.widen(z_bits, "bf16"), y, valid, cu, batch.logp_roll.double().numpy(),
                     batch.rewards.double().numpy(), shape.group_size)
    assert np.array_equal(F.widen(z_bits, "bf16"), batch.logits.double().numpy())      # widening is exact
    zpath = str(tmp_path / "z.npy")
    np.save(zpath, z_bits)
    a, b = 3, R - 2
    lp, lse = F.logprob_task((zpath, a, b, "bf16", y[a:b], valid[a:b], 1.0))
    assert np.array_equal(lp, ref["logp"][a:b]) and np.array_equal(lse, ref["lse"][a:b])

    g = ref["g"].copy()
    g[5] = 0.0                                                  # a row without gradient
    dz = O.dlogits_rows(F.widen(z_bits, "bf16"), ref["lse"], y, g)
    s = O.dlogits_rows(F.widen(z_bits, "bf16"), ref["lse"], y, (g != 0).astype(np.float64))

    def run(dz_bits, s_bits, g_scale):
        dzpath, spath = str(tmp_path / "dz.npy"), str(tmp_path / "s.npy")
        np.save(dzpath, dz_bits)
        np.save(spath, s_bits)
        F._MAPPED.clear()
        return F.gradient_task((zpath, dzpath, spath, a, b, "bf16", ref["lse"][a:b], y[a:b], g[a:b], g_scale[a:b], 1.0, True))

    good = run(_bf16_bits(dz), _bf16_bits(s), g)
    assert good["rows"] == b - a and good["dz_bad"] == 0 and good["gs_bad"] == 0 and good["first_bad"] is None
    assert good["dz_zero_rows_exact"] and good["gs_zero_rows_exact"] and good["dz_live_rows_written"]
    assert 0.0 < good["dz_worst"] <= 1.0 and 0.0 < good["gs_worst"] <= 1.0 and good["abs_sum"] > 0

    wrong = dz.copy()
    wrong[10, int(np.abs(dz[10]).argmax())] *= 1.05             # the row's largest element off by 5 %
    bad = run(_bf16_bits(wrong), _bf16_bits(s), g)
    assert bad["dz_bad"] >= 1 and bad["first_bad"][0] == "dz" and bad["first_bad"][1] == 10 and bad["gs_bad"] == 0
    wrong = dz.copy()
    wrong[5, 100] = 1e-6                                        # a row that must be exactly zero
    assert not run(_bf16_bits(wrong), _bf16_bits(s), g)["dz_zero_rows_exact"]
    wrong = dz.copy()
    wrong[12] = 0.0                                             # a row silently skipped
    assert not run(_bf16_bits(wrong), _bf16_bits(s), g)["dz_live_rows_written"]
    assert run(_bf16_bits(dz), _bf16_bits(s), g * 1.03)["gs_bad"] >= 1     # a wrong per-row scale
    assert run(_bf16_bits(dz), _bf16_bits(-s), g)["gs_bad"] >= 1            # a wrong sign of the direction
