"""Runs the oracle over row chunks in worker processes.  TEST INFRASTRUCTURE ONLY (CPU-baseline timing).

The workers call oracle/ais_oracle.py as it stands; this file only moves data: it widens raw bf16 bit
patterns to float64 exactly and splits the rows.  It imports neither torch nor the GPU package, so that
worker processes start quickly and never touch a GPU.
"""
from __future__ import annotations

import os
from concurrent.futures import ProcessPoolExecutor
import multiprocessing as mp

import numpy as np

from oracle import ais_oracle as O


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Raw logits -> float64, exactly.  bf16 arrives as uint16 bit patterns (the upper half of an fp32)."""
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.astype(np.float64)


def _logprob_chunk(args):
    bits, dtype, y, valid, inv_t = args
    return O.token_logprob(widen(bits, dtype), y, valid, inv_t)


def _dlogits_chunk(args):
    bits, dtype, lse, y, g, inv_t = args
    dz = O.dlogits_rows(widen(bits, dtype), lse, y, g, inv_t)
    return float(np.abs(dz).sum())          # the gradient itself stays in the worker: only a checksum returns


def _noop(_):
    return os.getpid()


class OraclePool:
    def __init__(self, workers: int):
        self.workers = workers
        self.pool = ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))
        list(self.pool.map(_noop, range(workers * 4)))      # start the workers before anything is timed

    def close(self):
        self.pool.shutdown()

    def whole_path(self, bits, dtype, y, valid, cu_rows, logp_roll, rewards, group_size, params: O.Params,
                   row_chunk: int = 64):
        """O1..O7 on the given rows; the two vocabulary-wide steps are spread over the workers."""
        R = bits.shape[0]
        cuts = [(r0, min(R, r0 + row_chunk)) for r0 in range(0, R, row_chunk)]
        res = list(self.pool.map(_logprob_chunk, [(bits[a:b], dtype, y[a:b], valid[a:b], params.inv_temperature)
                                                  for a, b in cuts]))
        logp = np.concatenate([r[0] for r in res])
        lse = np.concatenate([r[1] for r in res])
        adv = O.group_advantages(rewards, group_size, params.adv_mode, params.eps_std)
        diag = O.diagnostics(logp, logp_roll, valid, cu_rows, adv, params)
        loss, wtilde, g = O.loss_and_row_coeff(logp, logp_roll, None, None, valid, cu_rows, adv, diag["count"],
                                               diag["alpha"], params)
        sums = list(self.pool.map(_dlogits_chunk, [(bits[a:b], dtype, lse[a:b], y[a:b], g[a:b],
                                                    params.inv_temperature) for a, b in cuts]))
        return dict(logp=logp, lse=lse, diag=diag, loss=loss, g=g, abs_sum=float(sum(sums)))
