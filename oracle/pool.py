"""Runs the oracle over row chunks in worker processes.  TEST INFRASTRUCTURE ONLY (CPU-baseline timing).

The workers call oracle/ais_oracle.py as it stands; this file only moves data: it widens raw bf16 bit
patterns to float64 exactly and splits the rows.  The logits are placed once, before anything is timed, in a
memory-backed file that every worker maps read-only (the CPU's counterpart of inputs that are resident in device
memory); a task then names a row range instead of carrying the rows through a pipe.  It imports neither torch nor
the GPU package, so that worker processes start quickly and never touch a GPU.
"""
from __future__ import annotations

import os
import tempfile
import time
from concurrent.futures import ProcessPoolExecutor
import multiprocessing as mp

import numpy as np

from oracle import ais_oracle as O


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Raw logits -> float64, exactly.  bf16 arrives as uint16 bit patterns (the upper half of an fp32)."""
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.astype(np.float64)


_MAPPED = {}


def _rows(path, a, b):
    """Rows [a, b) of the shared logits file, mapped once per worker."""
    if path not in _MAPPED:
        _MAPPED.clear()
        _MAPPED[path] = np.load(path, mmap_mode="r")
    return np.asarray(_MAPPED[path][a:b])


def _logprob_chunk(args):
    path, a, b, dtype, y, valid, inv_t = args
    return O.token_logprob(widen(_rows(path, a, b), dtype), y, valid, inv_t)


def _dlogits_chunk(args):
    path, a, b, dtype, lse, y, g, inv_t = args
    dz = O.dlogits_rows(widen(_rows(path, a, b), dtype), lse, y, g, inv_t)
    return float(np.abs(dz).sum())          # the gradient itself stays in the worker: only a checksum returns


def _hold(seconds):
    time.sleep(seconds)                     # keeps this worker busy so that the executor has to start the next one
    return os.getpid()


class OraclePool:
    def __init__(self, workers: int):
        self.workers = workers
        self.path = None
        self.pool = ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))
        # start every worker before anything is timed: the executor starts them on demand, and a fresh interpreter
        # takes a second or more to come up
        for _ in range(20):
            if len(set(self.pool.map(_hold, [0.25] * workers))) == workers:
                break

    def close(self):
        self.pool.shutdown()
        self.unshare()

    def share(self, bits: np.ndarray) -> str:
        """Writes the raw logits to a file in memory-backed storage (not timed) and returns its path."""
        self.unshare()
        where = "/dev/shm" if os.path.isdir("/dev/shm") and os.access("/dev/shm", os.W_OK) else tempfile.gettempdir()
        fd, self.path = tempfile.mkstemp(prefix="ais_oracle_", suffix=".npy", dir=where)
        with os.fdopen(fd, "wb") as f:
            np.save(f, np.ascontiguousarray(bits))
        return self.path

    def unshare(self):
        if self.path is not None and os.path.exists(self.path):
            os.unlink(self.path)
        self.path = None

    def whole_path(self, path, n_rows, dtype, y, valid, cu_rows, logp_roll, rewards, group_size, params: O.Params,
                   row_chunk: int = 64):
        """O1..O7 on the rows of the shared file; the two vocabulary-wide steps are spread over the workers."""
        R = n_rows
        cuts = [(r0, min(R, r0 + row_chunk)) for r0 in range(0, R, row_chunk)]
        res = list(self.pool.map(_logprob_chunk, [(path, a, b, dtype, y[a:b], valid[a:b], params.inv_temperature)
                                                  for a, b in cuts]))
        logp = np.concatenate([r[0] for r in res])
        lse = np.concatenate([r[1] for r in res])
        adv = O.group_advantages(rewards, group_size, params.adv_mode, params.eps_std)
        diag = O.diagnostics(logp, logp_roll, valid, cu_rows, adv, params)
        loss, wtilde, g = O.loss_and_row_coeff(logp, logp_roll, None, None, valid, cu_rows, adv, diag["count"],
                                               diag["alpha"], params)
        sums = list(self.pool.map(_dlogits_chunk, [(path, a, b, dtype, lse[a:b], y[a:b], g[a:b],
                                                    params.inv_temperature) for a, b in cuts]))
        return dict(logp=logp, lse=lse, diag=diag, loss=loss, g=g, abs_sum=float(sum(sums)))
