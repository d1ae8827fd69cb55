"""Whole-batch parity at full size: every row of a workload goes through the CPU oracle.

The oracle (oracle/ais_oracle.py, as it stands) is spread over worker processes, segment by segment: the raw bits of
a few thousand logits rows, of the GPU's gradient rows and of the one-sweep direction rows are copied from the device
into memory-backed files, the workers map them, evaluate the oracle on their rows and compare element by element;
only error statistics travel back.  Nothing here computes anything of the method: the workers call the oracle's
functions and numpy comparisons.  This module imports neither torch nor the GPU package at import time, so that the
worker processes start quickly and never touch a GPU.
"""
from __future__ import annotations

import multiprocessing as mp
import os
import shutil
import tempfile
import time
from concurrent.futures import ProcessPoolExecutor

import numpy as np

from oracle import ais_oracle as O
from tests.tolerances import dz_tolerance

_MAPPED = {}


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Raw device values -> float64, exactly.  bf16 arrives as uint16 bit patterns (the upper half of an fp32)."""
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.astype(np.float64)


def _rows(path, a, b):
    if path not in _MAPPED:
        if len(_MAPPED) > 8:
            _MAPPED.clear()
        _MAPPED[path] = np.load(path, mmap_mode="r")
    return np.asarray(_MAPPED[path][a:b])


def _hold(seconds):
    time.sleep(seconds)
    return os.getpid()


def logprob_task(args):
    """O1 on rows [a, b) of a segment file."""
    path, a, b, dtype, y, valid, inv_t = args
    return O.token_logprob(widen(_rows(path, a, b), dtype), y, valid, inv_t)


def gradient_task(args):
    """O7 on rows [a, b) of a segment, compared element by element with the GPU's dlogits (three-call path) and with
    g * s of the one-sweep path.  Returns error statistics only."""
    (zpath, dzpath, spath, a, b, dtype, lse, y, g_ref, g_gpu, inv_t, strict) = args
    z = widen(_rows(zpath, a, b), dtype)
    ref = O.dlogits_rows(z, lse, y, g_ref, inv_t)
    del z
    tol = dz_tolerance(ref, g_ref, lse, strict)
    zero_rows = g_ref == 0
    out = {"rows": b - a, "first_bad": None}
    for name, path, scale in (("dz", dzpath, None), ("gs", spath, g_gpu)):
        if path is None:
            continue
        got = widen(_rows(path, a, b), dtype)
        if scale is not None:
            got *= scale[:, None]                       # the consumer's fold: dlogits = g[n] * s[n, :]
        out[name + "_zero_rows_exact"] = bool(np.all(got[zero_rows] == 0))
        live = ~zero_rows & (np.abs(ref).max(axis=1) > 1e-30)
        out[name + "_live_rows_written"] = bool(np.all(np.abs(got[live]).max(axis=1) > 0)) if live.any() else True
        np.subtract(got, ref, out=got)
        np.abs(got, out=got)
        bad = got > tol
        out[name + "_bad"] = int(bad.sum())
        if bad.any() and out["first_bad"] is None:
            n, v = np.argwhere(bad)[0]
            out["first_bad"] = (name, int(a + n), int(v), float(got[n, v]), float(tol[n, v]), float(ref[n, v]))
        nz = ~zero_rows
        out[name + "_worst"] = float((got[nz] / np.maximum(tol[nz], 1e-300)).max()) if nz.any() else 0.0
    out["abs_sum"] = float(np.abs(ref).sum())
    return out


class Workers:
    """A pool of oracle workers plus the memory-backed files they read."""

    def __init__(self, workers=None):
        self.n = workers or min(16, len(os.sched_getaffinity(0)))
        self.pool = ProcessPoolExecutor(max_workers=self.n, mp_context=mp.get_context("spawn"))
        for _ in range(20):          # start every worker now: a fresh interpreter takes a second or more to come up
            if len(set(self.pool.map(_hold, [0.25] * self.n))) == self.n:
                break
        shm = "/dev/shm"
        self.dir = tempfile.mkdtemp(prefix="ais_full_", dir=shm if os.path.isdir(shm) and os.access(shm, os.W_OK)
                                    else tempfile.gettempdir())

    def free_bytes(self):
        return shutil.disk_usage(self.dir).free

    def put(self, name, array):
        path = os.path.join(self.dir, name + ".npy")
        np.save(path, np.ascontiguousarray(array))
        return path

    def drop(self, *paths):
        for p in paths:
            if p is not None and os.path.exists(p):
                os.unlink(p)

    def close(self):
        self.pool.shutdown()
        shutil.rmtree(self.dir, ignore_errors=True)
