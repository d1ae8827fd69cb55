"""The parity bar in numbers (numpy only, so that worker processes can import it without torch).

  * log-prob, lse        |gpu - oracle| <= 2e-3 absolute
  * diagnostics, alpha, loss, w_tilde: relative 1e-3 (floors are documented in tests/parity.py)
  * dlogits              |gpu - oracle| <= 1e-2 |ref| + 1e-2 * 2^-8 * max_v |ref[n, :]|
    (one bf16 half-ulp of the row maximum as absolute cushion).  Outside strict mode, i.e. for random and
    adversarial inputs only, two absolute terms are added: 2^-126 (fp32 flushes what an fp64 oracle still resolves)
    and the oracle's own cancellation floor |g_n| * 8 * 2^-52 * max(1, |lse_n|).
"""
import numpy as np

LOGP_ATOL = 2e-3
REL = 1e-3
DZ_REL = 1e-2
DZ_CUSHION = 1e-2 * 2.0 ** -8
DZ_TINY = 2.0 ** -126
DZ_ORACLE_ULPS = 8 * 2.0 ** -52


def oracle_floor(coeff, lse):
    """Absolute rounding floor of the fp64 oracle's gradient rows, per row (column vector)."""
    return (np.abs(coeff) * DZ_ORACLE_ULPS * np.maximum(1.0, np.abs(lse)))[:, None]


def dz_tolerance(ref_dz, g, lse, strict, g_slack=None, inv_t=1.0):
    """Element-wise bound on |gpu - oracle| for a block of gradient rows."""
    rowmax = np.abs(ref_dz).max(axis=1, keepdims=True)
    tol = DZ_REL * np.abs(ref_dz) + DZ_CUSHION * rowmax
    if not strict:
        tol = tol + DZ_TINY + oracle_floor(g, lse)
        if g_slack is not None:
            tol = tol + (g_slack * inv_t)[:, None]          # what the observed log-prob error may do to g_n
    return tol
