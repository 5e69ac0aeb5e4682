"""Kernel-selection formula of the paper (Sec. 4.2.3, Eq. 1) -- TEST INFRASTRUCTURE ONLY.

    n         = ceil(seq_len / 16)
    threshold = valid16 / n^2  -  tau / (log2 n)^2,      tau = 1.2

valid16 = number of non-empty 16 x 16 tiles of the mask (load_row_ptr[n] of the
block format at tile size 16).  The row-wise kernel is chosen iff threshold < 0.
For n = 1 the logarithm is 0 and the formula is undefined; this build reads that
case as "row-wise" (one tile, nothing to block).

The paper states the formula for as many queries as keys.  For a mask with Sq
queries and Sk keys this build reads n^2 as the number of 16 x 16 tiles of the mask,
ceil(Sq/16) * ceil(Sk/16), and takes n = ceil(Sk/16) in the logarithm.
"""
from __future__ import annotations

import math

import numpy as np

TAU = 1.2


def valid16(M: np.ndarray) -> int:
    Sq, Sk = M.shape
    nq, nk = -(-Sq // 16), -(-Sk // 16)
    P = np.zeros((nq * 16, nk * 16), dtype=np.uint8)
    P[:Sq, :Sk] = (M != 0)
    return int((P.reshape(nq, 16, nk, 16).sum(axis=(1, 3)) > 0).sum())


def threshold(valid: int, S: int, tau: float = TAU, Sk: int | None = None) -> float:
    nq = -(-S // 16)
    n = nq if Sk is None else -(-Sk // 16)
    if n <= 1:
        return -math.inf
    return valid / float(nq * n) - tau / (math.log2(n) ** 2)


def choose(valid: int, S: int, tau: float = TAU) -> str:
    return "row" if threshold(valid, S, tau) < 0 else "block"
