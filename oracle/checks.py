"""Validity of a top-k selection that differs from the oracle's (TEST INFRASTRUCTURE ONLY).

The task's bar: span indices match the oracle bit-exactly, except on rows whose oracle k-th and
(k+1)-th candidate scores differ by less than a margin (1e-3, raw score units of eq. (2)).  On such
a row several selections are acceptable, but not any selection: with s_(k) the oracle's k-th
largest fp64 score, every span a correct implementation may have picked scores at least
s_(k) - margin, and every span it may have dropped scores at most s_(k) + margin (its own score
arithmetic is allowed to be off by less than the margin, nothing else is).  The functions below
check exactly that, plus the shape of the row (count, order, range, padding).
"""
from __future__ import annotations

import numpy as np


def selection_problems(scores, got, k: int, margin: float, ascending: bool = True):
    """Why `got` is not an acceptable top-k selection of `scores`; [] if it is acceptable.

    scores : fp64 scores of the c candidates (candidate number = position in the array)
    got    : the row as reported: candidate numbers, -1 in empty slots
    k      : slots per row; min(k, c) candidates must be listed
    ascending : the listed candidates must come in ascending candidate number (the grid's span
             order; for the paper's geometry candidate numbers are stride indices, nearest first)
    """
    scores = np.asarray(scores, dtype=np.float64)
    c = scores.shape[0]
    got = [int(j) for j in got]
    sel = [j for j in got if j >= 0]
    kk = min(k, c)
    out = []
    if len(got) != k:
        out.append(f"row has {len(got)} slots, expected {k}")
    if len(sel) != kk:
        out.append(f"{len(sel)} candidates listed, expected min(k, c) = {kk}")
    if got[:len(sel)] != sel or any(j != -1 for j in got[len(sel):]):
        out.append("empty slots must be -1 and come last")
    if any(j >= c for j in sel):
        out.append(f"candidate out of range [0, {c})")
        return out
    if len(set(sel)) != len(sel):
        out.append("a candidate is listed twice")
    if ascending and sel != sorted(sel):
        out.append("candidates are not in ascending order")
    if kk == 0 or out:
        return out
    s_k = np.sort(scores)[::-1][kk - 1]          # the oracle's k-th largest score
    lowest_in = float(np.min(scores[sel]))
    if lowest_in < s_k - margin:
        out.append(f"selected a candidate scoring {lowest_in:.6f}, more than {margin} below the k-th score {s_k:.6f}")
    rest = np.ones(c, dtype=bool)
    rest[sel] = False
    if rest.any():
        highest_out = float(np.max(scores[rest]))
        if highest_out > s_k + margin:
            out.append(f"dropped a candidate scoring {highest_out:.6f}, more than {margin} above the k-th score {s_k:.6f}")
    return out
