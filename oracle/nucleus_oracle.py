"""fp64 CPU oracle for the nucleus (top-p) transform of a logit row.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mpv_oracle.py): only the tests,
the smoke check and the benchmark's cpu_baseline leg may import it; it shares no
code with the HIP library and never calls it.

The paper evaluates two sampling settings with nucleus sampling (Sec. 4.1: top-p 0.9
and 0.99 at temperature 1) and says nothing else about it.  The definition taken
(a reading: the paper only names the setting) is the usual one: with p = softmax(z / T),
keep the smallest set of most probable tokens whose probabilities add up to at
least top_p, drop the rest, renormalise.  Tokens with equal logits are kept or
dropped together (the set is {v : z_v >= tau} for a threshold tau that is one of
the row's values), so the result does not depend on the order of the vocabulary.
Dropped tokens get the logit -inf: every later step then sees the renormalised
distribution without knowing about the transform.  The same transform, with the
same top_p, is applied to the target and the draft rows.
"""

from __future__ import annotations

import numpy as np

from . import mpv_oracle as base


def nucleus_threshold(z, T, top_p):
    """(tau, kept, margin) for one row of logits.

    tau: the smallest kept logit; kept: how many tokens are kept;
    margin: the smallest |mass of {z >= t} - top_p| over the row's values t (how close the
    choice of tau came to going the other way)."""
    z = np.asarray(z, dtype=np.float64)
    p = base.softmax_T(z, T)
    order = np.argsort(-z, kind="stable")           # largest logit first
    zs, ps = z[order], p[order]
    upper_mass = np.cumsum(ps)                      # mass of the first i+1 tokens in that order
    # a set {z >= t} ends where the sorted value changes (equal logits stay together)
    ends = np.nonzero(np.append(zs[1:] != zs[:-1], True))[0]
    mass = upper_mass[ends]                         # mass of {z >= zs[e]} for every distinct value
    reached = np.nonzero(mass >= float(top_p))[0]
    j = int(reached[0]) if len(reached) else len(ends) - 1      # top_p = 1 and a sum that rounds below 1: everything
    return float(zs[ends[j]]), int(ends[j]) + 1, float(np.min(np.abs(mass - float(top_p))))


def nucleus_mask(z, T, top_p):
    """The row with every token outside the nucleus set to -inf (same dtype as float64 copy)."""
    z = np.asarray(z, dtype=np.float64)
    tau, _, _ = nucleus_threshold(z, T, top_p)
    return np.where(z >= tau, z, -np.inf)


def nucleus_mask_rows(z, T, top_p):
    """Rows of a [rows, V] array; returns (masked float64 [rows, V], tau [rows], kept [rows], margin [rows])."""
    z = np.asarray(z)
    out = np.empty(z.shape, dtype=np.float64)
    tau = np.empty(len(z))
    kept = np.empty(len(z), dtype=np.int64)
    margin = np.empty(len(z))
    for r in range(len(z)):
        tau[r], kept[r], margin[r] = nucleus_threshold(z[r], T, top_p)
        out[r] = np.where(np.asarray(z[r], dtype=np.float64) >= tau[r], z[r], -np.inf)
    return out, tau, kept, margin
