"""CPU oracle of temperature / nucleus (top-p) sampling (test infrastructure only; nothing outside tests/ may import it).

App. C of the paper lists temperature and top-p among the generation parameters (its runs use temperature 0, which is
the greedy argmax).  The definition taken is the one stated in include/www.h: softmax of logits / T; the nucleus is the
set {i : p_i >= tau} for the largest tau among the probabilities whose members' mass reaches top_p (equal probabilities
are all in or all out); the token is the first member, in index order, whose running mass exceeds u times the nucleus
mass.  Plain numpy in fp64, written out step by step."""
from __future__ import annotations

import numpy as np


def nucleus(logits_row, temperature: float, top_p: float):
    """-> (e, member mask, tau): unnormalised probabilities e_i = exp(z_i - max z), z = logits / T"""
    z = np.asarray(logits_row, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    need = float(top_p) * e.sum()
    values = np.unique(e)[::-1]                      # distinct values, largest first
    tau = values[-1]
    for v in values:                                 # the largest value whose members already reach the mass wins
        if e[e >= v].sum() >= need:
            tau = v
            break
    return e, e >= tau, tau


def nucleus_fast(logits_row, temperature: float, top_p: float):
    """The same set for long rows: cumulative mass over the sorted values instead of one pass per distinct value."""
    z = np.asarray(logits_row, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    order = np.argsort(-e, kind="stable")
    es = e[order]
    cum = np.cumsum(es)
    need = float(top_p) * cum[-1]                    # the total in the same summation order as the masses below, so that
                                                     # top_p = 1 is reached by the whole vocabulary and by nothing less
    # mass of {e >= es[k]} = cum at the LAST position holding the value es[k]
    last_of_value = np.searchsorted(-es, -es, side="right") - 1
    mass = cum[last_of_value]
    k = int(np.argmax(mass >= need))                 # first (largest value) that reaches the mass
    tau = es[k]
    return e, e >= tau, tau


def sample(logits_row, temperature: float, top_p: float, u: float, fast: bool = True):
    """-> (token, e, mask, running mass through each index over the members, target)"""
    e, mask, _ = (nucleus_fast if fast else nucleus)(logits_row, temperature, top_p)
    run = np.cumsum(np.where(mask, e, 0.0))
    target = float(u) * run[-1]
    hit = np.flatnonzero(mask & (run > target))
    token = int(hit[0]) if len(hit) else int(np.flatnonzero(mask)[-1])
    return token, e, mask, run, target
