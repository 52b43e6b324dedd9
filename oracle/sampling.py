"""CPU oracle of the sampling variant (Appendix, "BiLD with Sampling").

TEST INFRASTRUCTURE ONLY; float64; shares no code with the HIP library.

The paper's only change for sampling is that both models DRAW their token from
their distribution instead of taking the argmax, with nucleus sampling at
p = 0.8 in its table; the fallback test (max probability) and the rollback test
(cross-entropy of the drafted token) are untouched.  The paper does not spell
out the draw, so this module fixes one reading:

  nucleus   the smallest set of highest-probability tokens whose total
            probability reaches top_p; tokens tied with the least likely
            member are members too (the set is then defined by a probability
            threshold alone, not by an order among equals);
  draw      inverse-CDF sampling inside the nucleus, renormalised, walking the
            members in increasing token id: the first member whose running
            mass exceeds u * mass(nucleus).

The uniform numbers u are inputs (one per sequence position and model, from
the seeded input generators), so neither side owns a random generator.
"""
from __future__ import annotations

import numpy as np

from . import policy


def nucleus(z: np.ndarray, top_p: float):
    """(members, mass, margin): boolean membership per token id, the nucleus' total probability,
    and how far the deciding cumulative sums are from top_p (for the parity margin rule)."""
    p = policy.softmax(z)
    order = np.argsort(-p, kind="stable")
    cs = np.cumsum(p[order])
    reached = np.nonzero(cs >= top_p)[0]
    k = int(reached[0]) if len(reached) else len(p) - 1      # top_p beyond the total (rounding): everything
    members = p >= p[order[k]]
    margin = abs(cs[k] - top_p)
    if k > 0:
        margin = min(margin, abs(top_p - cs[k - 1]))
    return members, float(np.sum(p[members])), float(margin)


def draw(z: np.ndarray, top_p: float, u: float):
    """(token, margin): the drawn token id and the smaller of the nucleus margin and the distance of
    u * mass from the nearest running-mass boundary, relative to the mass."""
    members, mass, cut_margin = nucleus(z, top_p)
    p = policy.softmax(z)
    ids = np.nonzero(members)[0]
    run = np.cumsum(p[ids])
    t = float(u) * mass
    hit = np.nonzero(run > t)[0]
    j = int(hit[0]) if len(hit) else len(ids) - 1
    bounds = np.abs(run - t) / mass
    return int(ids[j]), float(min(cut_margin, float(np.min(bounds))))


class Sampler:
    """top_p and the uniform numbers of both models, indexed by the position of the token drawn."""

    def __init__(self, top_p: float, u_small, u_large):
        assert 0.0 < top_p <= 1.0
        self.top_p = float(top_p)
        self.u = {"small": np.asarray(u_small, dtype=np.float64), "large": np.asarray(u_large, dtype=np.float64)}

    def pick(self, which: str, z: np.ndarray, position: int):
        return draw(z, self.top_p, self.u[which][position])
