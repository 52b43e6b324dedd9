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


def nucleus_probs(z: np.ndarray, top_p: float) -> np.ndarray:
    """The distribution `draw` samples from: softmax(z) restricted to the nucleus and renormalised."""
    members, mass, _ = nucleus(z, top_p)
    return np.where(members, policy.softmax(z), 0.0) / mass


# Rejection-sampling acceptance: the stochastic rule of the speculative-decoding methods the paper compares BiLD
# with (Section 4.2 and the appendix comparison, Tables 3 and 4), as an alternative to the rollback test of Section 3.4.
# With q the distribution the small model drew its token x from and p the large model's distribution of the same
# position, x is kept with probability min(1, p(x) / q(x)); a refused token is replaced by a draw from the
# normalised positive part of p - q.  Both rules together return a token distributed exactly as p.
def accept(z_small: np.ndarray, z_large: np.ndarray, top_p: float, token: int, u: float):
    """(accepted, margin): keep the drafted token iff u * q(token) < p(token); margin = |u q - p|."""
    q = nucleus_probs(z_small, top_p)[token]
    p = nucleus_probs(z_large, top_p)[token]
    return bool(u * q < p), float(abs(u * q - p))


def residual_draw(z_small: np.ndarray, z_large: np.ndarray, top_p: float, u: float):
    """(token, margin): inverse-CDF draw from max(0, p - q) / sum, members walked in increasing token id."""
    r = np.maximum(nucleus_probs(z_large, top_p) - nucleus_probs(z_small, top_p), 0.0)
    total = float(np.sum(r))
    ids = np.nonzero(r > 0.0)[0]
    run = np.cumsum(r[ids])
    t = float(u) * total
    hit = np.nonzero(run > t)[0]
    j = int(hit[0]) if len(hit) else len(ids) - 1
    return int(ids[j]), float(np.min(np.abs(run - t)) / total)


class Sampler:
    """top_p and the uniform numbers of both models, indexed by the position of the token drawn; `u_accept`
    (rejection-sampling acceptance only) is indexed by the position of the drafted token under review."""

    def __init__(self, top_p: float, u_small, u_large, u_accept=None):
        assert 0.0 < top_p <= 1.0
        self.top_p = float(top_p)
        self.u = {"small": np.asarray(u_small, dtype=np.float64), "large": np.asarray(u_large, dtype=np.float64)}
        self.u_accept = None if u_accept is None else np.asarray(u_accept, dtype=np.float64)

    def pick(self, which: str, z: np.ndarray, position: int):
        return draw(z, self.top_p, self.u[which][position])

    def accept(self, z_small, z_large, token: int, position: int):
        return accept(z_small, z_large, self.top_p, token, self.u_accept[position])

    def replace(self, z_small, z_large, position: int):
        """The large model's token for a refused draft: drawn with the large model's number of that position."""
        return residual_draw(z_small, z_large, self.top_p, self.u["large"][position])
