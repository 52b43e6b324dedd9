"""CPU oracle: the quantities the two BiLD policies test (Sections 3.3, 3.4).

TEST INFRASTRUCTURE ONLY; float64; shares no code with the HIP library.
"""
from __future__ import annotations

import numpy as np


def softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - np.max(z))
    return e / np.sum(e)


def logsumexp(z: np.ndarray) -> float:
    z = np.asarray(z, dtype=np.float64)
    m = np.max(z)
    return float(m + np.log(np.sum(np.exp(z - m))))


def argmax_lowest(z: np.ndarray) -> int:
    """Greedy choice; equal maxima resolve to the lowest token id."""
    return int(np.argmax(z))        # numpy returns the first maximum


def max_prob(z: np.ndarray) -> float:
    """max_y p(y): the confidence the fallback policy tests (Section 3.3)."""
    return float(np.exp(np.max(z) - logsumexp(z)))


def nll(z: np.ndarray, token: int) -> float:
    """Cross-entropy between a hard label and the soft label softmax(z), i.e.
    -ln p(token): the rollback distance d (Section 4.1, Inference; Appendix,
    evaluation details).  Natural logarithm."""
    return float(logsumexp(z) - z[token])


def top2_gap(z: np.ndarray) -> float:
    """Difference between the two largest logits (how close the argmax is to a tie)."""
    if len(z) < 2:
        return float("inf")
    part = np.partition(np.asarray(z, dtype=np.float64), -2)
    return float(part[-1] - part[-2])


def fallback(z_small: np.ndarray, alpha_fb: float) -> bool:
    """Fallback policy (Section 3.3): hand over iff max_y p_S(y) < alpha_FB."""
    return max_prob(z_small) < alpha_fb


def rollback(z_large: np.ndarray, small_token: int, alpha_rb: float) -> bool:
    """Rollback test for one drafted token (Section 3.4, Eq. 3 with the
    cross-entropy distance): reject iff -ln p_L(small_token) > alpha_RB."""
    return nll(z_large, small_token) > alpha_rb
