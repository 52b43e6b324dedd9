"""CPU oracle: Algorithm 1 (Big Little Decoder) and plain greedy decoding.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

BiLD's output is defined by its procedure, so this file is the procedure in the
order Algorithm 1 gives it, with these readings where the paper leaves a choice
(each is a parameter or a comment here, and is listed in the design notes):
  * fallback iff max p_S < alpha_FB, strictly (Section 3.3's statement of the
    policy; Algorithm 1's `>` differs from it only at exact equality);
  * the drafted token at position q is judged by the large model's distribution
    conditioned on y[:q] - the distribution that would have produced it - and a
    rollback keeps y[:q] and refills position q with the large model's token;
  * d = -ln p_L(token the small model emitted), natural log, rollback iff d > alpha_RB;
  * only tokens drafted since the large model last ran are judged;
  * the small model's low-confidence token that triggered the fallback is
    discarded, never judged;
  * `n_max` consecutive small-model tokens force a fallback (the appendix caps
    the small model's run at 10); 0 disables the cap;
  * the loop stops as soon as the last token is <eos> or `max_new` tokens exist,
    even if the trailing tokens are unreviewed drafts;
  * sample(.) is the argmax, ties to the lowest id (greedy decoding is what the
    paper's main results use).

`cached=False` evaluates every distribution from its definition (whole prefix,
no cache, one position at a time); `cached=True` uses KV caches and one T-row
pass of the large model per review.  Tests require identical output.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import policy
from .model import DecoderCache, Model


@dataclass
class Stats:
    small_steps: int = 0
    large_calls: int = 0
    rows_verified: int = 0
    fallbacks_conf: int = 0
    fallbacks_forced: int = 0
    rollbacks: int = 0
    tokens_discarded: int = 0


@dataclass
class Result:
    tokens: list                 # generated tokens only (without <s> / the prompt)
    from_small: list             # per generated token: True if the small model's
    trace: list                  # one record per model invocation, in order
    stats: Stats
    draft_start: int             # index into tokens of the first unreviewed draft


class Request:
    """Source-side state of one request for a (small, large) pair: encoder
    outputs and cross-attention K/V.  A small model without an encoder of its
    own attends to the large model's encoder output (early-exit arrangement,
    Section 4.4)."""

    def __init__(self, small: Model, large: Model, src, decoder_only: bool):
        assert small.s.vocab == large.s.vocab, "the pair must share a vocabulary (Section 3.5.1)"
        self.small, self.large, self.decoder_only = small, large, decoder_only
        self.src = [int(t) for t in src]
        if decoder_only:
            self.cross_s, self.cross_l = [], []
        else:
            enc_l = large.encode(self.src)
            self.cross_l = large.cross_kv(enc_l)
            enc_s = small.encode(self.src) if small.s.n_enc else enc_l
            self.cross_s = small.cross_kv(enc_s)

    def initial(self) -> list:
        return list(self.src) if self.decoder_only else [self.large.s.bos]

    def cross(self, which: str):
        return self.cross_s if which == "small" else self.cross_l

    def model(self, which: str) -> Model:
        return self.small if which == "small" else self.large


class _Definition:
    """p(. | y[:k]) from the no-cache forward."""

    def __init__(self, req: Request, which: str):
        self.m, self.cross = req.model(which), req.cross(which)

    def next_logits(self, y) -> np.ndarray:
        return self.m.logits_full(y, self.cross)[-1]

    def block_logits(self, y, first: int) -> np.ndarray:
        """Rows first-1 .. len(y)-1: distributions of positions first .. len(y)."""
        return np.stack([self.m.logits_full(y[:q], self.cross)[-1] for q in range(first, len(y) + 1)])

    def keep(self, length: int) -> None:
        pass


class _Cached:
    def __init__(self, req: Request, which: str, capacity: int):
        self.c = DecoderCache(req.model(which), req.cross(which), capacity)

    def next_logits(self, y) -> np.ndarray:
        return self.c.step(y[self.c.length:])[-1]

    def block_logits(self, y, first: int) -> np.ndarray:
        assert self.c.length <= first - 1
        z = self.c.step(y[self.c.length:])
        return z[-(len(y) - first + 1):]

    def keep(self, length: int) -> None:
        self.c.truncate(min(self.c.length, length))


def greedy(req: Request, which: str, max_new: int, eos: int = -1, cached: bool = True,
           keep_logits: bool = False, sampler=None) -> Result:
    """Vanilla inference: one model alone, autoregressive argmax (the baseline
    every speedup in the paper is normalised to when which == 'large'); with a
    sampler, each token is drawn instead (Appendix, BiLD with Sampling)."""
    y = req.initial()
    n0 = len(y)
    ev = _Cached(req, which, n0 + max_new + 1) if cached else _Definition(req, which)
    trace = []
    while len(y) - n0 < max_new and not (len(y) > n0 and y[-1] == eos):
        z = ev.next_logits(y)
        tok, dm = (policy.argmax_lowest(z), None) if sampler is None else sampler.pick(which, z, len(y))
        trace.append(dict(kind=which, pos=len(y), tok=tok, pmax=policy.max_prob(z), gap=policy.top2_gap(z),
                          draw_margin=dm))
        if keep_logits:
            trace[-1]["z"] = z
        y.append(tok)
    return Result(y[n0:], [which == "small"] * (len(y) - n0), trace, Stats(), len(y) - n0)


def bild_generate(req: Request, alpha_fb: float, alpha_rb: float, n_max: int, max_new: int,
                  eos: int = -1, cached: bool = True, keep_logits: bool = False, sampler=None,
                  acceptance: str = "threshold") -> Result:
    """Algorithm 1.  keep_logits stores every evaluated logit row in the trace
    (for element-wise comparison against another implementation).  With a
    sampler (oracle.sampling.Sampler) both models draw their tokens instead of
    taking the argmax; the two policies are unchanged (Appendix, BiLD with
    Sampling).

    acceptance="rejection" (needs a sampler with u_accept) replaces the rollback
    test by the rejection-sampling rule of the speculative-decoding methods the
    paper compares with (Section 4.2; appendix comparison): the first drafted
    token that the rule refuses is where the review stops, and its replacement is
    drawn from the normalised positive part of p_L - p_S; alpha_rb is not used.
    With alpha_fb = 0 and n_max = the window this is those methods' fixed-window
    procedure."""
    assert acceptance in ("threshold", "rejection")
    assert acceptance == "threshold" or (sampler is not None and sampler.u_accept is not None)
    z_small_at = {}                      # rejection acceptance: the small model's logits at each pending draft position
    y = req.initial()
    n0 = len(y)
    src_small = [False] * n0
    cap = n0 + max_new + 1
    small = _Cached(req, "small", cap) if cached else _Definition(req, "small")
    large = _Cached(req, "large", cap) if cached else _Definition(req, "large")
    draft_start = len(y)                 # y[draft_start:] are drafts the large model has not reviewed
    st, trace = Stats(), []
    while len(y) - n0 < max_new and not (len(y) > n0 and y[-1] == eos):
        z_s = small.next_logits(y)
        st.small_steps += 1
        n = len(y) - draft_start
        pmax = policy.max_prob(z_s)
        low_conf = policy.fallback(z_s, alpha_fb)
        forced = n_max > 0 and n >= n_max
        tok_s, dm_s = (policy.argmax_lowest(z_s), None) if sampler is None else sampler.pick("small", z_s, len(y))
        trace.append(dict(kind="small", pos=len(y), tok=tok_s, pmax=pmax, gap=policy.top2_gap(z_s),
                          fallback=bool(low_conf or forced), forced=bool(forced and not low_conf),
                          draw_margin=dm_s))
        if keep_logits:
            trace[-1]["z"] = z_s
        if not (low_conf or forced):
            if acceptance == "rejection":
                z_small_at[len(y)] = z_s
            y.append(tok_s)
            src_small.append(True)
            continue
        st.fallbacks_conf += int(low_conf)
        st.fallbacks_forced += int(forced and not low_conf)
        # the large model reviews the n pending drafts and predicts one more token
        z_l = large.block_logits(y, draft_start)          # row i: distribution of position draft_start+i
        st.large_calls += 1
        st.rows_verified += n + 1
        nlls = []
        accept_margins = []
        r = n
        for i in range(n):
            q = draft_start + i
            nlls.append(policy.nll(z_l[i], y[q]))
            if acceptance == "rejection":
                ok, am = sampler.accept(z_small_at[q], z_l[i], y[q], q)
                accept_margins.append(am)
                refused = not ok
            else:
                refused = policy.rollback(z_l[i], y[q], alpha_rb)
            if refused:
                r = i
                break
        if sampler is None:
            tok_l, dm_l = policy.argmax_lowest(z_l[r]), None
        elif acceptance == "rejection" and r < n:
            tok_l, dm_l = sampler.replace(z_small_at[draft_start + r], z_l[r], draft_start + r)
        else:
            tok_l, dm_l = sampler.pick("large", z_l[r], draft_start + r)
        trace.append(dict(kind="large", draft_start=draft_start, n=n, r=r, tok=tok_l, nll=nlls,
                          gaps=[policy.top2_gap(z_l[i]) for i in range(r + 1)],
                          pmax=policy.max_prob(z_l[r]), draw_margin=dm_l, accept_margins=accept_margins))
        z_small_at.clear()
        if keep_logits:
            trace[-1]["z"] = z_l
        if r < n:
            st.rollbacks += 1
            st.tokens_discarded += n - r
        y = y[:draft_start + r] + [tok_l]
        src_small = src_small[:draft_start + r] + [False]
        draft_start = len(y)
        large.keep(len(y) - 1)
        small.keep(len(y) - 1)
    return Result(y[n0:], src_small[n0:], trace, st, draft_start - n0)
