"""Pins for oracle/sampling.py (Appendix, "BiLD with Sampling"): a worked example, brute force on tiny
vocabularies, the closed-form draw frequencies, the library routine the draw reduces to at top_p = 1,
and the greedy limit of the whole loop."""
import itertools

import numpy as np
import pytest

import bild_inputs as bi
import oracle
from oracle import sampling


def _logits(p):
    return np.log(np.asarray(p, dtype=np.float64)) + 3.25      # any shift: softmax is shift-invariant


def test_worked_example_of_the_nucleus():
    z = _logits([0.05, 0.5, 0.15, 0.3])
    members, mass, _ = sampling.nucleus(z, 0.79)
    assert members.tolist() == [False, True, False, True] and abs(mass - 0.8) < 1e-12
    members, mass, _ = sampling.nucleus(z, 0.81)
    assert members.tolist() == [False, True, True, True] and abs(mass - 0.95) < 1e-12
    members, mass, _ = sampling.nucleus(z, 0.4)
    assert members.tolist() == [False, True, False, False]
    members, mass, _ = sampling.nucleus(z, 1.0)
    assert members.all() and abs(mass - 1.0) < 1e-12


def test_ties_with_the_last_member_are_members():
    z = _logits([0.3, 0.2, 0.2, 0.2, 0.1])
    members, mass, _ = sampling.nucleus(z, 0.45)              # 0.3 + one of the 0.2s reaches 0.45
    assert members.tolist() == [True, True, True, True, False] and abs(mass - 0.9) < 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_nucleus_is_the_smallest_set_reaching_top_p(seed):
    rng = np.random.default_rng(seed)
    v = 7
    p = rng.dirichlet(np.ones(v) * 0.7)
    z = _logits(p)
    for top_p in (0.2, 0.5, 0.8, 0.95):
        members, mass, margin = sampling.nucleus(z, top_p)
        if margin < 1e-9:
            continue
        best = None                                            # brute force over all subsets
        for k in range(1, v + 1):
            sets = [c for c in itertools.combinations(range(v), k) if p[list(c)].sum() >= top_p]
            if sets:
                best = max(sets, key=lambda c: p[list(c)].sum())
                break
        assert sorted(np.nonzero(members)[0].tolist()) == sorted(best)
        assert abs(mass - p[list(best)].sum()) < 1e-12


def test_draw_frequencies_match_the_renormalised_probabilities():
    p = np.array([0.02, 0.4, 0.08, 0.25, 0.05, 0.2])
    z = _logits(p)
    top_p = 0.8                                                # nucleus {1, 3, 5}: mass 0.85
    n = 20000
    us = (np.arange(n) + 0.5) / n
    toks = np.array([sampling.draw(z, top_p, u)[0] for u in us])
    assert set(toks.tolist()) == {1, 3, 5}
    for t in (1, 3, 5):
        assert abs(np.mean(toks == t) - p[t] / 0.85) < 2.0 / n
    assert np.all(np.diff(toks) >= 0)                          # members are walked in increasing id


@pytest.mark.parametrize("seed", range(4))
def test_top_p_one_is_inverse_cdf_sampling(seed):
    rng = np.random.default_rng(seed)
    z = rng.normal(size=50) * 2
    p = oracle.policy.softmax(z)
    cdf = np.cumsum(p)
    for u in rng.random(200):
        tok, margin = sampling.draw(z, 1.0, u)
        if margin > 1e-9:
            assert tok == int(np.searchsorted(cdf, u, side="right"))


def test_tiny_top_p_draws_the_argmax():
    rng = np.random.default_rng(1)
    for _ in range(20):
        z = rng.normal(size=40) * 3
        for u in (0.0, 0.37, 0.999):
            assert sampling.draw(z, 1e-6, u)[0] == int(np.argmax(z))


def _request(**kw):
    cfg = bi.toy_pair(**kw)
    ws, wl = bi.make_pair_weights(cfg)
    small, large = oracle.Model(cfg.small, ws), oracle.Model(cfg.large, wl)
    return cfg, oracle.Request(small, large, bi.make_source(cfg), cfg.decoder_only)


def _sampler(cfg, top_p, n):
    return oracle.Sampler(top_p, bi.make_uniforms(n, cfg.input_seed, 0), bi.make_uniforms(n, cfg.input_seed, 1))


@pytest.mark.parametrize("kw", [dict(), dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False)])
def test_sampling_loop_reduces_to_greedy_and_follows_its_definition(kw):
    cfg, req = _request(**kw)
    n = len(req.initial()) + cfg.max_new + 2
    # a nucleus that only ever holds the most likely token: Algorithm 1 with argmax
    ref = oracle.bild_generate(req, 0.5, 2.0, 10, cfg.max_new)
    got = oracle.bild_generate(req, 0.5, 2.0, 10, cfg.max_new, sampler=_sampler(cfg, 1e-9, n))
    assert got.tokens == ref.tokens and got.stats == ref.stats
    # a real nucleus: the cached loop equals the definition form, every token is a member of the nucleus of the
    # distribution that produced it, and the counters still add up
    smp = _sampler(cfg, 0.8, n)
    a = oracle.bild_generate(req, 0.5, 2.0, 10, cfg.max_new, sampler=smp, keep_logits=True)
    b = oracle.bild_generate(req, 0.5, 2.0, 10, cfg.max_new, sampler=smp, cached=False)
    assert a.tokens == b.tokens and a.stats == b.stats
    assert a.tokens != ref.tokens                              # the draws do change the sequence
    for rec in a.trace:
        z = rec["z"] if rec["kind"] == "small" else rec["z"][rec["r"]]
        members, _, _ = sampling.nucleus(z, 0.8)
        assert members[rec["tok"]]
    assert a.stats.rows_verified == sum(r["n"] + 1 for r in a.trace if r["kind"] == "large")
    # large-only sampling uses the large model's numbers alone
    g = oracle.greedy(req, "large", 8, sampler=smp)
    n0 = len(req.initial())
    y = req.initial()
    for i, tok in enumerate(g.tokens):
        z = req.large.logits_full(y, req.cross_l)[-1]
        assert tok == sampling.draw(z, 0.8, smp.u["large"][n0 + i])[0]
        y.append(tok)


# ---- rejection-sampling acceptance (Section 4.2 / appendix comparison: the rule of the speculative-decoding methods) ----

def test_worked_example_of_the_rejection_rule():
    # q = (0.5, 0.3, 0.2), p = (0.2, 0.5, 0.3): token 0 is kept with probability 0.2 / 0.5, tokens 1 and 2 always;
    # the positive part of p - q is (0, 0.2, 0.1), so a refused draft becomes token 1 with probability 2/3
    zq, zp = _logits([0.5, 0.3, 0.2]), _logits([0.2, 0.5, 0.3])
    assert sampling.accept(zq, zp, 1.0, 0, 0.39)[0] and not sampling.accept(zq, zp, 1.0, 0, 0.41)[0]
    assert abs(sampling.accept(zq, zp, 1.0, 0, 0.39)[1] - 0.005) < 1e-12          # |0.39 * 0.5 - 0.2|
    for u in (0.0, 0.5, 0.999999):
        assert sampling.accept(zq, zp, 1.0, 1, u)[0] and sampling.accept(zq, zp, 1.0, 2, u)[0]
    assert [sampling.residual_draw(zq, zp, 1.0, u)[0] for u in (0.0, 0.6, 0.66, 0.67, 0.99)] == [1, 1, 1, 2, 2]


def test_rejection_rule_with_a_nucleus_uses_the_renormalised_distributions():
    # top_p 0.75: the small model's nucleus is {0, 1} -> q = (0.625, 0.375, 0); the large model's is {1, 2} -> p = (0, 0.625, 0.375)
    zq, zp = _logits([0.5, 0.3, 0.2]), _logits([0.2, 0.5, 0.3])
    assert np.allclose(sampling.nucleus_probs(zq, 0.75), [0.625, 0.375, 0.0])
    assert np.allclose(sampling.nucleus_probs(zp, 0.75), [0.0, 0.625, 0.375])
    assert not sampling.accept(zq, zp, 0.75, 0, 0.0)[0]                            # p(0) = 0: never kept, not even at u = 0
    assert sampling.accept(zq, zp, 0.75, 1, 0.999)[0]
    # positive part of p - q = (0, 0.25, 0.375): token 1 up to u = 0.4
    assert [sampling.residual_draw(zq, zp, 0.75, u)[0] for u in (0.0, 0.39, 0.41, 0.99)] == [1, 1, 2, 2]


@pytest.mark.parametrize("seed,top_p", [(0, 1.0), (1, 1.0), (2, 0.8), (3, 0.6)])
def test_rejection_rule_returns_a_token_distributed_as_the_large_model(seed, top_p):
    """The property the rule exists for: draft from q, keep or replace, and the result follows p exactly.  Measured
    through the oracle's own functions on fine grids of the three uniform numbers (draft, acceptance, replacement)."""
    rng = np.random.default_rng(seed)
    v, n = 6, 4000
    zq, zp = rng.normal(size=v) * 1.5, rng.normal(size=v) * 1.5
    grid = (np.arange(n) + 0.5) / n
    q_hat = np.bincount([sampling.draw(zq, top_p, u)[0] for u in grid], minlength=v) / n
    out = np.zeros(v)
    repl = np.bincount([sampling.residual_draw(zq, zp, top_p, u)[0] for u in grid], minlength=v) / n
    for x in range(v):
        if q_hat[x] == 0:
            continue
        keep = np.mean([sampling.accept(zq, zp, top_p, x, u)[0] for u in grid])
        out[x] += q_hat[x] * keep
        out += q_hat[x] * (1.0 - keep) * repl
    assert np.max(np.abs(out - sampling.nucleus_probs(zp, top_p))) < 4.0 / n * v


def test_identical_distributions_are_never_refused():
    rng = np.random.default_rng(5)
    z = rng.normal(size=50) * 2
    for top_p in (0.5, 0.9, 1.0):
        members, _, _ = sampling.nucleus(z, top_p)
        for tok in np.nonzero(members)[0]:
            assert sampling.accept(z, z, top_p, int(tok), 0.999999)[0]


def _rejection_sampler(cfg, top_p, n):
    return oracle.Sampler(top_p, bi.make_uniforms(n, cfg.input_seed, 0), bi.make_uniforms(n, cfg.input_seed, 1),
                          bi.make_uniforms(n, cfg.input_seed, 2))


@pytest.mark.parametrize("kw", [dict(), dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False)])
def test_rejection_acceptance_in_the_loop(kw):
    cfg, req = _request(**kw)
    n0 = len(req.initial())
    n = n0 + cfg.max_new + 2
    smp = _rejection_sampler(cfg, 0.9, n)
    # fixed window of 4 (alpha_FB = 0): the cached loop equals the definition form
    a = oracle.bild_generate(req, 0.0, 0.0, 4, cfg.max_new, sampler=smp, acceptance="rejection", keep_logits=True)
    b = oracle.bild_generate(req, 0.0, 0.0, 4, cfg.max_new, sampler=smp, acceptance="rejection", cached=False)
    assert a.tokens == b.tokens and a.stats == b.stats
    assert a.stats.fallbacks_conf == 0 and a.stats.large_calls > 0
    # every review is the rule applied by hand to the distributions of the definition: kept drafts pass it, the first
    # refused one fails it and is replaced by the draw from the positive part of p_L - p_S
    y = req.initial()
    for rec in a.trace:
        if rec["kind"] == "small":
            if not rec["fallback"]:
                y.append(rec["tok"])
            continue
        ds, nd, r = rec["draft_start"], rec["n"], rec["r"]
        assert len(y) == ds + nd
        for i in range(min(r + 1, nd)):
            zs = req.small.logits_full(y[:ds + i], req.cross_s)[-1]
            zl = req.large.logits_full(y[:ds + i], req.cross_l)[-1]
            ok = sampling.accept(zs, zl, 0.9, y[ds + i], smp.u_accept[ds + i])[0]
            assert ok == (i < r)
        zl = req.large.logits_full(y[:ds + r], req.cross_l)[-1]
        if r < nd:
            zs = req.small.logits_full(y[:ds + r], req.cross_s)[-1]
            assert rec["tok"] == sampling.residual_draw(zs, zl, 0.9, smp.u["large"][ds + r])[0]
        else:
            assert rec["tok"] == sampling.draw(zl, 0.9, smp.u["large"][ds + r])[0]
        y = y[:ds + r] + [rec["tok"]]
    assert y[n0:] == a.tokens
    assert a.stats.rollbacks > 0                               # the toy pair does get refused now and then
    # a pair of identical models never refuses a draft
    same = oracle.Request(req.large, req.large, bi.make_source(cfg), cfg.decoder_only)
    c = oracle.bild_generate(same, 0.0, 0.0, 4, cfg.max_new, sampler=smp, acceptance="rejection")
    assert c.stats.rollbacks == 0 and c.stats.tokens_discarded == 0 and c.stats.large_calls > 0
