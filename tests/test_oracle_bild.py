"""Pins for oracle/bild.py: the limiting cases in which Algorithm 1 must reduce
to plain greedy decoding of one model, a from-scratch certificate for general
thresholds, and agreement of the cached loop with the definition form."""
import math

import numpy as np
import pytest

import bild_inputs as bi
import oracle
from oracle import policy

INF = float("inf")


def _request(**kw):
    cfg = bi.toy_pair(**kw)
    ws, wl = bi.make_pair_weights(cfg)
    small, large = oracle.Model(cfg.small, ws), oracle.Model(cfg.large, wl)
    return cfg, oracle.Request(small, large, bi.make_source(cfg), cfg.decoder_only)


PAIR_KW = [dict(), dict(truncate=True, dtype=bi.DT_BF16),
           dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False)]


@pytest.mark.parametrize("kw", PAIR_KW)
def test_alpha_fb_zero_is_small_greedy(kw):
    # max p < 0 never holds (Section 3.3), so with the cap disabled the large model never runs
    cfg, req = _request(**kw)
    r = oracle.bild_generate(req, 0.0, 2.0, 0, cfg.max_new)
    assert r.tokens == oracle.greedy(req, "small", cfg.max_new).tokens
    assert r.stats.large_calls == 0 and all(r.from_small)
    # with the cap of the appendix the large model is consulted every n_max tokens
    r10 = oracle.bild_generate(req, 0.0, INF, 5, cfg.max_new)
    assert r10.stats.large_calls == r10.stats.fallbacks_forced > 0 and r10.stats.fallbacks_conf == 0


@pytest.mark.parametrize("kw", PAIR_KW)
@pytest.mark.parametrize("alpha_rb", [-1.0, 0.5, INF])
def test_always_fallback_is_large_greedy(kw, alpha_rb):
    cfg, req = _request(**kw)
    r = oracle.bild_generate(req, 2.0, alpha_rb, 10, cfg.max_new)      # max p < 2 always holds
    assert r.tokens == oracle.greedy(req, "large", cfg.max_new).tokens
    assert r.stats.rollbacks == 0 and not any(r.from_small)
    assert r.stats.large_calls == cfg.max_new == r.stats.rows_verified


@pytest.mark.parametrize("kw", PAIR_KW)
@pytest.mark.parametrize("alpha_fb", [0.0, 0.4])
def test_always_rollback_verified_part_is_large_greedy(kw, alpha_fb):
    cfg, req = _request(**kw)
    r = oracle.bild_generate(req, alpha_fb, -1.0, 4, cfg.max_new)
    g = oracle.greedy(req, "large", cfg.max_new).tokens
    assert r.draft_start > 0
    assert r.tokens[:r.draft_start] == g[:r.draft_start]


def test_identical_models_never_roll_back():
    cfg = bi.toy_pair(n_small=3, n_large=3)
    _, wl = bi.make_pair_weights(cfg)
    m = oracle.Model(cfg.large, wl)
    req = oracle.Request(m, m, bi.make_source(cfg), False)
    alpha_fb = 0.3
    r = oracle.bild_generate(req, alpha_fb, -math.log(alpha_fb), 10, cfg.max_new)
    assert r.tokens == oracle.greedy(req, "large", cfg.max_new).tokens
    assert r.stats.rollbacks == 0
    assert any(r.from_small) and not all(r.from_small)


def _certify(req, r, alpha_fb, alpha_rb, n_max):
    """Re-derive every committed token from the definition (no cache, whole
    prefix): a token credited to the small model is its argmax with confidence
    >= alpha_FB, and if it was reviewed the large model's -ln p of it is
    <= alpha_RB; any other token is the large model's argmax."""
    y = req.initial()
    run = 0
    for i, tok in enumerate(r.tokens):
        if r.from_small[i]:
            z = req.small.logits_full(y, req.cross_s)[-1]
            assert tok == policy.argmax_lowest(z)
            assert policy.max_prob(z) >= alpha_fb
            if i < r.draft_start:
                zl = req.large.logits_full(y, req.cross_l)[-1]
                assert policy.nll(zl, tok) <= alpha_rb
            run += 1
            assert n_max == 0 or run <= n_max
        else:
            zl = req.large.logits_full(y, req.cross_l)[-1]
            assert tok == policy.argmax_lowest(zl)
            run = 0
        y.append(tok)


@pytest.mark.parametrize("kw", PAIR_KW)
@pytest.mark.parametrize("alpha_fb,alpha_rb,n_max", [(0.3, INF, 10), (0.5, 2.0, 10), (0.2, 0.7, 3), (0.6, 1.0, 0)])
def test_certificate_for_general_thresholds(kw, alpha_fb, alpha_rb, n_max):
    cfg, req = _request(**kw)
    r = oracle.bild_generate(req, alpha_fb, alpha_rb, n_max, cfg.max_new)
    assert len(r.tokens) == cfg.max_new
    _certify(req, r, alpha_fb, alpha_rb, n_max)
    st = r.stats
    assert st.large_calls == st.fallbacks_conf + st.fallbacks_forced
    accepted = st.small_steps - st.large_calls
    assert len(r.tokens) == accepted - st.tokens_discarded + st.large_calls
    assert sum(r.from_small) == accepted - st.tokens_discarded


def test_rollbacks_do_occur_and_are_exercised():
    # thresholds chosen so that this seeded toy pair shows every branch of Algorithm 1
    cfg, req = _request(truncate=True, dtype=bi.DT_BF16)
    seen = dict(rb=0, conf=0, forced=0, accept=0)
    for fb, rb, nm in ((0.2, 0.7, 3), (0.1, 0.3, 10), (0.3, 1.0, 4)):
        r = oracle.bild_generate(req, fb, rb, nm, cfg.max_new)
        seen["rb"] += r.stats.rollbacks
        seen["conf"] += r.stats.fallbacks_conf
        seen["forced"] += r.stats.fallbacks_forced
        seen["accept"] += sum(r.from_small)
    assert all(v > 0 for v in seen.values()), seen


@pytest.mark.parametrize("kw", PAIR_KW)
def test_cached_loop_equals_definition_form(kw):
    cfg, req = _request(**kw)
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        a = oracle.bild_generate(req, fb, rb, nm, 16, cached=True)
        b = oracle.bild_generate(req, fb, rb, nm, 16, cached=False)
        assert a.tokens == b.tokens and a.from_small == b.from_small and a.stats == b.stats
        for ta, tb in zip(a.trace, b.trace):
            assert ta["kind"] == tb["kind"] and ta["tok"] == tb["tok"]
            assert abs(ta["pmax"] - tb["pmax"]) < 1e-10


def test_eos_stops_immediately_even_with_pending_drafts():
    cfg, req = _request()
    full = oracle.bild_generate(req, 0.0, 2.0, 0, cfg.max_new)
    eos = full.tokens[5]
    first = full.tokens.index(eos)
    r = oracle.bild_generate(req, 0.0, 2.0, 0, cfg.max_new, eos=eos)
    assert r.tokens == full.tokens[:first + 1]
    assert r.stats.large_calls == 0                    # trailing drafts stay unreviewed


def test_rollback_position_and_refill():
    # hand-checkable: force one review over a block and compare with per-position definition
    cfg, req = _request(truncate=True, dtype=bi.DT_BF16)
    r = oracle.bild_generate(req, 0.0, 0.5, 6, 20)
    for rec in r.trace:
        if rec["kind"] != "large":
            continue
        n, rr = rec["n"], rec["r"]
        assert 0 <= rr <= n
        assert all(v <= 0.5 for v in rec["nll"][:rr])          # every draft before r passed
        if rr < n:
            assert rec["nll"][rr] > 0.5                        # the first failing draft is r
            assert len(rec["nll"]) == rr + 1                   # nothing after it is judged
    assert r.stats.rollbacks > 0


def test_pair_must_share_vocabulary():
    cfg = bi.toy_pair()
    ws, wl = bi.make_pair_weights(cfg)
    from dataclasses import replace
    bad = replace(cfg.small, vocab=cfg.small.vocab - 1)
    ws_bad = dict(ws)
    ws_bad["emb"] = ws["emb"][:-1]
    with pytest.raises(AssertionError):
        oracle.Request(oracle.Model(bad, ws_bad), oracle.Model(cfg.large, wl), [1, 2], False)
