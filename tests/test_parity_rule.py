"""The margin rule of the GPU comparisons, exercised on the oracle alone (no GPU): a token difference is
excused only by a marginal oracle decision about that very position."""
import pytest

import bild_inputs as bi
import oracle
from tests import parity


def _ref(n_max=10, max_new=24):
    cfg = bi.toy_pair()
    ws, wl = bi.make_pair_weights(cfg)
    req = oracle.Request(oracle.Model(cfg.small, ws), oracle.Model(cfg.large, wl), bi.make_source(cfg), False)
    return cfg, req, oracle.bild_generate(req, 0.5, 2.0, n_max, max_new)


def test_identical_tokens_pass_and_counters_are_checked():
    cfg, req, ref = _ref()
    stats = {k: getattr(ref.stats, k) for k in ("small_steps", "large_calls", "rows_verified", "fallbacks_conf",
                                                "fallbacks_forced", "rollbacks", "tokens_discarded")}
    assert parity.compare_generation(list(ref.tokens), stats, ref, 0.5, 2.0) == dict(exact=True, matched=len(ref.tokens))
    stats["rollbacks"] += 1
    with pytest.raises(AssertionError):                 # same tokens by another route needs a marginal decision somewhere
        parity.compare_generation(list(ref.tokens), stats, ref, 0.5, 2.0)
    rec = next(r for r in ref.trace if r["kind"] == "large" and r["n"] >= 1)
    rec["nll"][0] = 2.0 + 1e-4
    assert parity.compare_generation(list(ref.tokens), stats, ref, 0.5, 2.0) == dict(exact=False, matched=len(ref.tokens))


def test_a_difference_needs_a_marginal_decision_about_that_position():
    cfg, req, ref = _ref()
    n0 = parity.first_position(ref)
    assert n0 == 1
    for idx in (0, 5, len(ref.tokens) - 1):
        toks = list(ref.tokens)
        toks[idx] = (toks[idx] + 1) % cfg.large.vocab
        with pytest.raises(AssertionError):
            parity.compare_generation(toks, None, ref, 0.5, 2.0)
        # a near-tie two positions EARLIER does not excuse it ...
        _, _, ref2 = _ref()
        for rec in ref2.trace:
            if rec["kind"] == "small" and rec["pos"] == n0 + idx - 2:
                rec["gap"] = 1e-6
        with pytest.raises(AssertionError):
            parity.compare_generation(toks, None, ref2, 0.5, 2.0)
        # ... a near-tie, or a confidence next to the threshold, in a decision about that position does
        for field, value in (("gap", 1e-6), ("pmax", 0.5 + 1e-4)):
            _, _, ref3 = _ref()
            hit = False
            for rec in ref3.trace:
                if rec["kind"] == "small" and rec["pos"] == n0 + idx:
                    rec[field] = value
                    hit = True
                elif rec["kind"] == "large" and rec["draft_start"] + rec["r"] == n0 + idx and field == "gap":
                    rec["gaps"][rec["r"]] = value
                    hit = True
            assert hit
            assert parity.compare_generation(toks, None, ref3, 0.5, 2.0) == dict(exact=False, matched=idx)


def test_review_margins_count_for_the_draft_they_judge_only():
    cfg, req, ref = _ref()
    rec = next(r for r in ref.trace if r["kind"] == "large" and r["n"] >= 2)
    ds = rec["draft_start"]
    rec["nll"][1] = 2.0 - 1e-4                      # the second draft of this block sat next to alpha_RB
    assert parity.marginal_records(ref, ds + 1, 0.5, 2.0) == [rec]
    assert parity.marginal_records(ref, ds, 0.5, 2.0) == []
    assert parity.marginal_records(ref, ds + 1, 0.5, None) == []       # thresholds not given: not consulted


def test_plain_greedy_traces_use_the_same_rule():
    cfg, req, _ = _ref()
    g = oracle.greedy(req, "large", 8)
    assert parity.compare_generation(list(g.tokens), None, g)["exact"]
    toks = list(g.tokens)
    toks[3] = (toks[3] + 1) % cfg.large.vocab
    with pytest.raises(AssertionError):
        parity.compare_generation(toks, None, g)
    g.trace[3]["gap"] = 1e-5
    assert parity.compare_generation(toks, None, g) == dict(exact=False, matched=3)
