"""GPU parity of the sampling variant (Appendix, "BiLD with Sampling"): both models draw their tokens from
the nucleus of their distribution, with the uniform numbers passed in from the seeded input generator, and
the drawn tokens / flags / rollback indices are compared with the oracle step by step.

Margin rule: a difference is excused only where the ORACLE's own decision about that token was marginal.
The threshold distances (|max p - alpha_FB|, |nll - alpha_RB|) use the benchmark's 1e-3.  The draw has a
margin of its own: with every logit within eps of the oracle's, each exp(z_i - m) is within a factor
exp(+-2 eps) of its value, so the ratio (running mass) / (nucleus mass) that u is compared with - and the
ratio (top mass) / (total mass) that top_p is compared with - moves by at most 2 eps relative.  eps is the
logit tolerance of the storage type (1e-4 / 2e-2), so the draw margin is max(1e-3, 2 eps)."""
import numpy as np
import pytest

import bild_inputs as bi
import oracle
import paper_2302_07863_amd as pkg
from tests import parity
from tests.test_gpu_parity import Rig, TOY_VARIANTS

pytestmark = pytest.mark.gpu
TOP_P = 0.8


def _uniforms(cfg, n):
    return bi.make_uniforms(n, cfg.input_seed, 0), bi.make_uniforms(n, cfg.input_seed, 1)


def _margin(cfg):
    """Draw margin (see the module text)."""
    return max(parity.MARGIN, 2 * parity.logit_tol(cfg))


def _marginal(rec, fb, rb, margin):
    """Was this oracle step within reach of going the other way?  Thresholds: 1e-3; the draw: `margin`."""
    if rec.get("draw_margin") is not None and rec["draw_margin"] < margin:
        return True
    if rec["kind"] == "small":
        return abs(rec["pmax"] - fb) < parity.MARGIN
    return any(abs(v - rb) < parity.MARGIN for v in rec["nll"])


def replay(state, ref, n0, fb, rb, margin):
    """Replays the oracle's trajectory through small_step / large_verify, comparing every drawn token, flag
    and rollback index; after an excused difference the GPU is forced back onto the oracle's sequence."""
    y = list(state.sequence())
    ds = n0
    excused = steps = 0
    for rec in ref.trace:
        steps += 1
        if rec["kind"] == "small":
            tok, flag, pmax = state.small_step(fb)
            if not rec["fallback"]:
                y.append(rec["tok"])
            good = bool(flag) == rec["fallback"] and tok == rec["tok"]
        else:
            n, r_ref = rec["n"], rec["r"]
            out, r, nll = state.large_verify(rb)
            y = y[:ds + r_ref] + [rec["tok"]]
            good = r == r_ref and out[-1] == rec["tok"]
            ds = len(y)
        if not good:
            assert _marginal(rec, fb, rb, margin), ({k: v for k, v in rec.items() if k != "z"},)
            excused += 1
            state.force_tokens(n0, y[n0:], ds)
    assert state.sequence() == y
    return dict(steps=steps, excused=excused)


def free_running(tokens, stats, ref, n0, fb, rb, margin):
    """Whole-generation comparison: identical, or the first differing token traces back to a marginal oracle
    decision about that very position (parity.compare_generation with the draw margin)."""
    assert parity.first_position(ref) == n0
    return parity.compare_generation(tokens, stats, ref, fb, rb, draw_margin=margin)["exact"]


@pytest.mark.parametrize("route", ["spread", "one-workgroup"])
@pytest.mark.parametrize("name", ["f32-relu-tied", "f32-geglu-untied", "f32-rope-swiglu-deconly", "f32-wide",
                                  "bf16-relu-tied"])
def test_sampling_toy_parity(name, route, monkeypatch):
    """Both routes of the draw: spread over the chip (integer masses, one workgroup per 1024 ids; the default) and the
    policy kernel's own single workgroup (BILD_DRAW_ONE_WG=1, read when a state is created)."""
    monkeypatch.setenv("BILD_DRAW_ONE_WG", "0" if route == "spread" else "1")
    R = Rig(bi.toy_pair(**TOY_VARIANTS[name]))
    cfg = R.cfg
    n = R.n0 + cfg.max_new + 1
    us, ul = _uniforms(cfg, n)
    smp = oracle.Sampler(TOP_P, us, ul)
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, cfg.max_new, sampler=smp)
        st = R.state(cfg.max_new, nm)
        st.set_sampling(TOP_P, us, ul)
        st.encode(R.src)
        res = replay(st, ref, R.n0, fb, rb, _margin(cfg))
        toks, stats = st.generate(R.src, fb, rb, cfg.max_new)
        print(name, fb, rb, res, free_running(toks, stats, ref, R.n0, fb, rb, _margin(cfg)), stats)


def test_sampling_tiny_config_and_limits():
    cfg = bi.tiny_pair()
    R = Rig(cfg)
    n = R.n0 + cfg.max_new + 1
    us, ul = _uniforms(cfg, n)
    st = R.state(cfg.max_new, cfg.n_max)
    greedy_toks, greedy_stats = st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
    for top_p in (0.8, 0.5, 1.0):
        smp = oracle.Sampler(top_p, us, ul)
        ref = oracle.bild_generate(R.req, cfg.alpha_fb, cfg.alpha_rb, cfg.n_max, cfg.max_new, sampler=smp)
        st.set_sampling(top_p, us, ul)
        st.encode(R.src)
        res = replay(st, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, parity.MARGIN)
        toks, stats = st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
        print("tiny", top_p, res, free_running(toks, stats, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, parity.MARGIN))
        assert ref.tokens != greedy_toks
        # large-only sampling (vanilla inference with draws)
        g = oracle.greedy(R.req, "large", 16, sampler=smp)
        got = st.greedy(pkg.LARGE, R.src, 16)
        assert got == g.tokens or min(r["draw_margin"] for r in g.trace) < parity.MARGIN
    # a nucleus that only ever holds the most likely token is argmax decoding, and so is switching sampling off
    st.set_sampling(1e-9, us, ul)
    assert st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new) == (greedy_toks, greedy_stats)
    st.set_sampling(TOP_P, us, ul)
    st.set_sampling(0.0)
    assert st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new) == (greedy_toks, greedy_stats)


def test_sampling_argument_errors():
    R = Rig(bi.toy_pair())
    st = R.state(R.cfg.max_new, 4)
    n = R.n0 + R.cfg.max_new + 1
    us, ul = _uniforms(R.cfg, n)
    for bad in (lambda: st.set_sampling(1.5, us, ul), lambda: st.set_sampling(0.8, us[:3], ul[:3]),
                lambda: st.set_sampling(0.8, us + 1.0, ul)):
        with pytest.raises(pkg.BildError) as e:
            bad()
        assert e.value.code == -1
    toks, _ = st.generate(R.src, 0.5, 2.0, 8)               # still usable, still greedy
    assert toks == oracle.bild_generate(R.req, 0.5, 2.0, 4, 8).tokens


@pytest.mark.timeout(900)
def test_sampling_t5_full_size():
    """Config 2 at full size with nucleus sampling: 32k-wide rows, bf16."""
    cfg = bi.t5_pair()
    R = Rig(cfg)
    n = R.n0 + cfg.max_new + 1
    us, ul = _uniforms(cfg, n)
    smp = oracle.Sampler(TOP_P, us, ul)
    ref = oracle.bild_generate(R.req, cfg.alpha_fb, cfg.alpha_rb, cfg.n_max, cfg.max_new, sampler=smp)
    st = R.state(cfg.max_new, cfg.n_max)
    st.set_sampling(TOP_P, us, ul)
    st.encode(R.src)
    res = replay(st, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, _margin(cfg))
    print("t5 sampled", res, ref.stats, flush=True)
    assert res["excused"] <= 4
    toks, stats = st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
    print("t5 sampled free-running", free_running(toks, stats, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, _margin(cfg)), flush=True)


@pytest.mark.timeout(900)
def test_sampling_mt5_full_size():
    """Config 3 at full size with nucleus sampling: rows of 250 112 logits, which the drawing workgroup re-reads in
    every sweep of its threshold search (they no longer fit its registers); 24 new tokens keep the oracle affordable.

    Two checks per step.  (1) The draw itself, free of the models' arithmetic: the token the library commits must be
    the oracle's draw function applied to the LIBRARY'S OWN logits of that row (read back), with the same uniform
    number - only float32 against float64 inside the draw separates the two, so the margin is 1e-3.  (2) The
    trajectory against the oracle's, with the bf16 draw margin (logits of magnitude 20 that differ by up to 1.5e-2
    move a cumulative mass by up to 4e-2 relative): each excused step is checked to be marginal on the oracle's side."""
    from dataclasses import replace
    from oracle import sampling
    cfg = replace(bi.mt5_pair(), max_new=24)
    R = Rig(cfg)
    n = R.n0 + cfg.max_new + 1
    us, ul = _uniforms(cfg, n)
    smp = oracle.Sampler(TOP_P, us, ul)
    fb, rb = cfg.alpha_fb, cfg.alpha_rb
    ref = oracle.bild_generate(R.req, fb, rb, cfg.n_max, cfg.max_new, sampler=smp)
    st = R.state(cfg.max_new, cfg.n_max)
    st.set_sampling(TOP_P, us, ul)
    st.debug_enable_logits(True)
    st.encode(R.src)
    y, ds = list(st.sequence()), R.n0
    excused = own_marginal = 0
    for rec in ref.trace:
        if rec["kind"] == "small":
            pos = len(y)
            tok, flag, _ = st.small_step(fb)
            z = st.debug_logits(pkg.SMALL, 0).astype(np.float64)
            own, dm = sampling.draw(z, TOP_P, float(us[pos]))
            assert tok == own or dm < parity.MARGIN, ("small draw", pos, tok, own, dm)
            own_marginal += int(tok != own)
            if not rec["fallback"]:
                y.append(rec["tok"])
            good = bool(flag) == rec["fallback"] and tok == rec["tok"]
        else:
            out, r, _ = st.large_verify(rb)
            z = st.debug_logits(pkg.LARGE, r).astype(np.float64)
            own, dm = sampling.draw(z, TOP_P, float(ul[ds + r]))
            assert out[-1] == own or dm < parity.MARGIN, ("large draw", ds + r, out[-1], own, dm)
            own_marginal += int(out[-1] != own)
            y = y[:ds + rec["r"]] + [rec["tok"]]
            good = r == rec["r"] and out[-1] == rec["tok"]
            ds = len(y)
        if not good:
            assert _marginal(rec, fb, rb, _margin(cfg)), ({k: v for k, v in rec.items() if k != "z"},)
            excused += 1
            st.force_tokens(R.n0, y[R.n0:], ds)
    print("mt5 sampled: steps", len(ref.trace), "excused against the oracle", excused, "own-logit draws off", own_marginal,
          ref.stats, flush=True)
    assert st.sequence() == y and own_marginal <= 1 and excused <= len(ref.trace) // 4 and len(set(ref.tokens)) > 4


@pytest.mark.parametrize("route", ["spread", "one-workgroup"])
def test_sampling_vocabulary_beyond_the_register_cache(route, monkeypatch):
    """A vocabulary of 40 000 ids on a narrow model the oracle finishes in seconds; fp32 and bf16.  Spread route: 40
    slices, the last one ragged.  Single workgroup: more than 32 768 ids, so a row no longer stays in the registers of
    the 1024 threads that draw and every radix sweep re-reads it."""
    monkeypatch.setenv("BILD_DRAW_ONE_WG", "0" if route == "spread" else "1")
    for dtype in (bi.DT_F32, bi.DT_BF16):
        cfg = bi.toy_pair(dtype=dtype, vocab=40000, d=64, heads=2, d_head=16, d_ff=96, max_new=16, tie_shift=4099,
                          logit_scale=24.0)
        R = Rig(cfg)
        n = R.n0 + cfg.max_new + 1
        us, ul = _uniforms(cfg, n)
        for top_p in (TOP_P, 1.0):
            smp = oracle.Sampler(top_p, us, ul)
            ref = oracle.bild_generate(R.req, 0.15, 3.0, 5, cfg.max_new, sampler=smp)
            st = R.state(cfg.max_new, 5)
            st.set_sampling(top_p, us, ul)
            st.encode(R.src)
            res = replay(st, ref, R.n0, 0.15, 3.0, _margin(cfg))
            toks, stats = st.generate(R.src, 0.15, 3.0, cfg.max_new)
            print("V=40000", dtype, top_p, res, free_running(toks, stats, ref, R.n0, 0.15, 3.0, _margin(cfg)), ref.stats, flush=True)
            assert res["excused"] <= 3 and len(set(ref.tokens)) > 4      # (every excused step passed the margin rule) a real draw, not one repeated token
