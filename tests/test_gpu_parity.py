"""GPU parity: the HIP library against the CPU oracle, through the C ABI.

Toy pairs cover every architecture variant and ragged shapes (vocabulary not a
multiple of the feature tile, several k tiles, inner dim != model dim); the
`tiny` pair is the fp32 correctness configuration of the benchmark."""
import math

import numpy as np
import pytest

import bild_inputs as bi
import oracle
import paper_2302_07863_amd as pkg
from tests import parity

pytestmark = pytest.mark.gpu
INF = float("inf")


class Rig:
    """Weights, oracle request and GPU pair of one configuration."""

    def __init__(self, cfg, n_src=None, compact=False):
        self.cfg = cfg
        self.ws, self.wl = bi.make_pair_weights(cfg)
        self.src = bi.make_source(cfg, n_src)
        self.req = oracle.Request(oracle.Model(cfg.small, self.ws, compact), oracle.Model(cfg.large, self.wl, compact),
                                  self.src, cfg.decoder_only)
        self.pair = parity.make_gpu_pair(cfg, self.ws, self.wl)
        self.n0 = len(self.src) if cfg.decoder_only else 1

    def state(self, max_new, n_max):
        return pkg.State(self.pair, len(self.src), self.n0 + max_new + 1, n_max)


TOY_VARIANTS = {
    "f32-relu-tied": dict(),
    "bf16-relu-tied": dict(dtype=bi.DT_BF16),
    "f32-geglu-untied": dict(act=bi.ACT_GATED_GELU, tied=False),
    "bf16-trunc-geglu": dict(act=bi.ACT_GATED_GELU, tied=False, truncate=True, dtype=bi.DT_BF16),
    "f32-rope-swiglu-deconly": dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False),
    "bf16-rope-swiglu-deconly": dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False, dtype=bi.DT_BF16,
                                     truncate=True),
    "f32-wide": dict(d=256, heads=3, d_head=32, d_ff=160, vocab=1000, n_src=40),
    # relative-position scheme: score bias by clamped distance (the source and the generation are both
    # longer than the clamp of 5); the wide one runs its encoder over more than 32 rows at once
    "f32-relative": dict(pos=bi.POS_RELATIVE),
    "bf16-relative-trunc-geglu": dict(pos=bi.POS_RELATIVE, act=bi.ACT_GATED_GELU, truncate=True, dtype=bi.DT_BF16),
    "f32-relative-deconly": dict(pos=bi.POS_RELATIVE, cross=False, tied=False),
    "f32-relative-wide": dict(pos=bi.POS_RELATIVE, d=256, heads=3, d_head=32, d_ff=160, vocab=1000, n_src=40,
                              rel_max_dist=11, rel_buckets=8),
}
_rigs = {}


def rig(name):
    if name not in _rigs:
        _rigs[name] = Rig(bi.toy_pair(**TOY_VARIANTS[name]))
    return _rigs[name]


@pytest.mark.parametrize("name", list(TOY_VARIANTS))
@pytest.mark.parametrize("fb,rb,nm", [(0.5, 2.0, 10), (0.2, 0.7, 3)])
def test_toy_teacher_forced_logits_and_decisions(name, fb, rb, nm):
    R = rig(name)
    ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
    st = R.state(R.cfg.max_new, nm)
    st.encode(R.src)
    worst = parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg)
    print(name, worst)


@pytest.mark.parametrize("name", ["bf16-relu-tied", "bf16-trunc-geglu", "bf16-rope-swiglu-deconly",
                                  "bf16-relative-trunc-geglu"])
@pytest.mark.parametrize("first_rows", [1, 2])
def test_bf16_plane_handover_at_every_row_count(name, first_rows, monkeypatch):
    """bf16 passes hand activations from kernel to kernel as high / low bf16 planes from some row count on (by
    default only where that is faster); here from one row / from two rows on, so that every producer and consumer of
    the planes (embedding, residual projections, attention, merged key splits, FFN, LM head) meets the oracle at the
    small row counts as well.  The state reads the setting when it is created."""
    monkeypatch.setenv("BILD_PRE_MIN_ROWS", str(first_rows))
    R = rig(name)
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
        st = R.state(R.cfg.max_new, nm)
        st.encode(R.src)
        worst = parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg)
        print(name, first_rows, worst)
    # blocks of 1..32 rows with the planes against the same blocks without them: same distributions up to rounding order
    block = [int(t) for t in bi.make_tokens(R.cfg.large.vocab, 31, seed=5)]
    rows = {}
    for setting in (str(first_rows), "99"):
        monkeypatch.setenv("BILD_PRE_MIN_ROWS", setting)
        st = R.state(40, 10)
        st.encode(R.src)
        st.debug_enable_logits(True)
        out = []
        for n in (0, 1, 3, 4, 7, 15, 16, 31):
            st.force_tokens(R.n0, [], R.n0)
            st.large_verify(INF, draft=block[:n])
            out.append(np.stack([st.debug_logits(pkg.LARGE, i) for i in range(n + 1)]))
        rows[setting] = out
    for a, b in zip(rows[str(first_rows)], rows["99"]):
        assert np.max(np.abs(a - b)) <= parity.logit_tol(R.cfg)


@pytest.mark.parametrize("name", ["f32-relu-tied", "bf16-relu-tied", "bf16-trunc-geglu", "f32-rope-swiglu-deconly", "tiny"])
def test_split_ffn_output_projection_on_small_widths(name, monkeypatch):
    """Narrow models cut the FFN output projection of passes of one to four rows into slices of its inputs whose partial
    results the next projection (or the LM head) adds to the residual stream; by default only from an FFN width of 2048
    (configs 2 and 3 at full size).  Here from a width of 64, so that the toys and config 1 (whose widths also allow the
    two-to-four-row form) take that route against the oracle, logit by logit."""
    monkeypatch.setenv("BILD_KSPLIT_MIN_F", "64")
    if name == "tiny":
        R = Rig(bi.tiny_pair())
    else:
        R = Rig(bi.toy_pair(**dict(TOY_VARIANTS[name], d_ff=128)))
    for fb, rb, nm in ((R.cfg.alpha_fb, R.cfg.alpha_rb, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
        st = R.state(R.cfg.max_new, nm)
        st.encode(R.src)
        worst = parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg)
        print(name, worst)
        toks, stats = R.state(R.cfg.max_new, nm).generate(R.src, fb, rb, R.cfg.max_new)
        parity.compare_generation(toks, stats, ref, fb, rb)
    # the same generation twice is the same bits
    st = R.state(R.cfg.max_new, 10)
    a = st.generate(R.src, 0.5, 2.0, R.cfg.max_new)
    b = st.generate(R.src, 0.5, 2.0, R.cfg.max_new)
    assert a == b


FUSED_TOYS = {
    "f32-dh32": dict(d=128, heads=3, d_head=32, d_ff=128),
    "bf16-dh32-geglu": dict(d=128, heads=4, d_head=32, d_ff=128, dtype=bi.DT_BF16, act=bi.ACT_GATED_GELU, tied=False),
    "bf16-dh64-trunc": dict(d=128, heads=2, d_head=64, d_ff=128, dtype=bi.DT_BF16, truncate=True),
    "bf16-dh64-rope-deconly": dict(d=128, heads=2, d_head=64, d_ff=128, dtype=bi.DT_BF16, act=bi.ACT_SWIGLU, pos=bi.POS_ROPE,
                                   cross=False, tied=False),
    "bf16-dh32-relative": dict(d=128, heads=4, d_head=32, d_ff=128, dtype=bi.DT_BF16, pos=bi.POS_RELATIVE),
    # sources long enough that a head's cross-attention K/V exceed what one workgroup takes (key splits, merged by the
    # output projection) while the self-attention cache stays short (fused with its output projection)
    "bf16-dh64-long-source": dict(d=128, heads=2, d_head=64, d_ff=128, dtype=bi.DT_BF16, n_src=200),
    "f32-dh32-long-source": dict(d=128, heads=3, d_head=32, d_ff=128, n_src=200),
}


@pytest.mark.parametrize("name", list(FUSED_TOYS))
def test_single_row_passes_fuse_attention_with_its_output_projection(name, monkeypatch):
    """Single-row passes of models up to 1024 wide with heads of 32 or 64 dims run attention and its output projection
    as one kernel per (head, column group) and let the next projection add one partial result per head (configs 1-3
    take this route at full size).  The same toys with the fusion switched off must give the same distributions up
    to summation order, and both must meet the oracle."""
    monkeypatch.setenv("BILD_KSPLIT_MIN_F", "64")
    R = Rig(bi.toy_pair(**FUSED_TOYS[name]))
    tol = parity.logit_tol(R.cfg)
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
        st = R.state(R.cfg.max_new, nm)
        st.encode(R.src)
        worst = parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg)
        print(name, worst)
    rows = {}
    for fuse in ("1", "0"):
        monkeypatch.setenv("BILD_FUSE_ATTN", fuse)
        st = R.state(R.cfg.max_new, 0)
        st.debug_enable_logits(True)
        toks = st.greedy(pkg.LARGE, R.src, 12)
        rows[fuse] = (toks, st.debug_logits(pkg.LARGE, 0))
    assert rows["1"][0] == rows["0"][0] and np.max(np.abs(rows["1"][1] - rows["0"][1])) <= tol
    st = R.state(R.cfg.max_new, 10)
    assert st.generate(R.src, 0.5, 2.0, R.cfg.max_new) == st.generate(R.src, 0.5, 2.0, R.cfg.max_new)


@pytest.mark.parametrize("name", ["f32-relu-tied", "bf16-relu-tied", "bf16-trunc-geglu", "bf16-rope-swiglu-deconly", "f32-relative", "tiny"])
def test_single_row_passes_gather_the_embedding_in_their_first_projection(name, monkeypatch):
    """Single-row passes have no embedding kernel: the first projection gathers its input row from the embedding matrix
    (scaled, position term added in the same fused multiply-add the embedding kernel uses).  With the route switched off
    the embedding kernel runs in front as it does for passes of several rows; both must give the same bits - tokens,
    logits of every step - and the route must meet the oracle (sinusoidal, rotary and relative positions, shifted tied
    lookup, fp32 and bf16)."""
    R = Rig(bi.tiny_pair()) if name == "tiny" else rig(name)
    out = {}
    for fuse in ("1", "0"):
        monkeypatch.setenv("BILD_FUSE_EMBED", fuse)
        st = R.state(R.cfg.max_new, 10)
        st.debug_enable_logits(True)
        rows = []
        for which in (pkg.SMALL, pkg.LARGE):
            toks = st.greedy(which, R.src, 10)
            rows.append((toks, st.debug_logits(which, 0).copy()))
        st.debug_enable_logits(False)
        rows.append(st.generate(R.src, R.cfg.alpha_fb, R.cfg.alpha_rb, R.cfg.max_new))
        out[fuse] = rows
        if fuse == "1":
            ref = oracle.bild_generate(R.req, R.cfg.alpha_fb, R.cfg.alpha_rb, 10, R.cfg.max_new, keep_logits=True)
            st2 = R.state(R.cfg.max_new, 10)
            st2.encode(R.src)
            print(name, parity.teacher_forced(st2, ref, R.n0, R.cfg.alpha_fb, R.cfg.alpha_rb, R.cfg))
    for a, b in zip(out["1"][:2], out["0"][:2]):
        assert a[0] == b[0] and np.array_equal(a[1], b[1])
    assert out["1"][2] == out["0"][2]


@pytest.mark.parametrize("name", list(TOY_VARIANTS))
def test_toy_free_running_generate(name):
    R = rig(name)
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3), (0.0, 0.5, 6)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new)
        st = R.state(R.cfg.max_new, nm)
        toks, stats = st.generate(R.src, fb, rb, R.cfg.max_new)
        res = parity.compare_generation(toks, stats, ref, fb, rb)
        print(name, fb, rb, nm, res, stats)


@pytest.mark.parametrize("name", ["f32-relu-tied", "bf16-trunc-geglu", "bf16-rope-swiglu-deconly"])
def test_limiting_cases_on_the_gpu(name):
    R = rig(name)
    n = R.cfg.max_new
    st = R.state(n, 0)
    small_greedy = st.greedy(pkg.SMALL, R.src, n)
    large_greedy = st.greedy(pkg.LARGE, R.src, n)
    ref_s = oracle.greedy(R.req, "small", n)
    ref_l = oracle.greedy(R.req, "large", n)
    parity.compare_generation(small_greedy, None, ref_s)
    parity.compare_generation(large_greedy, None, ref_l)
    # alpha_FB = 0 and no cap: small-model greedy, the large model never runs
    toks, stats = st.generate(R.src, 0.0, 2.0, n)
    assert toks == small_greedy and stats["large_calls"] == 0
    # alpha_FB > 1: always fall back -> large-model greedy for any alpha_RB
    st10 = R.state(n, 10)
    for rb in (-1.0, 0.5, INF):
        toks, stats = st10.generate(R.src, 2.0, rb, n)
        assert toks == large_greedy and stats["rollbacks"] == 0 and stats["large_calls"] == n
    # alpha_RB < 0: every reviewed draft is rejected; the reviewed part is large-model greedy
    toks, stats = st10.generate(R.src, 0.0, -1.0, n)
    ds = st10.lengths()["draft_start"] - R.n0
    assert ds > 0 and toks[:ds] == large_greedy[:ds]


@pytest.mark.parametrize("name", ["f32-relu-tied", "bf16-trunc-geglu", "f32-rope-swiglu-deconly"])
def test_review_pass_equals_sequential_steps(name):
    """One pass over n+1 rows gives the distributions of n+1 single-row passes (Section 3.2)."""
    R = rig(name)
    tol = parity.logit_tol(R.cfg)
    block = [int(t) for t in bi.make_tokens(R.cfg.large.vocab, 9, seed=11)]
    st = R.state(40, 10)
    st.encode(R.src)
    st.debug_enable_logits(True)
    out, r, nll = st.large_verify(INF, draft=block)          # never roll back: all rows are kept
    assert r == len(block)
    rows = [st.debug_logits(pkg.LARGE, i) for i in range(len(block) + 1)]
    # oracle: the same rows from the definition
    y = R.req.initial() + block
    z = R.req.large.logits_full(y, R.req.cross_l)[len(y) - len(block) - 1:]
    assert np.max(np.abs(np.stack(rows) - z)) <= tol
    # the same block, one row at a time
    st2 = R.state(40, 10)
    st2.encode(R.src)
    st2.debug_enable_logits(True)
    for i in range(len(block) + 1):
        st2.force_tokens(R.n0, block[:i], R.n0 + i)
        out2, r2, _ = st2.large_verify(INF, draft=[])
        z1 = st2.debug_logits(pkg.LARGE, 0)
        # one more row in the same pass only changes the summation order
        assert np.max(np.abs(z1 - rows[i])) <= (1e-5 if R.cfg.large.dtype == bi.DT_F32 else 5e-3)
        assert out2[0] == int(np.argmax(z1))


def test_truncate_then_continue_equals_fresh_prefix():
    R = rig("bf16-trunc-geglu")
    fb, rb, nm, n = 0.3, 1.0, 4, R.cfg.max_new
    st = R.state(n, nm)
    toks, _ = st.generate(R.src, fb, rb, n)
    keep = 7
    st.seq_truncate(R.n0 + keep)
    ln = st.lengths()
    assert ln["y_len"] == R.n0 + keep and ln["len_small"] <= R.n0 + keep - 1 and ln["len_large"] <= ln["draft_start"] - 1
    # continue with always-fallback: every further token is the large model's greedy choice given its prefix
    for _ in range(5):
        tok, flag, _ = st.small_step(2.0)
        assert flag == 1
        st.large_verify(rb)
    seq = st.sequence()
    assert len(seq) == R.n0 + keep + 5 and seq[R.n0:R.n0 + keep] == toks[:keep]
    for p in range(R.n0 + keep, len(seq)):
        z = R.req.large.logits_full(seq[:p], R.req.cross_l)[-1]
        assert seq[p] == int(np.argmax(z)) or oracle.policy.top2_gap(z) < parity.MARGIN


def test_state_errors_on_the_device():
    R = rig("f32-relu-tied")
    b = pkg.binding
    st = R.state(8, 2)
    with pytest.raises(pkg.BildError) as e:
        st.small_step(0.5)                                  # before encode
    assert e.value.code == b.ESTATE
    with pytest.raises(pkg.BildError) as e:
        st.encode(list(R.src) + [1])                        # longer than max_src
    assert e.value.code == b.ECAP
    with pytest.raises(pkg.BildError) as e:
        st.encode([R.cfg.large.vocab])                      # token id out of range
    assert e.value.code == b.EINVAL
    st.encode(R.src)
    tok, flag, _ = st.small_step(2.0)
    assert flag == 1
    before = st.lengths()
    with pytest.raises(pkg.BildError) as e:
        st.small_step(2.0)                                  # nothing unconsumed after a fallback
    assert e.value.code == b.ESTATE
    assert st.lengths() == before                           # state unchanged by the failed call
    with pytest.raises(pkg.BildError) as e:
        st.kv_truncate(pkg.SMALL, before["len_small"] + 1)
    assert e.value.code == b.EINVAL
    with pytest.raises(pkg.BildError) as e:
        st.large_verify(1.0, draft=[0] * 32)                # more rows than one pass takes
    assert e.value.code == b.ECAP
    with pytest.raises(pkg.BildError) as e:
        st.large_verify(1.0, draft=[R.cfg.large.vocab])
    assert e.value.code == b.EINVAL
    assert st.lengths() == before
    out, r, _ = st.large_verify(1.0)
    assert r == 0 and len(out) == 1
    # generation longer than the state's capacity
    with pytest.raises(pkg.BildError) as e:
        st.generate(R.src, 0.5, 2.0, 64)
    assert e.value.code == b.ECAP
    # mismatched vocabularies cannot be paired
    other = bi.toy_pair(vocab=R.cfg.large.vocab + 8)
    ws2, _ = bi.make_pair_weights(other)
    m2 = parity.make_gpu_model(other.small, ws2)
    with pytest.raises(pkg.BildError) as e:
        pkg.Pair(m2, R.pair.large)
    assert e.value.code == b.EINVAL


def test_kv_truncate_recomputes_identically():
    R = rig("bf16-relu-tied")
    st = R.state(24, 10)
    st.encode(R.src)
    st.debug_enable_logits(True)
    block = [int(t) for t in bi.make_tokens(R.cfg.large.vocab, 6, seed=3)]
    st.large_verify(INF, draft=block)
    a = np.stack([st.debug_logits(pkg.LARGE, i) for i in range(7)])
    # cut both caches to nothing and review the same block again: bit-identical (deterministic kernels)
    st.force_tokens(R.n0, block, R.n0)
    st.kv_truncate(pkg.BOTH, 0)
    st.large_verify(INF)
    b2 = np.stack([st.debug_logits(pkg.LARGE, i) for i in range(7)])
    assert np.array_equal(a, b2)


def test_concurrent_requests_on_streams_of_their_own():
    """Independent requests may run at once: one state each (a stream of its own), one host thread each, weights shared
    through the pair.  Every request must produce exactly what it produces alone (config 1 and a bf16 toy)."""
    import threading
    for R in (Rig(bi.tiny_pair()), rig("bf16-trunc-geglu")):
        cfg = R.cfg
        alone = R.state(cfg.max_new, cfg.n_max).generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
        ref = oracle.bild_generate(R.req, cfg.alpha_fb, cfg.alpha_rb, cfg.n_max, cfg.max_new)
        parity.compare_generation(alone[0], alone[1], ref, cfg.alpha_fb, cfg.alpha_rb)
        states = [R.state(cfg.max_new, cfg.n_max) for _ in range(4)]
        got = [[] for _ in states]
        start = threading.Barrier(len(states))

        def work(i):
            start.wait()
            for _ in range(5):
                got[i].append(states[i].generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new))

        threads = [threading.Thread(target=work, args=(i,)) for i in range(len(states))]
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=120)
        assert all(not t.is_alive() for t in threads)
        assert all(g == alone for per in got for g in per)


def test_tiny_config_full_parity():
    """Config 1: fp32, logits within 1e-4, decisions identical."""
    cfg = bi.tiny_pair()
    R = Rig(cfg)
    ref = oracle.bild_generate(R.req, cfg.alpha_fb, cfg.alpha_rb, cfg.n_max, cfg.max_new, keep_logits=True)
    st = R.state(cfg.max_new, cfg.n_max)
    st.encode(R.src)
    worst = parity.teacher_forced(st, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, cfg)
    print("tiny teacher-forced", worst, ref.stats)
    toks, stats = st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
    print("tiny free-running", parity.compare_generation(toks, stats, ref, cfg.alpha_fb, cfg.alpha_rb), stats)
    for fb, rb in ((0.3, 1.0), (0.7, 4.0), (0.0, 0.3)):
        ref = oracle.bild_generate(R.req, fb, rb, cfg.n_max, cfg.max_new)
        toks, stats = st.generate(R.src, fb, rb, cfg.max_new)
        parity.compare_generation(toks, stats, ref, fb, rb)


# ---------------------------------------------------------------------------------------------
# Full-size configurations, in the launch configuration bench.py times.  The oracle runs the same
# request end to end (it finishes in about a minute per configuration on the host cores).
def _full_size(cfg, max_new, n_src=None, compact=False, thresholds=None):
    R = Rig(cfg, n_src=n_src, compact=compact)
    fb, rb = thresholds or (cfg.alpha_fb, cfg.alpha_rb)
    ref = oracle.bild_generate(R.req, fb, rb, cfg.n_max, max_new, keep_logits=True)
    st = R.state(max_new, cfg.n_max)
    st.encode(R.src)
    worst = parity.teacher_forced(st, ref, R.n0, fb, rb, cfg)
    print(cfg.name, "teacher-forced", worst, ref.stats, flush=True)
    for rec in ref.trace:
        rec.pop("z", None)
    toks, stats = st.generate(R.src, fb, rb, max_new)
    res = parity.compare_generation(toks, stats, ref, fb, rb)
    print(cfg.name, "free-running", res, stats, flush=True)
    return R, st


@pytest.mark.timeout(900)
def test_t5_config_full_size():
    """Config 2: T5-small + T5-large shapes, bf16, 512 source tokens, 64 new tokens."""
    cfg = bi.t5_pair()
    R, st = _full_size(cfg, cfg.max_new)
    # the other thresholds of the sweep, free-running
    for fb, rb in ((0.3, 1.0), (0.7, 4.0)):
        ref = oracle.bild_generate(R.req, fb, rb, cfg.n_max, 32)
        toks, stats = st.generate(R.src, fb, rb, 32)
        print("t5", fb, rb, parity.compare_generation(toks, stats, ref, fb, rb), stats, flush=True)


@pytest.mark.timeout(900)
def test_t5_relative_position_config_full_size():
    """Config 2's shapes with the T5 family's position scheme (score bias by clamped distance, 128; 32 tied
    values per head): 512 source tokens through the biased encoder, 32 new tokens."""
    cfg = bi.PAIRS["t5rel"]()
    _full_size(cfg, 32)


@pytest.mark.timeout(900)
def test_mt5_config_full_size():
    """Config 3: mT5 shapes, 250k vocabulary (the LM head dominates), gated-GELU, 6 heads of the small model."""
    cfg = bi.mt5_pair()
    _full_size(cfg, 32)


# ---------------------------------------------------------------------------------------------
# Decoder-only, 128-wide heads, long prompt: the shape family of configs 4 and 5 at a size the
# oracle finishes in seconds.  Covers prompt prefill in 32-row chunks, RoPE at large positions,
# key-split attention (cache > 512 rows) and review blocks of 1..32 rows with truncation between.
def _llama_mini():
    from dataclasses import replace
    cfg = bi.llama_pair()
    large = replace(cfg.large, n_dec=3, d=512, heads=4, d_ff=1408, vocab=4000, name="llama-mini-large")
    small = replace(cfg.small, n_dec=2, d=256, heads=2, d_ff=704, vocab=4000, name="llama-mini-small")
    return replace(cfg, name="llama-mini", small=small, large=large, n_src=700, max_new=24)


def test_llama_shaped_prefill_and_generation():
    cfg = _llama_mini()
    R = Rig(cfg)
    fb, rb = 0.5, 2.0
    ref = oracle.bild_generate(R.req, fb, rb, cfg.n_max, cfg.max_new, keep_logits=True)
    st = R.state(cfg.max_new, cfg.n_max)
    st.encode(R.src)
    ln = st.lengths()
    assert ln["y_len"] == len(R.src) and ln["len_small"] == ln["len_large"] == len(R.src) - 1
    worst = parity.teacher_forced(st, ref, R.n0, fb, rb, cfg)
    print("llama-mini", worst, ref.stats, flush=True)
    toks, stats = st.generate(R.src, fb, rb, cfg.max_new)
    print(parity.compare_generation(toks, stats, ref, fb, rb), stats, flush=True)


def test_review_stress_blocks_and_random_truncation():
    """Config-5 style: large_verify alone over forced blocks of n+1 in {1,4,8,16,32} rows on a long cache, with
    kv_truncate to random positions in between; every row's logits against the no-cache definition."""
    cfg = _llama_mini()
    R = Rig(cfg)
    tol = parity.logit_tol(cfg)
    rng = np.random.default_rng(5)
    st = pkg.State(R.pair, len(R.src), len(R.src) + 80, 31)
    st.encode(R.src)
    st.debug_enable_logits(True)
    n0 = R.n0
    for n in (0, 3, 7, 15, 31, 7):
        block = [int(t) for t in bi.make_tokens(cfg.large.vocab, n, seed=100 + n)]
        out, r, nll = st.large_verify(INF, draft=block)            # never roll back
        assert r == n and out[:n] == block
        seq = st.sequence()
        y = seq[:-1]                                               # what the pass saw
        z = R.req.large.logits_full(y, [])[len(y) - n - 1:]
        for i in (0, n // 2, n):
            zi = st.debug_logits(pkg.LARGE, i)
            assert np.max(np.abs(zi - z[i])) <= tol, (n, i)
            assert abs(float(nll[i]) - oracle.policy.nll(z[i], block[i])) <= 2 * tol if i < n else True
        assert out[n] == int(np.argmax(z[n])) or oracle.policy.top2_gap(z[n]) < parity.MARGIN
        # cut the large cache at a random row inside the prompt and the sequence back to the prompt:
        # the next review recomputes the cut rows (catch-up) before it reviews its block
        cut = int(rng.integers(1, n0 - 1))
        st.force_tokens(n0, [], n0)
        st.kv_truncate(pkg.LARGE, cut)
        assert st.lengths()["len_large"] == cut


def test_head_dim_128_and_64_bf16_toys():
    for dh, heads in ((128, 1), (64, 2)):
        cfg = bi.toy_pair(dtype=bi.DT_BF16, act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=True, d=128,
                          heads=heads, d_head=dh, d_ff=160, vocab=333, n_src=40)
        R = Rig(cfg)
        ref = oracle.bild_generate(R.req, 0.4, 1.0, 5, cfg.max_new, keep_logits=True)
        st = R.state(cfg.max_new, 5)
        st.encode(R.src)
        print(dh, parity.teacher_forced(st, ref, R.n0, 0.4, 1.0, cfg), ref.stats, flush=True)


def test_two_way_key_splits_merged_by_the_output_projection():
    """Cross-attention over a source whose K/V per head are between one and two split sizes (32 KiB): two key splits,
    merged while the output projection stages its input - bf16 (200 keys) and fp32 (100 keys) storage."""
    for dtype, n_src in ((bi.DT_BF16, 200), (bi.DT_F32, 100)):
        assert pkg.binding.attn_shape(2, 64, 1, n_src, 8, 1 if dtype == bi.DT_BF16 else 0)["splits"] == 2
        cfg = bi.toy_pair(dtype=dtype, act=bi.ACT_RELU, pos=bi.POS_SINUSOIDAL, cross=True, tied=False, d=128, heads=2, d_head=64,
                          d_ff=192, vocab=211, n_src=n_src)
        R = Rig(cfg)
        ref = oracle.bild_generate(R.req, 0.4, 1.0, 6, cfg.max_new, keep_logits=True)
        st = R.state(cfg.max_new, 6)
        st.encode(R.src)
        print(dtype, parity.teacher_forced(st, ref, R.n0, 0.4, 1.0, cfg), ref.stats, flush=True)


def test_relative_bias_with_key_splits_and_long_prompt():
    """Decoder-only relative-position toy with a 300-token prompt: the prefill runs the biased attention over
    row blocks, the steps after it over a cache long enough for key splits, and nearly every distance is clamped (20)."""
    cfg = bi.toy_pair(dtype=bi.DT_BF16, act=bi.ACT_SWIGLU, pos=bi.POS_RELATIVE, cross=False, tied=True, d=128,
                      heads=2, d_head=64, d_ff=160, vocab=333, n_src=300, rel_max_dist=20, rel_buckets=12)
    R = Rig(cfg)
    ref = oracle.bild_generate(R.req, 0.4, 1.0, 5, cfg.max_new, keep_logits=True)
    st = R.state(cfg.max_new, 5)
    st.encode(R.src)
    print(parity.teacher_forced(st, ref, R.n0, 0.4, 1.0, cfg), ref.stats, flush=True)


@pytest.mark.parametrize("kw", [
    dict(n_src=600),                                                                       # fp32, ReLU, encoder + cross K/V
    dict(n_src=530, dtype=bi.DT_BF16, act=bi.ACT_GATED_GELU, tied=False, truncate=True),   # bf16, gated, both encoders
    dict(n_src=577, act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False),          # fp32 prompt prefill with RoPE
    dict(n_src=640, dtype=bi.DT_BF16, pos=bi.POS_RELATIVE, d=128, heads=2, d_head=64, d_ff=160, vocab=333),
])
def test_passes_over_more_than_512_rows_take_the_dense_tile_kernel(kw):
    """Sources / prompts longer than 512 tokens: the encoder (or the prompt prefill) runs on the dense-tile GEMM,
    64 rows per workgroup with a ragged last block, in every epilogue it has (Q/K/V split with and without RoPE,
    cross K/V without queries, residual add, ReLU and gated activation), fp32 and bf16 storage."""
    cfg = bi.toy_pair(**kw)
    assert pkg.binding.gemm_shape(cfg.large.d, cfg.large.d, cfg.n_src - 1, False, False, cfg.large.dtype)["kc"] == 128
    R = Rig(cfg)
    ref = oracle.bild_generate(R.req, 0.4, 1.0, 5, 12, keep_logits=True)
    st = R.state(12, 5)
    st.encode(R.src)
    print(kw, parity.teacher_forced(st, ref, R.n0, 0.4, 1.0, cfg), ref.stats, flush=True)


def _bf16_step(a):
    """Spacing of bf16 values at the magnitude of a (8 significant bits)."""
    return np.ldexp(1.0, np.frexp(np.maximum(np.abs(a), 1e-30))[1] - 8)


def _cache_differences(st, which, cache, layers, n):
    """Per layer (share, worst): the share of cached K/V elements on which the library and the oracle hold
    different bf16 values, and the largest difference relative to the largest value of its tensor.
    In layer 0 both sides start from identical inputs, so the values before rounding differ by fp32-vs-float64
    accumulation noise only (about 1e-7 of the tensor's scale): an element is then either equal or ONE bf16 step
    off (its value fell on the other side of a rounding boundary), except for elements so small that this
    noise already spans several of their own steps - asserted here.  Deeper layers inherit the flipped values
    of the layers below through the hidden state; their differences are reported and bounded by the caller."""
    out = {}
    for l in layers:
        bad = total = 0
        worst = 0.0
        for is_v, ref in ((0, cache.k[l][:n]), (1, cache.v[l][:n])):
            got = st.debug_kv(which, l, bool(is_v), 0, n).astype(np.float64)
            diff = np.abs(got - ref)
            scale = float(np.max(np.abs(ref)))
            if l == 0:
                step = _bf16_step(np.maximum(np.abs(got), np.abs(ref)))
                beyond = diff > step * (1 + 1e-6)
                assert np.all(~beyond | (diff <= 1e-6 * scale)), \
                    ("layer 0: cached values differ by more than one bf16 step", is_v, float(np.max(diff[beyond])) / scale)
            bad += int(np.count_nonzero(diff))
            total += diff.size
            worst = max(worst, float(np.max(diff)) / scale)
        out[l] = (bad / total, worst)
    return out


_llama = {}


def llama_rig():
    """Config 4 at its full widths and depth (weights of both models, the oracle's request on a shortened prompt, the
    uploaded pair); built once for the two tests that use it and released by the second."""
    if "rig" not in _llama:
        from dataclasses import replace
        _llama["rig"] = Rig(replace(bi.llama_pair(), n_src=48, max_new=8), compact=True)
    return _llama["rig"]


@pytest.mark.timeout(1500)
def test_llama_config_full_width_meets_the_bf16_bar_once_storage_rounding_is_aligned():
    """Config 4 at its full widths (32 layers, d 4096, 32 heads of 128, FFN 11008, vocab 32000) on a shortened
    prompt.  The rows of one review pass and of one small step against the oracle, element by element.

    At this depth and width the large model's logits (magnitude 50-140) do NOT meet the 2e-2 bar of the bf16
    configurations: they are off by up to about 5e-2.  What this test pins is the cause and its size:
      * every decision (argmax of the reviewed rows, the small model's token and flag) agrees with the oracle;
      * in layer 0, where both sides start from identical inputs, the library's cached K/V equal the oracle's
        except for a few elements in ten thousand (measured: 4e-4) that are exactly ONE bf16 step off: values
        whose fp32 and float64 results straddle a rounding boundary.  Those flips (2^-8 relative each) enter the
        hidden state, so deeper layers differ on more and more elements (measured: 2 % in layer 1, 28 % in
        layer 8, 50 % in layer 31) - but never by more than one bf16 step of the tensor's largest values (2^-7 of
        the largest magnitude): the noise saturates at the granularity of the storage format;
      * the same widths with fp32 storage (first 8 layers, so that it stays affordable) agree to 3e-6 of the
        largest logit, i.e. the arithmetic itself is fp32-accurate;
      * the logit error stays below 5x the bar (0.1); the small model (16 layers, d 2048) is held to the bar itself;
      * WITH THE STORAGE-ROUNDING DECISIONS ALIGNED THE BAR IS MET: a second oracle pass caches, in every layer, the
        values the library stored (read back) instead of rounding its own - after checking, element by element in all
        32 layers, that each stored value is the bf16 rounding of a number within 1e-4 of the tensor's scale of the
        oracle's exact one (fp32 against float64 accumulation; measured: up to 2e-5 by layer 27, bound 1e-4).  Rounding to the storage type is a decision floating
        point takes about an integer code; taken the same way on both sides, the logits agree to 6e-4 (bar 2e-2);
        1.2 % of the stored values are not the oracle's own rounding of its exact value."""
    from dataclasses import replace
    R = llama_rig()
    cfg = R.cfg
    tol = parity.logit_tol(cfg)
    st = R.state(cfg.max_new + 8, cfg.n_max)
    st.encode(R.src)
    st.debug_enable_logits(True)
    block = [int(t) for t in bi.make_tokens(cfg.large.vocab, 5, seed=9)]
    out, r, nll = st.large_verify(INF, draft=block)
    y = list(R.src) + block
    cache = oracle.model.DecoderCache(R.req.large, [], len(y) + 1)
    z = cache.step(y, last=6)
    worst = 0.0
    for i in range(6):
        zi = st.debug_logits(pkg.LARGE, i)
        err = float(np.max(np.abs(zi - z[i])))
        worst = max(worst, err)
        assert int(np.argmax(zi)) == int(np.argmax(z[i])) or oracle.policy.top2_gap(z[i]) < parity.MARGIN
        if i < 5:
            assert abs(float(nll[i]) - oracle.policy.nll(z[i], block[i])) <= 5 * 2 * tol
    print("large: max |logit|", float(np.max(np.abs(z))), "worst logit error", worst, "bar", tol, flush=True)
    assert worst <= 5 * tol, worst
    assert out[5] == int(np.argmax(z[5])) or oracle.policy.top2_gap(z[5]) < parity.MARGIN
    diffs = _cache_differences(st, pkg.LARGE, cache, (0, 1, 8, 16, 31), len(y))
    print("cached K/V against the oracle's, by layer (share of differing elements, largest difference / tensor scale):",
          diffs, flush=True)
    assert diffs[0][0] < 2e-3, diffs
    assert max(w for _, w in diffs.values()) <= 2.0 ** -7, diffs
    del cache
    # the same rows with the library's storage-rounding decisions: every cached element is checked as it is taken over
    flips = {"n": 0, "total": 0, "worst": 0.0}

    def stored_by_the_library(l, kind, exact, t0):
        got = st.debug_kv(pkg.LARGE, l, kind == "v", t0, exact.shape[0]).astype(np.float64)
        scale = float(np.max(np.abs(exact)))
        # a correct rounding of a value within 1e-4 * scale of the exact one: at most half a bf16 step (of the stored
        # value's binade, or of the exact value's if that is larger) plus that noise away from it
        step = np.maximum(_bf16_step(got), _bf16_step(exact))
        off = np.abs(got - exact)
        assert np.all(off <= 0.5 * step + 1e-4 * scale), (l, kind, float(np.max((off - 0.5 * step) / scale)))
        assert np.all(oracle.model.round_bf16(got) == got)
        flips["n"] += int(np.count_nonzero(got != oracle.model.round_bf16(exact)))
        flips["total"] += got.size
        flips["worst"] = max(flips["worst"], float(np.max((off - 0.5 * step) / scale)))
        return got

    z2 = oracle.model.DecoderCache(R.req.large, [], len(y) + 1, store=stored_by_the_library).step(y, last=6)
    aligned = max(float(np.max(np.abs(st.debug_logits(pkg.LARGE, i) - z2[i]))) for i in range(6))
    print("storage rounding aligned: worst logit error", aligned, "bar", tol, "; stored values that are not the oracle's own rounding:",
          flips["n"], "of", flips["total"], "; worst excess over half a step / scale", flips["worst"], flush=True)
    assert aligned <= tol, aligned
    assert flips["n"] <= 0.03 * flips["total"], flips  # (measured: 1.2 % of the elements sit that close to a rounding boundary)
    # the small model of the pair: one step
    tok, flag, pmax = st.small_step(0.5)
    seq = st.sequence()
    pre = seq if flag else seq[:-1]
    zs = R.req.small.logits_full(pre, [])[-1]
    zg = st.debug_logits(pkg.SMALL, 0)
    err_s = float(np.max(np.abs(zg - zs)))
    print("small: max |logit|", float(np.max(np.abs(zs))), "logit error", err_s, flush=True)
    assert err_s <= tol and abs(pmax - oracle.policy.max_prob(zs)) <= 2 * tol
    assert tok == int(np.argmax(zs)) or oracle.policy.top2_gap(zs) < parity.MARGIN
    assert bool(flag) == (oracle.policy.max_prob(zs) < 0.5) or abs(oracle.policy.max_prob(zs) - 0.5) < parity.MARGIN
    # control: the first 8 layers of the same large model with fp32 storage of weights and K/V (the weights hold the
    # same bf16-representable values): no rounding of K/V on either side, so the difference is arithmetic alone
    del st
    shape32 = replace(cfg.large, n_dec=8, dtype=bi.DT_F32, name="llama-large-8-f32")
    names = bi.tensor_names(shape32)
    w32 = {n: R.wl[n] for n in names}
    m32 = parity.make_gpu_model(shape32, w32)
    small32 = replace(cfg.small, n_dec=1, dtype=bi.DT_F32)
    ms32 = parity.make_gpu_model(small32, {n: R.ws[n] for n in bi.tensor_names(small32)})
    pair32 = pkg.Pair(ms32, m32)
    st32 = pkg.State(pair32, len(R.src), len(R.src) + 16, cfg.n_max)
    st32.encode(R.src)
    st32.debug_enable_logits(True)
    st32.large_verify(INF, draft=block)
    o32 = oracle.Model(shape32, w32, compact=True)
    z32 = oracle.model.DecoderCache(o32, [], len(y) + 1).step(y, last=6)
    rel = max(float(np.max(np.abs(st32.debug_logits(pkg.LARGE, i) - z32[i]))) for i in range(6)) / float(np.max(np.abs(z32)))
    print("fp32 storage, 8 layers: logit error relative to the largest logit", rel, flush=True)
    assert rel <= 3e-6, rel


@pytest.mark.timeout(900)
def test_llama_config_full_size_in_the_launch_configuration_of_the_benchmark():
    """Config 4 exactly as `bench.py --workload llama` runs it: prompt of 1024 Zipf ids (prefilled in one pass by the
    dense-tile kernel), 256 new tokens, alpha_FB 0.5 / alpha_RB 2, n_max 10, every pass a replayed graph.  The oracle
    cannot follow at this size (the shortened-prompt test above compares its rows element by element), so this test
    holds the run to what is true at any size:
      * the loop is the composition of the calls: the same request driven through bild_small_step / bild_large_verify
        by Algorithm 1 written out here gives the same tokens and the same counters as bild_generate;
      * alpha_FB = 0 without a cap is the small model's greedy output and never runs the large model; alpha_FB > 1 is the
        large model's greedy output for any alpha_RB (the limiting cases of Sections 3.3 / 3.4);
      * every accepted draft passed both tests: replaying the final sequence, each token produced by a small step has
        max p_S >= alpha_FB there, and each reviewed draft that was kept has -ln p_L <= alpha_RB (read back from the review);
      * the prompt's cache does not depend on how it was filled: cutting the large model's cache to 700 rows makes the
        next pass recompute rows 700..1023 in row-block launches (fewer than 513 rows) instead of the dense-tile kernel, and the next token's
        distribution stays within the storage-rounding noise measured above (0.1) with the same argmax;
      * the same request twice gives the same bits."""
    R = llama_rig()
    cfg = bi.llama_pair()
    src = bi.make_source(cfg)
    n0, n = len(src), cfg.max_new
    fb, rb = cfg.alpha_fb, cfg.alpha_rb
    st = pkg.State(R.pair, n0, n0 + n + 2, cfg.n_max)
    toks, stats = st.generate(src, fb, rb, n)
    assert len(toks) == n and stats["n_generated"] == n and stats["large_calls"] > 0 and stats["rollbacks"] > 0
    st.seq_truncate(n0)
    assert st.generate(None, fb, rb, n) == (toks, stats)
    # Algorithm 1 through the calls
    st.seq_truncate(n0)
    small_steps = large_calls = rollbacks = discarded = rows = 0
    kept_pmax, kept_nll = [], []
    while st.lengths()["y_len"] - n0 < n:
        tok, flag, pmax = st.small_step(fb)
        small_steps += 1
        if not flag:
            kept_pmax.append(pmax)
            continue
        before = st.lengths()
        pending = before["y_len"] - before["draft_start"]
        out, r, nll = st.large_verify(rb)
        large_calls += 1
        rows += pending + 1
        rollbacks += int(r < pending)
        discarded += pending - r
        kept_nll.extend(float(v) for v in nll[:r])
        assert all(float(v) <= rb for v in nll[:r]) and (r == pending or float(nll[r]) > rb)
    assert st.sequence()[n0:n0 + n] == toks
    assert (small_steps, large_calls, rows, rollbacks, discarded) == (
        stats["small_steps"], stats["large_calls"], stats["rows_verified"], stats["rollbacks"], stats["tokens_discarded"])
    assert min(kept_pmax) >= fb and len(kept_nll) > 0
    # limiting cases
    st0 = pkg.State(R.pair, n0, n0 + n + 2, 0)
    small_greedy = st0.greedy(pkg.SMALL, src, 64)
    t0, s0 = st0.generate(src, 0.0, rb, 64)
    assert t0 == small_greedy and s0["large_calls"] == 0
    large_greedy = st.greedy(pkg.LARGE, src, 48)
    for rb_any in (-1.0, INF):
        t1, s1 = st.generate(src, 2.0, rb_any, 48)
        assert t1 == large_greedy and s1["rollbacks"] == 0 and s1["large_calls"] == 48
    # the prompt's cache filled by the dense-tile kernel / recomputed in row blocks
    st.encode(src)
    st.debug_enable_logits(True)
    st.large_verify(INF, draft=[])
    za = st.debug_logits(pkg.LARGE, 0).copy()
    st.force_tokens(n0, [], n0)
    st.kv_truncate(pkg.LARGE, 700)
    st.large_verify(INF, draft=[])
    zb = st.debug_logits(pkg.LARGE, 0)
    print("config 4 full size:", stats, "next-token logits, dense prefill against row-block recompute:",
          float(np.max(np.abs(za - zb))), "of", float(np.max(np.abs(za))), flush=True)
    assert int(np.argmax(za)) == int(np.argmax(zb)) and np.max(np.abs(za - zb)) <= 0.1
    _llama.clear()


@pytest.mark.timeout(1500)
def test_verify_stress_7b_widths_cache_of_4096_rows():
    """Config 5 (review-pass stress) at the 7B-shaped large model's full widths with 4 of its layers, so that
    the oracle stays affordable: a cache of 4095 prompt rows, review passes of T = n+1 in {1, 4, 8, 16, 32} rows
    (many key splits joined by the merge kernel), the large cache cut back to a random row between passes (the
    next pass first recomputes the cut rows in row-block launches).  Sampled rows of every pass against the
    oracle's cached forward; one block also against T single-row passes (Section 3.2: one pass over n tokens
    equals n sequential steps)."""
    from dataclasses import replace
    base = bi.llama_pair()
    large = replace(base.large, n_dec=4, name="llama-large-4")
    small = replace(base.small, n_dec=1, name="llama-small-1")
    cfg = replace(base, name="verify-stress", small=small, large=large, n_src=4096, max_new=40)
    R = Rig(cfg, compact=True)
    tol = parity.logit_tol(cfg)
    n0 = R.n0
    assert pkg.binding.attn_shape(large.heads, large.d_head, 8, n0 + 8, 8, 1)["splits"] >= 8
    st = pkg.State(R.pair, n0, n0 + 40, 31)
    st.encode(R.src)
    st.debug_enable_logits(True)
    cache = oracle.model.DecoderCache(R.req.large, [], n0 + 40)
    prompt = [int(t) for t in R.src]
    cache.step(prompt[:n0 - 1], last=0)
    rng = np.random.default_rng(17)
    worst = 0.0
    for n in (0, 3, 7, 15, 31, 7):
        block = [int(t) for t in bi.make_tokens(large.vocab, n, seed=200 + n)]
        out, r, nll = st.large_verify(INF, draft=block)            # never roll back
        assert r == n and out[:n] == block
        have = cache.length
        z = cache.step(prompt[have:] + block, last=n + 1)           # catches up on rows cut earlier, then the block
        for i in sorted({0, n // 2, n}):
            zi = st.debug_logits(pkg.LARGE, i)
            err = float(np.max(np.abs(zi - z[i])))
            worst = max(worst, err)
            assert err <= tol, (n, i, err)
            if i < n:
                assert abs(float(nll[i]) - oracle.policy.nll(z[i], block[i])) <= 2 * tol
        assert out[n] == int(np.argmax(z[n])) or oracle.policy.top2_gap(z[n]) < parity.MARGIN
        if n == 7:
            # the same block one row per pass: the distributions of sequential steps
            rows = [st.debug_logits(pkg.LARGE, i) for i in range(n + 1)]
            for i in range(n + 1):
                st.force_tokens(n0, block[:i], n0 + i)
                out1, _, _ = st.large_verify(INF, draft=[])
                z1 = st.debug_logits(pkg.LARGE, 0)
                assert np.max(np.abs(z1 - rows[i])) <= 5e-3, (i, float(np.max(np.abs(z1 - rows[i]))))
                assert out1[0] == int(np.argmax(z1))
        # cut the large model's cache at a random row near the end of the prompt, the sequence back to the prompt
        cut = int(rng.integers(n0 - 300, n0 - 1))
        st.force_tokens(n0, [], n0)
        st.kv_truncate(pkg.LARGE, cut)
        assert st.lengths()["len_large"] == cut
        cache.truncate(cut)
    print("verify stress: worst logit error", worst, "bar", tol, flush=True)
