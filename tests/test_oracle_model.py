"""Pins for oracle/model.py.

Each primitive is held to a library routine (torch, float64) or a closed form;
the layer wiring is held to a decoder assembled from torch modules; the cached
and T-row forms are held to the no-cache definition (Section 3.2: one pass over
n rows gives the distributions of n sequential steps)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import bild_inputs as bi
from oracle import model as om

torch.set_default_dtype(torch.float64)
RNG = np.random.default_rng(42)


# ---------------------------------------------------------------- primitives
def test_round_bf16_matches_library_and_ties_to_even():
    a = (RNG.standard_normal(50000) * np.exp(RNG.uniform(-30, 30, 50000))).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(om.round_bf16(a.astype(np.float64)), ref)
    assert om.round_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0                   # tie -> even (down)
    assert om.round_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6     # tie -> even (up)
    assert om.round_bf16(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1 + 2.0 ** -7
    assert om.round_bf16(np.array([0.0, -2.5]))[0] == 0.0


def test_rmsnorm_matches_library():
    x = RNG.standard_normal((5, 48))
    g = RNG.standard_normal(48)
    ref = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.allclose(om.rmsnorm(x, g, 1e-6), ref, rtol=1e-13, atol=1e-14)
    # closed form: a constant row has rms |c|
    assert np.allclose(om.rmsnorm(np.full((1, 8), -3.0), np.ones(8), 0.0), -1.0)


def test_activations_match_library():
    u = RNG.standard_normal(1000) * 3
    t = torch.from_numpy(u)
    assert np.allclose(om.gelu_tanh(u), F.gelu(t, approximate="tanh").numpy(), rtol=1e-13, atol=1e-15)
    assert np.allclose(om.silu(u), F.silu(t).numpy(), rtol=1e-13, atol=1e-15)


def test_sinusoid_closed_form():
    d = 12
    pe = om.sinusoid(np.array([0, 1, 5]), d)
    assert np.allclose(pe[0, 0::2], 0) and np.allclose(pe[0, 1::2], 1)
    assert abs(pe[1, 0] - math.sin(1.0)) < 1e-15 and abs(pe[1, 1] - math.cos(1.0)) < 1e-15
    i = d // 2 - 1
    assert abs(pe[2, 2 * i] - math.sin(5.0 / 10000 ** (2 * i / d))) < 1e-15
    assert abs(pe[2, 2 * i + 1] - math.cos(5.0 / 10000 ** (2 * i / d))) < 1e-15


def test_rope_properties():
    h, dh = 3, 8
    x = RNG.standard_normal((4, h * dh))
    y = RNG.standard_normal((4, h * dh))
    pos = np.array([0, 1, 7, 30])
    rx = om.rope(x, pos, h, dh, 10000.0)
    assert np.allclose(rx[0], x[0])                                         # position 0: identity
    assert np.allclose(np.linalg.norm(rx.reshape(4, h, dh), axis=2), np.linalg.norm(x.reshape(4, h, dh), axis=2))
    # first pair rotates by exactly `position` radians, the last by position * base^(-(dh-2)/dh)
    c, s = math.cos(7.0), math.sin(7.0)
    assert np.allclose(rx[2, :2], [x[2, 0] * c - x[2, 1] * s, x[2, 0] * s + x[2, 1] * c])
    a = 30.0 * 10000.0 ** (-(dh - 2) / dh)
    c, s = math.cos(a), math.sin(a)
    assert np.allclose(rx[3, dh - 2:dh], [x[3, dh - 2] * c - x[3, dh - 1] * s, x[3, dh - 2] * s + x[3, dh - 1] * c])
    # scores depend on the position difference only
    q1 = om.rope(x[:1], np.array([9]), h, dh, 10000.0)
    k1 = om.rope(y[:1], np.array([4]), h, dh, 10000.0)
    q2 = om.rope(x[:1], np.array([25]), h, dh, 10000.0)
    k2 = om.rope(y[:1], np.array([20]), h, dh, 10000.0)
    assert np.allclose((q1.reshape(h, dh) * k1.reshape(h, dh)).sum(1), (q2.reshape(h, dh) * k2.reshape(h, dh)).sum(1))


def _sdpa(q, k, v, heads, dh, mask):
    tq = torch.from_numpy(q).reshape(q.shape[0], heads, dh).transpose(0, 1)
    tk = torch.from_numpy(k).reshape(k.shape[0], heads, dh).transpose(0, 1)
    tv = torch.from_numpy(v).reshape(v.shape[0], heads, dh).transpose(0, 1)
    o = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)
    return o.transpose(0, 1).reshape(q.shape[0], heads * dh).numpy()


def test_attention_matches_library_sdpa():
    heads, dh, t, p = 3, 8, 4, 11
    q = RNG.standard_normal((t, heads * dh))
    k = RNG.standard_normal((p, heads * dh))
    v = RNG.standard_normal((p, heads * dh))
    assert np.allclose(om.attention(q, k, v, heads, dh, None), _sdpa(q, k, v, heads, dh, None), rtol=1e-12, atol=1e-13)
    qpos = np.arange(p - t, p)                      # the T new rows sit at the end of the cache
    mask = torch.from_numpy(np.arange(p)[None, :] <= qpos[:, None])
    assert np.allclose(om.attention(q, k, v, heads, dh, qpos), _sdpa(q, k, v, heads, dh, mask), rtol=1e-12, atol=1e-13)


def test_attention_zero_query_is_prefix_mean():
    heads, dh, p = 2, 4, 6
    k = RNG.standard_normal((p, heads * dh))
    v = RNG.standard_normal((p, heads * dh))
    out = om.attention(np.zeros((p, heads * dh)), k, v, heads, dh, np.arange(p))
    for r in range(p):
        assert np.allclose(out[r], v[:r + 1].mean(axis=0))


def _one_hot_table(heads, dmax, offsets):
    """Bias table that is 0 at one signed distance per head and -1e9 elsewhere."""
    t = np.full((heads, 2 * dmax + 1), -1e9)
    for h, r in enumerate(offsets):
        t[h, r + dmax] = 0.0
    return t


def test_relative_bias_selects_keys_by_signed_distance():
    """Closed forms.  A table that admits a single distance turns attention into a shift of V: head 0
    looks one key back, head 1 two keys ahead (not causal).  Rows whose admitted key does not exist see
    every key at the same (huge negative) bias and q = 0, i.e. the plain mean."""
    heads, dh, p, dmax = 2, 4, 9, 3
    v = RNG.standard_normal((p, heads * dh))
    k = RNG.standard_normal((p, heads * dh))
    q = 0.3 * RNG.standard_normal((p, heads * dh))     # finite scores cannot compete with 1e9
    pos = np.arange(p)
    out = om.attention(q, k, v, heads, dh, None, _one_hot_table(heads, dmax, (-1, 2)), pos)
    for r in range(1, p):
        assert np.allclose(out[r, :dh], v[r - 1, :dh], atol=1e-9)
    for r in range(p - 2):
        assert np.allclose(out[r, dh:], v[r + 2, dh:], atol=1e-9)
    out0 = om.attention(np.zeros_like(q), k, v, heads, dh, None, _one_hot_table(heads, dmax, (-1, 2)), pos)
    assert np.allclose(out0[0, :dh], v[:, :dh].mean(axis=0))
    assert np.allclose(out0[p - 1, dh:], v[:, dh:].mean(axis=0))


def test_relative_bias_clamps_far_distances_and_respects_the_causal_mask():
    """Admitting only the clamped end of the table (-D) gives the mean over every key at least D back;
    under the causal mask an admitted FUTURE distance never shows, so the row falls back to the mean of
    its visible prefix; row positions are absolute (a block of new rows at the end of a cache)."""
    heads, dh, p, dmax, t = 2, 4, 12, 3, 5
    v = RNG.standard_normal((p, heads * dh))
    k = RNG.standard_normal((p, heads * dh))
    pos = np.arange(p - t, p)
    out = om.attention(np.zeros((t, heads * dh)), k, v, heads, dh, pos, _one_hot_table(heads, dmax, (-dmax, 1)), pos)
    for i, r in enumerate(pos):
        assert np.allclose(out[i, :dh], v[:r - dmax + 1, :dh].mean(axis=0))
        assert np.allclose(out[i, dh:], v[:r + 1, dh:].mean(axis=0))


def test_relative_bias_matches_library_sdpa_with_an_additive_mask():
    heads, dh, t, p, dmax = 3, 8, 4, 11, 2
    q, k, v = (RNG.standard_normal((n, heads * dh)) for n in (t, p, p))
    table = RNG.standard_normal((heads, 2 * dmax + 1))
    qpos = np.arange(p - t, p)
    add = np.zeros((heads, t, p))
    for h in range(heads):
        for r in range(t):
            for c in range(p):
                add[h, r, c] = table[h, min(max(c - int(qpos[r]), -dmax), dmax) + dmax] if c <= qpos[r] else -np.inf
    ref = _sdpa(q, k, v, heads, dh, torch.from_numpy(add))
    assert np.allclose(om.attention(q, k, v, heads, dh, qpos, table, qpos), ref, rtol=1e-12, atol=1e-13)


def test_relative_models_see_order_only_through_the_table():
    """With an all-zero table a relative-position encoder is permutation equivariant (nothing else
    carries position); with the drawn table it is not."""
    cfg = bi.toy_pair(pos=bi.POS_RELATIVE)
    _, wl = bi.make_pair_weights(cfg)
    src = bi.make_source(cfg)
    perm = np.random.default_rng(3).permutation(len(src))
    m = om.Model(cfg.large, wl)
    assert not np.allclose(m.encode(src[perm]), m.encode(src)[perm], atol=1e-6)
    wz = dict(wl, enc_rel_bias=np.zeros_like(wl["enc_rel_bias"]))
    mz = om.Model(cfg.large, wz)
    assert np.allclose(mz.encode(src[perm]), mz.encode(src)[perm], rtol=1e-10, atol=1e-12)


def test_synthetic_bias_tables_tie_distances_in_log_spaced_ranges():
    from bild_inputs.generate import distance_ties
    one = distance_ties(128, 32, False)
    back = one[:129][::-1]                                 # distances 0, 1, ..., 128 behind the query
    assert list(back[:16]) == list(range(16)) and back[128] == 31 and np.all(np.diff(back) >= 0)
    assert len(set(back)) == 32 and np.all(one[129:] == 0)
    widths = np.bincount(back)[16:31]
    assert widths[-1] >= 4 * widths[0] and np.all(widths[8:] > widths[:7].max() - 1)   # ranges grow with distance
    assert back[112] == 30 and back[113] == 31             # 16 * 8^(15/16) = 112.4: the last value starts at 113
    two = distance_ties(128, 32, True)
    assert np.array_equal(two[129:] - 16, two[:128][::-1]) and two[128] == 0 and len(set(two)) == 31
    cfg = bi.toy_pair(pos=bi.POS_RELATIVE, truncate=True)
    ws, wl = bi.make_pair_weights(cfg)
    for name, two_sided in (("enc_rel_bias", True), ("dec_rel_bias", False)):
        tab = wl[name]
        ties = distance_ties(cfg.large.rel_max_dist, cfg.large.rel_buckets, two_sided)
        assert tab.shape == (cfg.large.heads, 2 * cfg.large.rel_max_dist + 1) and tab.dtype == np.float32
        for a in range(len(ties)):
            for b in range(len(ties)):
                assert (ties[a] == ties[b]) == bool(np.all(tab[:, a] == tab[:, b]))
        assert np.array_equal(ws[name], tab[:cfg.small.heads])


# ------------------------------------------------------- wiring vs torch modules
def _torch_decoder(shape, w, y, cross_src):
    """A pre-norm decoder assembled from library modules (nn.MultiheadAttention,
    F.rms_norm, F.linear).  Only valid for heads*d_head == d, ReLU, sinusoidal."""
    d, h = shape.d, shape.heads
    tw = {k: torch.from_numpy(np.asarray(a, dtype=np.float64)) for k, a in w.items()}

    def mha(pre, names, xq, xkv, mask):
        m = torch.nn.MultiheadAttention(d, h, bias=False, batch_first=False, dtype=torch.float64)
        with torch.no_grad():
            m.in_proj_weight.copy_(torch.cat([tw[pre + n].T for n in names[:3]], 0))
            m.out_proj.weight.copy_(tw[pre + names[3]].T)
        return m(xq[:, None], xkv[:, None], xkv[:, None], attn_mask=mask, need_weights=False)[0][:, 0]

    n = len(y)
    pos = torch.arange(n, dtype=torch.float64)
    i = torch.arange(d // 2, dtype=torch.float64)
    ang = pos[:, None] / (10000.0 ** (2 * i / d))[None]
    pe = torch.stack([ang.sin(), ang.cos()], -1).reshape(n, d)
    rows = (torch.tensor(y) + shape.tie_shift) % shape.vocab
    x = shape.embed_scale * F.embedding(rows, tw["emb"]) + pe
    causal = torch.triu(torch.ones(n, n, dtype=torch.bool), 1)        # True = masked
    with torch.no_grad():
        for l in range(shape.n_dec):
            p = f"dec.{l}."
            xn = F.rms_norm(x, (d,), tw[p + "ln1"], eps=shape.eps)
            x = x + mha(p, ("wq", "wk", "wv", "wo"), xn, xn, causal)
            xn = F.rms_norm(x, (d,), tw[p + "lnc"], eps=shape.eps)
            x = x + mha(p, ("cwq", "cwk", "cwv", "cwo"), xn, cross_src, None)
            xn = F.rms_norm(x, (d,), tw[p + "ln2"], eps=shape.eps)
            x = x + F.linear(F.relu(F.linear(xn, tw[p + "w_in"].T)), tw[p + "w_out"].T)
        xn = F.rms_norm(x, (d,), tw["dec_final_norm"], eps=shape.eps)
        return (shape.logit_scale * F.linear(xn, tw["emb"])).numpy()


def test_decoder_wiring_matches_torch_modules():
    cfg = bi.toy_pair(d=32, heads=2, d_head=16, d_ff=40, vocab=50)
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    enc = RNG.standard_normal((7, 32))                 # any memory: the encoder is pinned separately
    y = [0, 13, 49, 2, 2, 31]
    ours = m.logits_full(y, m.cross_kv(enc))
    ref = _torch_decoder(cfg.large, wl, y, torch.from_numpy(enc))
    assert np.allclose(ours, ref, rtol=1e-11, atol=1e-11)


def test_encoder_layer_matches_torch_modules():
    cfg = bi.toy_pair(d=32, heads=2, d_head=16, d_ff=40, vocab=50)
    _, wl = bi.make_pair_weights(cfg)
    shape = cfg.large
    m = om.Model(shape, wl)
    src = [5, 9, 0, 44, 17]
    ours = m.encode(src)
    tw = {k: torch.from_numpy(np.asarray(a, dtype=np.float64)) for k, a in wl.items()}
    d = shape.d
    x = torch.from_numpy(m.embed(src, np.arange(len(src))))       # embed is pinned by its own test
    with torch.no_grad():
        for l in range(shape.n_enc):
            p = f"enc.{l}."
            mha = torch.nn.MultiheadAttention(d, shape.heads, bias=False, dtype=torch.float64)
            mha.in_proj_weight.copy_(torch.cat([tw[p + n].T for n in ("wq", "wk", "wv")], 0))
            mha.out_proj.weight.copy_(tw[p + "wo"].T)
            xn = F.rms_norm(x, (d,), tw[p + "ln1"], eps=shape.eps)
            x = x + mha(xn[:, None], xn[:, None], xn[:, None], need_weights=False)[0][:, 0]
            xn = F.rms_norm(x, (d,), tw[p + "ln2"], eps=shape.eps)
            x = x + F.linear(F.relu(F.linear(xn, tw[p + "w_in"].T)), tw[p + "w_out"].T)
        ref = F.rms_norm(x, (d,), tw["enc_final_norm"], eps=shape.eps).numpy()
    assert np.allclose(ours, ref, rtol=1e-11, atol=1e-11)


def test_embed_closed_form_and_tie_shift():
    cfg = bi.toy_pair()
    _, wl = bi.make_pair_weights(cfg)
    s = cfg.large
    m = om.Model(s, wl)
    x = m.embed([3, s.vocab - 1], np.array([0, 4]))
    e0 = s.embed_scale * wl["emb"][(3 + s.tie_shift) % s.vocab].astype(np.float64)
    e0[1::2] += 1.0                                         # PE(0) = (0, 1, 0, 1, ...)
    assert np.allclose(x[0], e0, rtol=0, atol=1e-15)
    assert abs(x[1, 0] - (s.embed_scale * float(wl["emb"][(s.vocab - 1 + s.tie_shift) % s.vocab, 0]) + math.sin(4.0))) < 1e-14


def test_gated_ffn_matches_library_composition():
    for act, fn in ((bi.ACT_GATED_GELU, lambda t: F.gelu(t, approximate="tanh")), (bi.ACT_SWIGLU, F.silu)):
        cfg = bi.toy_pair(act=act)
        _, wl = bi.make_pair_weights(cfg)
        m = om.Model(cfg.large, wl)
        xn = RNG.standard_normal((3, cfg.large.d))
        t = torch.from_numpy(xn)
        w = {k: torch.from_numpy(wl["dec.1." + k].astype(np.float64)) for k in ("w_in", "w_up", "w_out")}
        ref = F.linear(fn(F.linear(t, w["w_in"].T)) * F.linear(t, w["w_up"].T), w["w_out"].T).numpy()
        assert np.allclose(m.ffn("dec.1.", xn), ref, rtol=1e-12, atol=1e-14)


def test_zeroed_sublayers_reduce_to_embedding_times_head():
    cfg = bi.toy_pair(tied=False)
    _, wl = bi.make_pair_weights(cfg)
    for k in wl:
        if k.endswith((".wo", ".cwo", ".w_out")):
            wl[k] = np.zeros_like(wl[k])
    s = cfg.large
    m = om.Model(s, wl)
    y = [0, 7, 150]
    z = m.logits_full(y, m.cross_kv(RNG.standard_normal((4, s.d))))
    x = s.embed_scale * wl["emb"][y].astype(np.float64) + om.sinusoid(np.arange(3), s.d)
    xn = x / np.sqrt((x * x).mean(1, keepdims=True) + s.eps) * wl["dec_final_norm"]
    assert np.allclose(z, s.logit_scale * xn @ wl["head"].astype(np.float64).T, rtol=1e-12, atol=1e-12)


# ------------------------------------------------ cached / T-row == definition
VARIANTS = [
    dict(),
    dict(dtype=bi.DT_BF16),
    dict(act=bi.ACT_GATED_GELU, tied=False),
    dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False),
    dict(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False, dtype=bi.DT_BF16),
    dict(truncate=True, dtype=bi.DT_BF16),
    dict(pos=bi.POS_RELATIVE),
    dict(pos=bi.POS_RELATIVE, truncate=True, dtype=bi.DT_BF16, act=bi.ACT_GATED_GELU),
    dict(pos=bi.POS_RELATIVE, cross=False, tied=False),
]


@pytest.mark.parametrize("kw", VARIANTS)
def test_cached_and_block_passes_equal_the_definition(kw):
    cfg = bi.toy_pair(**kw)
    ws, wl = bi.make_pair_weights(cfg)
    for shape, w in ((cfg.large, wl), (cfg.small, ws)):
        m = om.Model(shape, w)
        if shape.cross:
            enc = m.encode(bi.make_source(cfg)) if shape.n_enc else RNG.standard_normal((cfg.n_src, shape.d))
            cross = m.cross_kv(enc)
        else:
            cross = []
        y = [int(t) for t in bi.make_tokens(shape.vocab, 13, seed=5)]
        full = m.logits_full(y, cross)
        # one row at a time
        c = om.DecoderCache(m, cross, 32)
        seq = np.stack([c.step([t])[0] for t in y])
        assert np.allclose(seq, full, rtol=1e-12, atol=1e-12)
        # ragged blocks: 1, 5, 1, 6 rows (a T-row pass equals T sequential steps)
        c = om.DecoderCache(m, cross, 32)
        blocks, at = [], 0
        for n in (1, 5, 1, 6):
            blocks.append(c.step(y[at:at + n]))
            at += n
        assert np.allclose(np.concatenate(blocks), full, rtol=1e-12, atol=1e-12)
        # the `last` option only drops rows of the result
        c2 = om.DecoderCache(m, cross, 32)
        assert c2.step(y[:6], last=0).shape == (0, shape.vocab)
        assert np.allclose(c2.step(y[6:], last=3), full[-3:], rtol=1e-12, atol=1e-12) and c2.length == len(y)
        # truncate, then continue with different tokens == fresh run on the new prefix
        c.truncate(4)
        y2 = y[:4] + [int(t) for t in bi.make_tokens(shape.vocab, 5, seed=6)]
        again = c.step(y2[4:])
        assert np.allclose(again, m.logits_full(y2, cross)[4:], rtol=1e-12, atol=1e-12)


def test_cache_store_hook_only_replaces_the_storage_rounding():
    """`DecoderCache(store=...)` hands every new K / V block (exact values, layer, kind, first row) to the caller and
    caches what comes back.  The model's own rounding supplied through the hook is the plain cache bit for bit; in a
    bf16 model the identity hook is the fp32-storage forward (no rounding anywhere), which differs from the bf16 one."""
    cfg = bi.toy_pair(dtype=bi.DT_BF16, pos=bi.POS_ROPE, cross=False, tied=False, act=bi.ACT_SWIGLU)
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    y = [int(t) for t in bi.make_tokens(cfg.large.vocab, 11, seed=3)]
    c0 = om.DecoderCache(m, [], 16)
    plain = np.concatenate([c0.step(y[:4]), c0.step(y[4:])])
    seen = []

    def own(l, kind, exact, t0):
        seen.append((l, kind, exact.shape, t0))
        return om.round_bf16(exact)

    c = om.DecoderCache(m, [], 16, store=own)
    hooked = np.concatenate([c.step(y[:4]), c.step(y[4:])])
    assert np.array_equal(hooked, plain)
    inner = cfg.large.inner
    assert seen[:2] == [(0, "k", (4, inner), 0), (0, "v", (4, inner), 0)] and seen[-1] == (cfg.large.n_dec - 1, "v", (7, inner), 4)
    assert len(seen) == 2 * 2 * cfg.large.n_dec
    c1 = om.DecoderCache(m, [], 16, store=lambda l, kind, exact, t0: exact)
    unrounded = np.concatenate([c1.step(y[:4]), c1.step(y[4:])])
    from dataclasses import replace
    c32 = om.DecoderCache(om.Model(replace(cfg.large, dtype=bi.DT_F32), wl), [], 16)
    assert np.array_equal(unrounded, np.concatenate([c32.step(y[:4]), c32.step(y[4:])]))
    assert np.max(np.abs(unrounded - plain)) > 1e-6


def test_causality_and_encoder_bidirectionality():
    cfg = bi.toy_pair()
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    src = [int(t) for t in bi.make_source(cfg)]
    e1 = m.encode(src)
    src2 = list(src)
    src2[-1] = (src2[-1] + 1) % cfg.large.vocab
    e2 = m.encode(src2)
    assert np.abs(e1[0] - e2[0]).max() > 1e-6           # the first source position sees the last one
    cross = m.cross_kv(e1)
    y = [0, 5, 9, 11, 3]
    z1 = m.logits_full(y, cross)
    y2 = list(y)
    y2[3] = 12
    z2 = m.logits_full(y2, cross)
    assert np.array_equal(z1[:3], z2[:3])               # rows before the change are untouched
    assert np.abs(z1[3:] - z2[3:]).max() > 1e-6


def test_compact_storage_gives_identical_values():
    cfg = bi.toy_pair(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False, dtype=bi.DT_BF16)
    _, wl = bi.make_pair_weights(cfg)
    y = [1, 2, 3, 100]
    a = om.Model(cfg.large, wl).logits_full(y, [])
    b = om.Model(cfg.large, wl, compact=True).logits_full(y, [])
    assert np.allclose(a, b, rtol=1e-13, atol=1e-13)      # same values; only the BLAS call pattern differs


# ------------------------------------------- RoPE / decoder-only wiring vs library pieces
def _polar_rotate(t: torch.Tensor, positions, heads: int, dh: int, base: float) -> torch.Tensor:
    """Rotary position by an explicit complex multiply: pair (2i, 2i+1) of every head is read as the
    complex number a + ib and multiplied by the unit number of angle position * base^(-2i/d_head)."""
    n = t.shape[0]
    z = torch.view_as_complex(t.reshape(n, heads, dh // 2, 2).contiguous())
    i = torch.arange(dh // 2, dtype=torch.float64)
    ang = torch.as_tensor(positions, dtype=torch.float64)[:, None] * base ** (-2.0 * i / dh)[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.view_as_real(z * rot).reshape(n, heads * dh)


def _library_bf16(t: torch.Tensor) -> torch.Tensor:
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _torch_rope_stack(shape, w, tokens, causal: bool, prefix: str, store_bf16: bool):
    """A pre-norm stack assembled from F.rms_norm, F.linear, F.silu / F.gelu / F.relu and
    F.scaled_dot_product_attention, with q and k rotated by _polar_rotate and v left alone.  K and V are
    rounded to bf16 AFTER the rotation when store_bf16.  Calls nothing of the oracle.  Returns the hidden
    state [n, d] after the last layer (no final norm)."""
    d, h, dh = shape.d, shape.heads, shape.d_head
    tw = {k: torch.from_numpy(np.asarray(a, dtype=np.float64)) for k, a in w.items()}
    n = len(tokens)
    pos = list(range(n))
    rows = (torch.tensor(list(tokens), dtype=torch.int64) + shape.tie_shift) % shape.vocab
    x = shape.embed_scale * F.embedding(rows, tw["emb"])             # rotary models add nothing to the embedding
    n_layers = shape.n_dec if prefix == "dec" else shape.n_enc
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool)) if causal else None     # True = visible
    for l in range(n_layers):
        p = f"{prefix}.{l}."
        xn = F.rms_norm(x, (d,), tw[p + "ln1"], eps=shape.eps)
        q = _polar_rotate(F.linear(xn, tw[p + "wq"].T), pos, h, dh, shape.rope_base)
        k = _polar_rotate(F.linear(xn, tw[p + "wk"].T), pos, h, dh, shape.rope_base)
        v = F.linear(xn, tw[p + "wv"].T)
        if store_bf16:
            k, v = _library_bf16(k), _library_bf16(v)
        split = lambda a: a.reshape(n, h, dh).transpose(0, 1)
        o = F.scaled_dot_product_attention(split(q), split(k), split(v), attn_mask=mask)
        x = x + F.linear(o.transpose(0, 1).reshape(n, h * dh), tw[p + "wo"].T)
        xn = F.rms_norm(x, (d,), tw[p + "ln2"], eps=shape.eps)
        u = F.linear(xn, tw[p + "w_in"].T)
        if shape.act == bi.ACT_RELU:
            hid = F.relu(u)
        else:
            gate = F.silu(u) if shape.act == bi.ACT_SWIGLU else F.gelu(u, approximate="tanh")
            hid = gate * F.linear(xn, tw[p + "w_up"].T)
        x = x + F.linear(hid, tw[p + "w_out"].T)
    return x, tw


def _torch_rope_decoder_logits(shape, w, y, store_bf16):
    x, tw = _torch_rope_stack(shape, w, y, True, "dec", store_bf16)
    xn = F.rms_norm(x, (shape.d,), tw["dec_final_norm"], eps=shape.eps)
    return (shape.logit_scale * F.linear(xn, tw["emb" if shape.tied else "head"])).numpy()


@pytest.mark.parametrize("tied", [False, True])
def test_decoder_only_rope_swiglu_wiring_matches_library_pieces(tied):
    """The decoder-only RoPE + SwiGLU stack (the shape family of the 7B-shaped configurations) against an
    assembly of library pieces that never calls the oracle's own rotation: q and k rotated, v not, causal
    mask, residual order, head.  Both routes of the oracle (definition and cached T-row passes)."""
    cfg = bi.toy_pair(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=tied, d=32, heads=3, d_head=8, d_ff=40, vocab=61)
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    y = [0, 13, 60, 2, 2, 31, 7, 19, 44]
    ref = _torch_rope_decoder_logits(cfg.large, wl, y, store_bf16=False)
    assert np.allclose(m.logits_full(y, []), ref, rtol=1e-11, atol=1e-11)
    c = om.DecoderCache(m, [], 16)
    blocks = np.concatenate([c.step(y[:1]), c.step(y[1:6]), c.step(y[6:])])
    assert np.allclose(blocks, ref, rtol=1e-11, atol=1e-11)


def test_bf16_rope_models_round_k_after_the_rotation_and_leave_q_unrounded():
    """bf16 storage: K and V are rounded (library conversion) after the rotation; q, the scores and
    everything else stay unrounded.  Rounding before the rotation, or rounding q too, moves the logits by
    far more than the tolerance used here."""
    cfg = bi.toy_pair(act=bi.ACT_SWIGLU, pos=bi.POS_ROPE, cross=False, tied=False, d=32, heads=3, d_head=8, d_ff=40,
                      vocab=61, dtype=bi.DT_BF16)
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    y = [5, 13, 60, 2, 9, 31, 7, 19, 44, 3, 3, 58]
    ref = _torch_rope_decoder_logits(cfg.large, wl, y, store_bf16=True)
    ours = m.logits_full(y, [])
    assert np.allclose(ours, ref, rtol=1e-11, atol=1e-11)
    # the rounding is visible at all (else this test would not tell the orders apart) ...
    unrounded = _torch_rope_decoder_logits(cfg.large, wl, y, store_bf16=False)
    assert np.abs(unrounded - ref).max() > 1e-5
    # ... and so is its place: the same assembly with K rounded BEFORE the rotation differs
    d, h, dh, s = cfg.large.d, cfg.large.heads, cfg.large.d_head, cfg.large
    tw = {k: torch.from_numpy(np.asarray(a, dtype=np.float64)) for k, a in wl.items()}
    xn = F.rms_norm(s.embed_scale * F.embedding((torch.tensor(y) + s.tie_shift) % s.vocab, tw["emb"]), (d,),
                    tw["dec.0.ln1"], eps=s.eps)
    k_raw = F.linear(xn, tw["dec.0.wk"].T)
    pos = list(range(len(y)))
    after = _library_bf16(_polar_rotate(k_raw, pos, h, dh, s.rope_base)).numpy()
    before = _polar_rotate(_library_bf16(k_raw), pos, h, dh, s.rope_base).numpy()
    assert np.abs(after - before).max() > 1e-6
    c = om.DecoderCache(m, [], 16)
    c.step(y)
    assert np.array_equal(c.k[0][:len(y)], after)                      # the cache holds rotate-then-round, bit for bit
    xv = _library_bf16(F.linear(xn, tw["dec.0.wv"].T)).numpy()
    assert np.array_equal(c.v[0][:len(y)], xv)                         # V: rounded, never rotated


def test_rope_encoder_wiring_matches_library_pieces():
    """An encoder with rotary positions (bidirectional attention, q and k rotated) against the same assembly."""
    cfg = bi.toy_pair(pos=bi.POS_ROPE, cross=True, d=32, heads=3, d_head=8, d_ff=40, vocab=61)
    _, wl = bi.make_pair_weights(cfg)
    m = om.Model(cfg.large, wl)
    src = [5, 9, 0, 44, 17, 17, 60]
    x, tw = _torch_rope_stack(cfg.large, wl, src, False, "enc", store_bf16=False)
    ref = F.rms_norm(x, (cfg.large.d,), tw["enc_final_norm"], eps=cfg.large.eps).numpy()
    assert np.allclose(m.encode(src), ref, rtol=1e-11, atol=1e-11)


def test_decoder_relative_table_turns_causal_self_attention_into_a_shift():
    """Which stack gets which table, and where: the DECODER's table admits only the key one position back
    (every other distance gets -1e9), the encoder's table only the key two ahead.  Causal self-attention of the
    decoder is then exactly a shift of V by one row (row 0 sees only itself), cross-attention carries no bias
    at all, and the logits equal those of an assembly of library pieces in which the self-attention is
    written as that shift."""
    cfg = bi.toy_pair(pos=bi.POS_RELATIVE, d=32, heads=2, d_head=16, d_ff=40, vocab=50, rel_max_dist=3)
    _, wl = bi.make_pair_weights(cfg)
    s = cfg.large
    wl = dict(wl, dec_rel_bias=_one_hot_table(s.heads, s.rel_max_dist, (-1,) * s.heads),
              enc_rel_bias=_one_hot_table(s.heads, s.rel_max_dist, (2,) * s.heads))
    m = om.Model(s, wl)
    enc = RNG.standard_normal((7, s.d))
    cross = m.cross_kv(enc)
    y = [0, 13, 49, 2, 2, 31, 8]
    n, d, h, dh = len(y), s.d, s.heads, s.d_head
    tw = {k: torch.from_numpy(np.asarray(a, dtype=np.float64)) for k, a in wl.items()}
    x = s.embed_scale * F.embedding((torch.tensor(y) + s.tie_shift) % s.vocab, tw["emb"])     # no additive position
    mem = torch.from_numpy(enc)
    split = lambda a: a.reshape(a.shape[0], h, dh).transpose(0, 1)
    for l in range(s.n_dec):
        p = f"dec.{l}."
        v = F.linear(F.rms_norm(x, (d,), tw[p + "ln1"], eps=s.eps), tw[p + "wv"].T)
        shifted = torch.cat([v[:1], v[:-1]], 0)                       # row r takes v[r-1]; row 0 only sees key 0
        x = x + F.linear(shifted, tw[p + "wo"].T)
        xn = F.rms_norm(x, (d,), tw[p + "lnc"], eps=s.eps)
        o = F.scaled_dot_product_attention(split(F.linear(xn, tw[p + "cwq"].T)), split(F.linear(mem, tw[p + "cwk"].T)),
                                           split(F.linear(mem, tw[p + "cwv"].T)))
        x = x + F.linear(o.transpose(0, 1).reshape(n, h * dh), tw[p + "cwo"].T)
        xn = F.rms_norm(x, (d,), tw[p + "ln2"], eps=s.eps)
        x = x + F.linear(F.relu(F.linear(xn, tw[p + "w_in"].T)), tw[p + "w_out"].T)
    ref = (s.logit_scale * F.linear(F.rms_norm(x, (d,), tw["dec_final_norm"], eps=s.eps), tw["emb"])).numpy()
    assert np.allclose(m.logits_full(y, cross), ref, rtol=1e-9, atol=1e-9)
    c = om.DecoderCache(m, cross, 16)
    blocks = np.concatenate([c.step(y[:2]), c.step(y[2:3]), c.step(y[3:])])
    assert np.allclose(blocks, ref, rtol=1e-9, atol=1e-9)
