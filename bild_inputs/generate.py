"""Seeded synthetic weights and token ids, handed unchanged to both the CPU
oracle and the HIP library.

Nothing here evaluates a model: tensors are drawn, optionally rounded to
bf16-representable values, and sliced.  Every tensor is an fp32 numpy array in
"math layout": a matrix W is [inputs, outputs] so that a layer computes
`x @ W`; the embedding and the LM head are [vocab, d].

Tensor names (l = layer index):
  emb, head (absent when tied), enc_final_norm, dec_final_norm
  enc_rel_bias, dec_rel_bias (relative-position models only): [heads][2*rel_max_dist + 1] fp32, entry
  [h][r + rel_max_dist] is the score bias of head h for a key r positions after the query
  enc.l.{ln1,wq,wk,wv,wo,ln2,w_in,w_up,w_out}
  dec.l.{ln1,wq,wk,wv,wo,lnc,cwq,cwk,cwv,cwo,ln2,w_in,w_up,w_out}
`w_in` is the gate projection of a gated FFN and `w_up` its linear branch
(absent for the plain ReLU FFN); `lnc`/`cw*` exist only with cross-attention.
"""
from __future__ import annotations

import numpy as np

from .configs import DT_BF16, POS_RELATIVE, ModelShape, PairConfig


def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bf16-representable value (ties to
    even) and return it as fp32.  Storage formatting of inputs only."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32)


def tensor_names(m: ModelShape) -> list[str]:
    names = ["emb"]
    if not m.tied:
        names.append("head")
    if m.n_enc:
        names.append("enc_final_norm")
    names.append("dec_final_norm")
    if m.pos == POS_RELATIVE:
        if m.n_enc:
            names.append("enc_rel_bias")
        names.append("dec_rel_bias")
    for l in range(m.n_enc):
        names += [f"enc.{l}.{k}" for k in ("ln1", "wq", "wk", "wv", "wo", "ln2", "w_in")]
        if m.gated:
            names.append(f"enc.{l}.w_up")
        names.append(f"enc.{l}.w_out")
    for l in range(m.n_dec):
        names += [f"dec.{l}.{k}" for k in ("ln1", "wq", "wk", "wv", "wo")]
        if m.cross:
            names += [f"dec.{l}.{k}" for k in ("lnc", "cwq", "cwk", "cwv", "cwo")]
        names += [f"dec.{l}.{k}" for k in ("ln2", "w_in")]
        if m.gated:
            names.append(f"dec.{l}.w_up")
        names.append(f"dec.{l}.w_out")
    return names


def tensor_shape(m: ModelShape, name: str) -> tuple:
    leaf = name.split(".")[-1]
    d, i, f, v = m.d, m.inner, m.d_ff, m.vocab
    if leaf in ("emb", "head"):
        return (v, d)
    if leaf in ("enc_rel_bias", "dec_rel_bias"):
        return (m.heads, 2 * m.rel_max_dist + 1)
    if leaf in ("enc_final_norm", "dec_final_norm", "ln1", "ln2", "lnc"):
        return (d,)
    if leaf in ("wq", "wk", "wv", "cwq", "cwk", "cwv"):
        return (d, i)
    if leaf in ("wo", "cwo"):
        return (i, d)
    if leaf in ("w_in", "w_up"):
        return (d, f)
    if leaf == "w_out":
        return (f, d)
    raise KeyError(name)


def _is_gain(name: str) -> bool:
    return name.split(".")[-1] in ("enc_final_norm", "dec_final_norm", "ln1", "ln2", "lnc")


def _stable_id(name: str) -> int:
    """A name-derived integer that does not depend on the model's other
    tensors, so a tensor's values are a function of (seed, name, shape)."""
    h = 1469598103934665603
    for c in name.encode():
        h = ((h ^ c) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return h & 0x7FFFFFFF


def distance_ties(max_dist: int, buckets: int, two_sided: bool) -> np.ndarray:
    """Which entries of a synthetic relative-position table share a value: for every signed distance
    r in [-max_dist, max_dist] the index of the drawn value it takes.  The tie pattern is the T5 family's
    log-spaced one: with `half` = buckets (one-sided tables) or buckets/2 (two-sided: the second half serves
    r > 0), distances |r| < half/2 have a value of their own and larger ones share a value over ranges whose
    ends grow geometrically up to max_dist.  Integer arithmetic only, so the pattern is exact."""
    half = buckets // 2 if two_sided else buckets
    exact = max(1, half // 2)
    steps = half - exact
    out = np.zeros(2 * max_dist + 1, dtype=np.int64)
    for r in range(-max_dist, max_dist + 1):
        n = abs(r) if two_sided else max(-r, 0)
        if n < exact:
            b = n
        else:
            # largest j with (n/exact)^steps >= (max_dist/exact)^j
            j = 0
            while j < steps and n ** steps * exact ** (j + 1) >= exact ** steps * max_dist ** (j + 1):
                j += 1
            b = min(half - 1, exact + j)
        out[r + max_dist] = b + (half if two_sided and r > 0 else 0)
    return out


def make_weights(m: ModelShape, seed: int, std: float = 0.02, gain_jitter: float = 0.0) -> dict:
    """N(0, std) matrices (bf16-representable when the model stores bf16) and
    norm gains 1 + gain_jitter*N(0,1), each from its own Philox stream."""
    out = {}
    for name in tensor_names(m):
        rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, _stable_id(name)])))
        shape = tensor_shape(m, name)
        if name in ("enc_rel_bias", "dec_rel_bias"):
            # N(0, 1) values: score biases of the size of the scores themselves (not rounded: the table stays fp32)
            drawn = rng.standard_normal((m.heads, m.rel_buckets), dtype=np.float32)
            out[name] = np.ascontiguousarray(drawn[:, distance_ties(m.rel_max_dist, m.rel_buckets, name == "enc_rel_bias")])
        elif _is_gain(name):
            g = np.ones(shape, dtype=np.float32)
            if gain_jitter:
                g += (gain_jitter * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
            out[name] = g
        else:
            w = rng.standard_normal(shape, dtype=np.float32)
            w *= np.float32(std)
            out[name] = to_bf16_values(w) if m.dtype == DT_BF16 else w
    return out


def truncate_weights(large: ModelShape, wl: dict, small: ModelShape) -> dict:
    """The small model as the leading sub-blocks of the large one: first
    layers, first `d` rows/columns, first heads, first FFN units.  Views are
    copied so the two models own separate buffers."""
    assert small.d <= large.d and small.inner <= large.inner and small.d_ff <= large.d_ff
    assert small.n_dec <= large.n_dec and small.n_enc <= large.n_enc
    assert small.vocab == large.vocab and small.d_head == large.d_head
    assert small.pos == large.pos and small.rel_max_dist == large.rel_max_dist and small.heads <= large.heads
    d, i, f = small.d, small.inner, small.d_ff
    out = {}
    for name in tensor_names(small):
        src = wl[name]
        leaf = name.split(".")[-1]
        if leaf in ("emb", "head"):
            t = src[:, :d]
        elif leaf in ("enc_rel_bias", "dec_rel_bias"):
            t = src[:small.heads]
        elif _is_gain(name):
            t = src[:d]
        elif leaf in ("wq", "wk", "wv", "cwq", "cwk", "cwv"):
            t = src[:d, :i]
        elif leaf in ("wo", "cwo"):
            t = src[:i, :d]
        elif leaf in ("w_in", "w_up"):
            t = src[:d, :f]
        elif leaf == "w_out":
            t = src[:f, :d]
        else:
            raise KeyError(name)
        out[name] = np.ascontiguousarray(t)
    return out


def make_pair_weights(cfg: PairConfig) -> tuple[dict, dict]:
    """(small, large) weight dictionaries of a pair."""
    wl = make_weights(cfg.large, cfg.weight_seed, cfg.weight_std, cfg.gain_jitter)
    ws = truncate_weights(cfg.large, wl, cfg.small)
    return ws, wl


def make_source(cfg: PairConfig, n: int | None = None, seed: int | None = None) -> np.ndarray:
    """Source (or prompt) token ids: uniform on [0, V), or Zipf with exponent
    1.1 over ranks 1..V by inverse CDF, rank k mapped to id k-1."""
    n = cfg.n_src if n is None else n
    seed = cfg.input_seed if seed is None else seed
    v = cfg.large.vocab
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 1])))
    if cfg.src_dist == "uniform":
        return rng.integers(0, v, size=n, dtype=np.int64).astype(np.int32)
    cdf = np.cumsum(np.arange(1, v + 1, dtype=np.float64) ** -1.1)
    cdf /= cdf[-1]
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="left"), v - 1).astype(np.int32)


def make_tokens(vocab: int, n: int, seed: int) -> np.ndarray:
    """Uniform token ids for forced draft blocks in stress tests."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 2])))
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def make_uniforms(n: int, seed: int, stream: int) -> np.ndarray:
    """n uniform numbers in [0, 1) for the sampling variant, one per sequence position; `stream`
    separates the small model's draws (0) from the large model's (1).  Each is k / 2^24 for an
    integer k, so float32 and float64 hold exactly the same value."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 3, stream])))
    return (rng.integers(0, 1 << 24, size=n, dtype=np.int64).astype(np.float64) / float(1 << 24)).astype(np.float32)
