"""CPU oracle: the Transformer distributions p_S(y | x, y_1..k) and p_L(...) that
the paper's problem formulation (Section 3.2, Eq. 1) takes as given.

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, no blocking, no fusion.  The
product (the HIP library) never imports this package and shares no code with it.

Two routes to the same numbers are kept on purpose:
  * `Model.logits_full`  - the definition: run the whole prefix through every
    layer with a causal mask, no cache (textbook pre-norm Transformer decoder);
  * `DecoderCache.step`  - the KV-cached form processing T new rows at once.
    Section 3.2 states that one pass over n rows yields the same distributions
    as n single-row steps; tests/test_oracle_*.py hold the two to 1e-12.

Model contract (the paper fixes none of this; it is the benchmark's choice):
  embed    x = embed_scale * E[row] + PE(position)              (sinusoidal models)
           x = embed_scale * E[row]                              (RoPE models)
           row = (token + tie_shift) mod vocab; tie_shift = 0 is the ordinary
           lookup.  With a tied head and random weights E E^T is diagonally
           dominant and every model would repeat its input token for ever; a
           non-zero shift turns that fixed point into a walk over the vocabulary.
           PE(p)[2i] = sin(p / 10000^(2i/d)), PE(p)[2i+1] = cos(same)
  norm     RMSNorm: x / sqrt(mean(x^2) + eps) * gain
  attn     per head softmax(q k^T / sqrt(d_head)) v ; decoder self-attention is
           causal, encoder self-attention and cross-attention are not
  RoPE     on q and k, pairs (2i, 2i+1) rotated by position * base^(-2i/d_head)
  relative no position enters the embedding; every self-attention score (encoder and
           decoder, all layers of a stack sharing one table) gets
           bias[head][clip(key position - query position, -D, D) + D] added before the
           softmax, D = rel_max_dist.  Cross-attention has no bias.  (The position
           scheme of the T5 family; its log-spaced buckets are a tie pattern inside
           the table and need no arithmetic here.)
  ffn      relu(x W_in) W_out, or (act(x W_in) * (x W_up)) W_out with
           act = tanh-approximated GELU, or SiLU
  sublayer x <- x + f(norm(x)); decoder order self-attn, cross-attn, ffn
  head     logits = logit_scale * norm_final(x) @ E_out^T  (E_out = E when tied)
  storage  in bf16 models every K and V vector (decoder self, cross, encoder
           self) is rounded to bf16 (nearest even) before it is used; weights
           arrive already bf16-representable; everything else is real arithmetic.
"""
from __future__ import annotations

import numpy as np

ACT_RELU, ACT_GATED_GELU, ACT_SWIGLU = 0, 1, 2
POS_SINUSOIDAL, POS_ROPE, POS_RELATIVE = 0, 1, 2
DT_F32, DT_BF16 = 0, 1


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (8 significant bits), ties to even, from float64."""
    m, e = np.frexp(np.asarray(a, dtype=np.float64))     # a = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def sinusoid(positions: np.ndarray, d: int) -> np.ndarray:
    i = np.arange(d // 2, dtype=np.float64)
    ang = positions[:, None].astype(np.float64) / (10000.0 ** (2.0 * i / d))[None, :]
    pe = np.empty((len(positions), d), dtype=np.float64)
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe


def rope(x: np.ndarray, positions: np.ndarray, heads: int, d_head: int, base: float) -> np.ndarray:
    """x: [T, heads*d_head]; rotate each (2i, 2i+1) pair of every head."""
    t = x.shape[0]
    xh = x.reshape(t, heads, d_head // 2, 2)
    i = np.arange(d_head // 2, dtype=np.float64)
    ang = positions[:, None].astype(np.float64) * (base ** (-2.0 * i / d_head))[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    out = np.empty_like(xh)
    out[..., 0] = xh[..., 0] * c - xh[..., 1] * s
    out[..., 1] = xh[..., 0] * s + xh[..., 1] * c
    return out.reshape(t, heads * d_head)


def gelu_tanh(u: np.ndarray) -> np.ndarray:
    return 0.5 * u * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (u + 0.044715 * u ** 3)))


def silu(u: np.ndarray) -> np.ndarray:
    return u / (1.0 + np.exp(-u))


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, heads: int, d_head: int,
              q_pos: np.ndarray | None, rel_bias: np.ndarray | None = None,
              row_pos: np.ndarray | None = None) -> np.ndarray:
    """q: [T, I], k, v: [P, I]; key p sits at position p.  Row r may see key p iff
    q_pos is None (not causal) or p <= q_pos[r].  rel_bias [heads, 2D+1], if given,
    adds rel_bias[h, clip(p - row_pos[r], -D, D) + D] to the score of (r, p).  Returns [T, I]."""
    t, p = q.shape[0], k.shape[0]
    out = np.empty((t, heads * d_head), dtype=np.float64)
    if rel_bias is not None:
        dmax = (rel_bias.shape[1] - 1) // 2
        rel_idx = np.clip(np.arange(p)[None, :] - np.asarray(row_pos)[:, None], -dmax, dmax) + dmax
    for h in range(heads):
        sl = slice(h * d_head, (h + 1) * d_head)
        s = q[:, sl] @ k[:, sl].T / np.sqrt(float(d_head))
        if rel_bias is not None:
            s = s + np.asarray(rel_bias[h], dtype=np.float64)[rel_idx]
        if q_pos is not None:
            s = np.where(np.arange(p)[None, :] <= q_pos[:, None], s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w /= w.sum(axis=1, keepdims=True)
        out[:, sl] = w @ v[:, sl]
    return out


class Model:
    """One network's weights (float64 copies of the shared fp32 buffers)."""

    def __init__(self, shape, weights: dict, compact: bool = False):
        """compact=True keeps the fp32 buffers and widens each matrix to
        float64 at the point of use (same values, less memory; for the
        7B-shaped model whose float64 copy would not fit the host)."""
        self.s = shape
        self.w = dict(weights) if compact else {k: np.asarray(a, dtype=np.float64) for k, a in weights.items()}
        self.head = self.w["emb"] if shape.tied else self.w["head"]

    # -- pieces -------------------------------------------------------------
    def _store(self, a: np.ndarray) -> np.ndarray:
        return round_bf16(a) if self.s.dtype == DT_BF16 else a

    def embed(self, tokens, positions: np.ndarray) -> np.ndarray:
        rows = (np.asarray(tokens, dtype=np.int64) + self.s.tie_shift) % self.s.vocab
        x = self.s.embed_scale * np.asarray(self.w["emb"][rows], dtype=np.float64)
        if self.s.pos == POS_SINUSOIDAL:
            x = x + sinusoid(positions, self.s.d)
        return x

    def _qk_pos(self, a: np.ndarray, positions: np.ndarray) -> np.ndarray:
        if self.s.pos == POS_ROPE:
            return rope(a, positions, self.s.heads, self.s.d_head, self.s.rope_base)
        return a

    def _rel(self, name: str):
        return self.w[name] if self.s.pos == POS_RELATIVE else None

    def ffn(self, pre: str, xn: np.ndarray) -> np.ndarray:
        u = xn @ self.w[pre + "w_in"]
        if self.s.act == ACT_RELU:
            h = np.maximum(u, 0.0)
        elif self.s.act == ACT_GATED_GELU:
            h = gelu_tanh(u) * (xn @ self.w[pre + "w_up"])
        else:
            h = silu(u) * (xn @ self.w[pre + "w_up"])
        return h @ self.w[pre + "w_out"]

    def logits_from_hidden(self, x: np.ndarray) -> np.ndarray:
        xn = rmsnorm(x, self.w["dec_final_norm"], self.s.eps)
        return self.s.logit_scale * (xn @ self.head.T)

    # -- encoder --------------------------------------------------------------
    def encode(self, src) -> np.ndarray:
        """Encoder output [S, d] (after the encoder's final norm)."""
        s = self.s
        pos = np.arange(len(src))
        x = self.embed(src, pos)
        for l in range(s.n_enc):
            p = f"enc.{l}."
            xn = rmsnorm(x, self.w[p + "ln1"], s.eps)
            q = self._qk_pos(xn @ self.w[p + "wq"], pos)
            k = self._store(self._qk_pos(xn @ self.w[p + "wk"], pos))
            v = self._store(xn @ self.w[p + "wv"])
            x = x + attention(q, k, v, s.heads, s.d_head, None, self._rel("enc_rel_bias"), pos) @ self.w[p + "wo"]
            x = x + self.ffn(p, rmsnorm(x, self.w[p + "ln2"], s.eps))
        return rmsnorm(x, self.w["enc_final_norm"], s.eps)

    def cross_kv(self, enc_out: np.ndarray) -> list:
        """Per decoder layer (K, V) of the source positions; [] without cross-attention."""
        if not self.s.cross:
            return []
        return [(self._store(enc_out @ self.w[f"dec.{l}.cwk"]), self._store(enc_out @ self.w[f"dec.{l}.cwv"]))
                for l in range(self.s.n_dec)]

    # -- decoder, definition form (no cache) -----------------------------------
    def logits_full(self, y, cross: list) -> np.ndarray:
        """Logits of every position of the prefix y: row m is the distribution
        of the token after y[0..m] (Section 3.2: p(y | y_1..m))."""
        s = self.s
        pos = np.arange(len(y))
        x = self.embed(y, pos)
        for l in range(s.n_dec):
            p = f"dec.{l}."
            xn = rmsnorm(x, self.w[p + "ln1"], s.eps)
            q = self._qk_pos(xn @ self.w[p + "wq"], pos)
            k = self._store(self._qk_pos(xn @ self.w[p + "wk"], pos))
            v = self._store(xn @ self.w[p + "wv"])
            x = x + attention(q, k, v, s.heads, s.d_head, pos, self._rel("dec_rel_bias"), pos) @ self.w[p + "wo"]
            if s.cross:
                xn = rmsnorm(x, self.w[p + "lnc"], s.eps)
                ck, cv = cross[l]
                x = x + attention(xn @ self.w[p + "cwq"], ck, cv, s.heads, s.d_head, None) @ self.w[p + "cwo"]
            x = x + self.ffn(p, rmsnorm(x, self.w[p + "ln2"], s.eps))
        return self.logits_from_hidden(x)


class DecoderCache:
    """KV-cached decoder of one model for one request.  `length` rows are
    valid; truncation only lowers `length` (stale rows are overwritten later)."""

    def __init__(self, model: Model, cross: list, capacity: int, store=None):
        """store(layer, "k" | "v", exact [T, I], first_row) -> the values to cache, in place of the model's own
        rounding to its storage type: for tests that take the storage-rounding decisions from elsewhere (the
        arithmetic around them is unchanged)."""
        self.m, self.cross = model, cross
        self.store = store
        i = model.s.inner
        self.k = [np.zeros((capacity, i)) for _ in range(model.s.n_dec)]
        self.v = [np.zeros((capacity, i)) for _ in range(model.s.n_dec)]
        self.length = 0

    def truncate(self, length: int) -> None:
        assert 0 <= length <= self.length
        self.length = length

    def step(self, tokens, last: int | None = None) -> np.ndarray:
        """Consume T tokens at positions length..length+T-1; return their T
        rows of logits and advance the cache by T.  `last` (0..T) limits the
        returned logits to the last `last` rows (the head is then evaluated on
        those rows only; the cache advances all the same)."""
        m, s = self.m, self.m.s
        t0, t = self.length, len(tokens)
        pos = np.arange(t0, t0 + t)
        x = m.embed(tokens, pos)
        for l in range(s.n_dec):
            p = f"dec.{l}."
            xn = rmsnorm(x, m.w[p + "ln1"], s.eps)
            q = m._qk_pos(xn @ m.w[p + "wq"], pos)
            k_new, v_new = m._qk_pos(xn @ m.w[p + "wk"], pos), xn @ m.w[p + "wv"]
            self.k[l][t0:t0 + t] = m._store(k_new) if self.store is None else self.store(l, "k", k_new, t0)
            self.v[l][t0:t0 + t] = m._store(v_new) if self.store is None else self.store(l, "v", v_new, t0)
            a = attention(q, self.k[l][:t0 + t], self.v[l][:t0 + t], s.heads, s.d_head, pos, m._rel("dec_rel_bias"), pos)
            x = x + a @ m.w[p + "wo"]
            if s.cross:
                xn = rmsnorm(x, m.w[p + "lnc"], s.eps)
                ck, cv = self.cross[l]
                x = x + attention(xn @ m.w[p + "cwq"], ck, cv, s.heads, s.d_head, None) @ m.w[p + "cwo"]
            x = x + m.ffn(p, rmsnorm(x, m.w[p + "ln2"], s.eps))
        self.length = t0 + t
        if last is not None:
            assert 0 <= last <= t
            x = x[t - last:]
        return m.logits_from_hidden(x)
