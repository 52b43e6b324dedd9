"""Shapes of the synthetic model pairs and the run parameters of each workload.

Pure data: layer counts, widths, vocabulary sizes, thresholds and seeds.  The
Transformer arithmetic itself lives elsewhere (once in the CPU oracle, once in
the HIP library); both read these records.

The four encoder-decoder shapes follow the paper's Table 2 (layers, model
dimension, FFN dimension); head counts, activation, vocabulary and positional
scheme are choices of this synthetic benchmark, not of the paper.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional

ACT_RELU, ACT_GATED_GELU, ACT_SWIGLU = 0, 1, 2
POS_SINUSOIDAL, POS_ROPE, POS_RELATIVE = 0, 1, 2
DT_F32, DT_BF16 = 0, 1


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_enc: int          # encoder layers (0: no encoder of its own)
    n_dec: int          # decoder layers
    d: int              # model dimension
    heads: int
    d_head: int
    d_ff: int
    act: int            # ACT_*
    pos: int            # POS_*
    vocab: int
    tied: bool          # LM head shares the embedding matrix
    dtype: int          # DT_*: storage type of weights and of cached K/V
    cross: bool         # decoder layers have a cross-attention sublayer
    logit_scale: float = 1.0
    embed_scale: float = 1.0
    eps: float = 1e-6
    rope_base: float = 10000.0
    bos: int = 0
    tie_shift: int = 0  # input embedding of token t is row (t + tie_shift) mod vocab of the embedding matrix
    rel_max_dist: int = 0   # POS_RELATIVE: key-query distances are clamped to [-rel_max_dist, rel_max_dist]
    rel_buckets: int = 0    # POS_RELATIVE: distinct values per head in a synthetic bias table (log-spaced ties)

    @property
    def inner(self) -> int:
        return self.heads * self.d_head

    @property
    def gated(self) -> bool:
        return self.act != ACT_RELU

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == DT_F32 else 2

    # ---- shape accounting (pure counting) -------------------------------
    def decoder_params(self) -> int:
        """Decoder weight-matrix parameters without embeddings and norm gains
        (the quantity Table 2 lists)."""
        attn = 4 * self.d * self.inner
        per_layer = attn * (2 if self.cross else 1) + (3 if self.gated else 2) * self.d * self.d_ff
        return self.n_dec * per_layer

    def encoder_params(self) -> int:
        per_layer = 4 * self.d * self.inner + (3 if self.gated else 2) * self.d * self.d_ff
        return self.n_enc * per_layer

    def pass_bytes(self, t_cache: int, n_src: int, rows: int = 1) -> int:
        """Bytes one decoder pass must read: every decoder weight, the LM head,
        the self-attention cache up to t_cache+rows positions and the
        cross-attention K/V of n_src positions (Appendix 'Model Analysis':
        memory operations per pass do not grow with the number of rows)."""
        b = self.elem_bytes
        w = self.decoder_params() + self.vocab * self.d
        kv_self = self.n_dec * 2 * self.inner * (t_cache + rows)
        kv_cross = self.n_dec * 2 * self.inner * n_src if self.cross else 0
        return b * (w + kv_self + kv_cross)

    def pass_flops(self, t_cache: int, n_src: int, rows: int = 1) -> int:
        """Multiply-add flops of one pass over `rows` rows: 2 per weight per
        row plus the attention products (Section 3.2: a pass over n rows costs
        the flops of n single-row passes)."""
        w = self.decoder_params() + self.vocab * self.d
        total = 0
        for r in range(rows):
            keys = t_cache + r + 1
            att = 4 * self.n_dec * self.inner * (keys + (n_src if self.cross else 0))
            total += 2 * w + att
        return total


@dataclass(frozen=True)
class PairConfig:
    name: str
    small: ModelShape
    large: ModelShape
    n_src: int
    max_new: int
    alpha_fb: float
    alpha_rb: float
    n_max: int = 10            # cap on consecutive small-model tokens (Appendix, evaluation details)
    src_dist: str = "zipf"     # "uniform" or "zipf" (exponent 1.1)
    weight_seed: int = 20230207
    input_seed: int = 7863
    weight_std: float = 0.02
    gain_jitter: float = 0.0   # norm gains are 1 + jitter*N(0,1); 0 in the benchmark configs
    decoder_only: bool = False
    early_exit: bool = False   # the small model is a prefix of the large one (same widths, first n_dec layers, shared head)
    alpha_fb_sweep: tuple = ()
    alpha_rb_sweep: tuple = ()


def _t5(name, n_layers, d, heads, d_ff, act, vocab, tied, dtype, logit_scale, embed_scale, relative=False):
    return ModelShape(name=name, n_enc=n_layers, n_dec=n_layers, d=d, heads=heads, d_head=64,
                      d_ff=d_ff, act=act, pos=POS_RELATIVE if relative else POS_SINUSOIDAL, vocab=vocab, tied=tied,
                      dtype=dtype, cross=True, logit_scale=logit_scale, embed_scale=embed_scale,
                      tie_shift=7919 if tied else 0, rel_max_dist=128 if relative else 0,
                      rel_buckets=32 if relative else 0)


def tiny_pair() -> PairConfig:
    """Config 1: fp32 correctness pair; the small model is the large one's
    first two decoder layers with the shared embedding, final norm and head
    (the early-exit arrangement of Section 4.4)."""
    ls_s, ls_l, es = CAL["tiny"]
    large = ModelShape("tiny-large", n_enc=4, n_dec=4, d=256, heads=4, d_head=64, d_ff=1024,
                       act=ACT_RELU, pos=POS_SINUSOIDAL, vocab=1024, tied=True, dtype=DT_F32,
                       cross=True, logit_scale=ls_l, embed_scale=es, tie_shift=331)
    small = replace(large, name="tiny-small", n_enc=0, n_dec=2, logit_scale=ls_s)
    return PairConfig("tiny", small, large, n_src=32, max_new=32, alpha_fb=0.5, alpha_rb=2.0,
                      src_dist="uniform", early_exit=True)


def t5_pair() -> PairConfig:
    """Config 2: T5-small / T5-large shapes (Table 2), bf16, summarisation-like lengths."""
    ls_s, ls_l, es = CAL["t5"]
    small = _t5("t5-small", 6, 512, 8, 2048, ACT_RELU, 32128, True, DT_BF16, ls_s, es)
    large = _t5("t5-large", 24, 1024, 16, 4096, ACT_RELU, 32128, True, DT_BF16, ls_l, es)
    return PairConfig("t5", small, large, n_src=512, max_new=64, alpha_fb=0.5, alpha_rb=2.0,
                      alpha_fb_sweep=(0.3, 0.5, 0.7), alpha_rb_sweep=(1.0, 2.0, 4.0))


def t5_relative_pair() -> PairConfig:
    """Config 2's shapes with the position scheme of the T5 family: no position added to the embedding, a
    learned bias on the self-attention scores indexed by the clamped key-query distance (128), 32 log-spaced
    distinct values per head.  Thresholds are config 2's; the small model's logit scale is calibrated separately."""
    ls_s, ls_l, es = CAL["t5rel"]
    small = _t5("t5-small-rel", 6, 512, 8, 2048, ACT_RELU, 32128, True, DT_BF16, ls_s, es, relative=True)
    large = _t5("t5-large-rel", 24, 1024, 16, 4096, ACT_RELU, 32128, True, DT_BF16, ls_l, es, relative=True)
    return PairConfig("t5rel", small, large, n_src=512, max_new=64, alpha_fb=0.5, alpha_rb=2.0)


def t5_early_exit_pair() -> PairConfig:
    """Early-exit arrangement (Section 4.4) at config 2's large shape: the small model is the first six
    decoder layers of the T5-large-shaped model with its final norm and head."""
    ls_s, ls_l, es = CAL["t5ee"]
    large = _t5("t5-large", 24, 1024, 16, 4096, ACT_RELU, 32128, True, DT_BF16, ls_l, es)
    small = replace(large, name="t5-large-first6", n_enc=0, n_dec=6, logit_scale=ls_s)
    return PairConfig("t5ee", small, large, n_src=512, max_new=64, alpha_fb=0.5, alpha_rb=2.0, early_exit=True)


def mt5_pair() -> PairConfig:
    """Config 3: mT5-small / mT5-large shapes (Table 2), 250k vocabulary, translation-like lengths."""
    ls_s, ls_l, es = CAL["mt5"]
    small = _t5("mt5-small", 8, 512, 6, 1024, ACT_GATED_GELU, 250112, True, DT_BF16, ls_s, es)
    large = _t5("mt5-large", 24, 1024, 16, 2816, ACT_GATED_GELU, 250112, True, DT_BF16, ls_l, es)
    return PairConfig("mt5", small, large, n_src=64, max_new=64, alpha_fb=0.5, alpha_rb=2.0)


def _llama(name, n_layers, d, heads, d_ff, logit_scale, embed_scale):
    return ModelShape(name=name, n_enc=0, n_dec=n_layers, d=d, heads=heads, d_head=128, d_ff=d_ff,
                      act=ACT_SWIGLU, pos=POS_ROPE, vocab=32000, tied=True, dtype=DT_BF16,
                      cross=False, logit_scale=logit_scale, embed_scale=embed_scale, tie_shift=7919)


def llama_pair() -> PairConfig:
    """Config 4: decoder-only pair, RoPE + SwiGLU, long prompt."""
    ls_s, ls_l, es = CAL["llama"]
    small = _llama("llama-small", 16, 2048, 16, 5632, ls_s, es)
    large = _llama("llama-large", 32, 4096, 32, 11008, ls_l, es)
    return PairConfig("llama", small, large, n_src=1024, max_new=256, alpha_fb=0.5, alpha_rb=2.0,
                      decoder_only=True)


def toy_pair(dtype=DT_F32, act=ACT_RELU, pos=POS_SINUSOIDAL, cross=True, tied=True,
             d=64, heads=2, d_head=16, d_ff=96, vocab=200, n_small=1, n_large=3,
             truncate=False, logit_scale=16.0, embed_scale=14.0, gain_jitter=0.1,
             n_src=9, max_new=24, tie_shift=37, rel_max_dist=5, rel_buckets=6) -> PairConfig:
    """Unit-test pair, small enough for the no-cache oracle and for brute
    force.  Norm gains are jittered so that a dropped gain shows up, widths are
    deliberately not powers of two and `heads*d_head != d`."""
    n_enc = 2 if cross else 0
    mul = 2 if truncate else 1          # a truncated pair: the large model is twice as wide as the small one
    large = ModelShape("toy-large", n_enc=n_enc, n_dec=n_large, d=d * mul, heads=heads * mul, d_head=d_head,
                       d_ff=d_ff * mul, act=act, pos=pos, vocab=vocab, tied=tied, dtype=dtype, cross=cross,
                       logit_scale=logit_scale, embed_scale=embed_scale, tie_shift=tie_shift if tied else 0,
                       rel_max_dist=rel_max_dist if pos == POS_RELATIVE else 0,
                       rel_buckets=rel_buckets if pos == POS_RELATIVE else 0)
    if truncate:
        small = replace(large, name="toy-small", n_enc=min(1, n_enc), n_dec=n_small, d=d, heads=heads, d_ff=d_ff)
    else:
        small = replace(large, name="toy-small", n_enc=0, n_dec=n_small)
    return PairConfig("toy", small, large, n_src=n_src, max_new=max_new, alpha_fb=0.5, alpha_rb=2.0,
                      src_dist="uniform", gain_jitter=gain_jitter, decoder_only=not cross)


# (logit_scale of the small model, logit_scale of the large model, embed_scale) per pair.
# N(0, 0.02) weights give almost flat softmaxes, for which every step would fall back, and a
# truncated small model is systematically MORE peaked than its deeper parent, which makes every
# review a rollback.  These constants were chosen by sweeping them (CPU oracle for `tiny`, the
# GPU path checked against the oracle for the others) until, at the middle thresholds
# (alpha_FB 0.5, alpha_RB 2), the share of tokens that fall back and the share of reviews that
# roll back land in the range the paper's Table 4 reports (about 20-35 % and 1.5-6.5 %).
CAL = {
    "tiny": (8.0, 8.0, 12.0),
    "t5": (2.0, 4.0, 36.0),
    "mt5": (2.0, 4.0, 36.0),
    "llama": (0.9, 4.0, 50.0),
    "t5ee": (1.65, 4.0, 36.0),
    "t5rel": (1.63, 4.0, 36.0),
}

PAIRS = {"tiny": tiny_pair, "t5": t5_pair, "mt5": mt5_pair, "llama": llama_pair, "t5ee": t5_early_exit_pair,
         "t5rel": t5_relative_pair}
