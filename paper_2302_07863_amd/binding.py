"""Thin ctypes binding of libbild.so: argument marshalling only.  Every step of
the decoding path runs in the library's HIP kernels; there is no Python or CPU
fallback, and a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libbild.so")

OK, EINVAL, ESTATE, ECAP, EHIP, ENOMEM = 0, -1, -2, -3, -4, -5
MAX_ROWS = 32
SMALL, LARGE, BOTH = 1, 2, 3
ACCEPT_THRESHOLD, ACCEPT_REJECTION = 0, 1


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_enc_layers", "n_dec_layers", "d_model", "n_heads", "d_head", "d_ff", "act", "pos", "vocab",
        "tied_head", "dtype", "cross_attn", "bos", "tie_shift")] + [
        (n, C.c_float) for n in ("logit_scale", "embed_scale", "norm_eps", "rope_base")] + [
        ("rel_max_dist", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "small_steps", "large_calls", "rows_verified", "fallbacks_conf", "fallbacks_forced", "rollbacks",
        "tokens_discarded", "n_generated")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Profile(C.Structure):
    _fields_ = [("launches", (C.c_int64 * 2) * 2), ("bytes", (C.c_int64 * 2) * 2), ("ms", (C.c_double * 2) * 2),
                ("dropped", C.c_int32)]


class BildError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {code} ({strerror(code)})")
        self.code = code


_lib = None

_SIGS = {
    "bild_model_num_tensors": (C.c_int, [C.POINTER(ModelConfig)]),
    "bild_model_create": (C.c_int, [C.POINTER(ModelConfig), C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_void_p)]),
    "bild_model_destroy": (C.c_int, [C.c_void_p]),
    "bild_pair_create": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "bild_pair_create_early_exit": (C.c_int, [C.c_void_p, C.c_int, C.c_float, C.POINTER(C.c_void_p)]),
    "bild_pair_destroy": (C.c_int, [C.c_void_p]),
    "bild_state_create": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.POINTER(C.c_void_p)]),
    "bild_state_destroy": (C.c_int, [C.c_void_p]),
    "bild_encode": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int]),
    "bild_small_step": (C.c_int, [C.c_void_p, C.c_float, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                  C.POINTER(C.c_float)]),
    "bild_large_verify": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_void_p, C.POINTER(C.c_int32),
                                    C.POINTER(C.c_int32), C.c_void_p]),
    "bild_set_sampling": (C.c_int, [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_int]),
    "bild_set_acceptance": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int]),
    "bild_kv_truncate": (C.c_int, [C.c_void_p, C.c_int, C.c_int]),
    "bild_seq_truncate": (C.c_int, [C.c_void_p, C.c_int]),
    "bild_force_tokens": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int]),
    "bild_generate": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_float, C.c_int, C.c_int32,
                                C.c_void_p, C.POINTER(C.c_int32), C.POINTER(Stats)]),
    "bild_greedy": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int32, C.c_void_p,
                              C.POINTER(C.c_int32)]),
    "bild_head_stats": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "bild_head_stats_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "bild_get_lengths": (C.c_int, [C.c_void_p] + [C.POINTER(C.c_int32)] * 4),
    "bild_get_sequence": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int32)]),
    "bild_debug_enable_logits": (C.c_int, [C.c_void_p, C.c_int]),
    "bild_debug_logits": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "bild_debug_kv": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "bild_bench_pass": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float)]),
    "bild_bench_gemm": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_int64),
                                  C.POINTER(C.c_int64)]),
    "bild_gemm_tally": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_int]),
    "bild_pass_stages": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32)]),
    "bild_probe_stream": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float)]),
    "bild_probe_launch": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_float)]),
    "bild_debug_tiled_bytes": (C.c_int64, [C.c_int, C.c_int, C.c_int]),
    "bild_debug_tile_matrix": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "bild_debug_attn_shape": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)]),
    "bild_debug_gemm_shape": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)]),
    "bild_probe_copy": (C.c_int, [C.c_void_p, C.c_int64, C.c_int]),
    "bild_profile_begin": (C.c_int, [C.c_void_p, C.c_int]),
    "bild_profile_end": (C.c_int, [C.c_void_p, C.POINTER(Profile)]),
    "bild_pass_bytes": (C.c_int64, [C.c_void_p, C.c_int, C.c_int, C.c_int]),
    "bild_strerror": (C.c_char_p, [C.c_int]),
}


def exported_symbols() -> list:
    return sorted(_SIGS)


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().bild_strerror(code).decode()


def _check(code: int, what: str):
    if code != OK:
        raise BildError(code, what)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def config_from_shape(shape) -> ModelConfig:
    """ModelConfig from a bild_inputs.ModelShape-like record (plain field copy)."""
    return ModelConfig(n_enc_layers=shape.n_enc, n_dec_layers=shape.n_dec, d_model=shape.d, n_heads=shape.heads,
                       d_head=shape.d_head, d_ff=shape.d_ff, act=shape.act, pos=shape.pos, vocab=shape.vocab,
                       tied_head=int(shape.tied), dtype=shape.dtype, cross_attn=int(shape.cross), bos=shape.bos,
                       tie_shift=shape.tie_shift, logit_scale=shape.logit_scale, embed_scale=shape.embed_scale,
                       norm_eps=shape.eps, rope_base=shape.rope_base,
                       rel_max_dist=getattr(shape, "rel_max_dist", 0))


class Model:
    h = None

    def __init__(self, cfg: ModelConfig, tensors: Sequence[np.ndarray]):
        arrs = [np.ascontiguousarray(t, dtype=np.float32) for t in tensors]
        ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
        h = C.c_void_p()
        _check(lib().bild_model_create(C.byref(cfg), ptrs, len(arrs), C.byref(h)), "bild_model_create")
        self.h, self.cfg = h, cfg

    def close(self):
        if self.h:
            lib().bild_model_destroy(self.h)
            self.h = None

    __del__ = close


ROW_STATS_DTYPE = np.dtype([("zmax", np.float32), ("lse", np.float32), ("argmax", np.int32), ("z_target", np.float32)])


def head_stats(model: Model, x_dev_ptr: int, rows: int, targets_dev_ptr: Optional[int], out_dev_ptr: int,
               stream: Optional[int] = None, entry: str = "bild_head_stats"):
    """Device pointers in, device pointer out (rows records of ROW_STATS_DTYPE); see bild.h."""
    _check(getattr(lib(), entry)(model.h, C.c_void_p(x_dev_ptr), rows, C.c_void_p(targets_dev_ptr or 0),
                                 C.c_void_p(out_dev_ptr), C.c_void_p(stream or 0)), entry)


class Pair:
    h = None

    def __init__(self, small: Model, large: Model):
        h = C.c_void_p()
        _check(lib().bild_pair_create(small.h, large.h, C.byref(h)), "bild_pair_create")
        self.h, self.small, self.large = h, small, large

    @classmethod
    def early_exit(cls, large: Model, k: int, small_logit_scale: float) -> "Pair":
        """The small model is the first k decoder layers of `large` with the shared head."""
        h = C.c_void_p()
        _check(lib().bild_pair_create_early_exit(large.h, k, small_logit_scale, C.byref(h)), "bild_pair_create_early_exit")
        self = cls.__new__(cls)
        self.h, self.small, self.large = h, None, large
        return self

    def close(self):
        if self.h:
            lib().bild_pair_destroy(self.h)
            self.h = None

    __del__ = close


class State:
    h = None

    def __init__(self, pair: Pair, max_src: int, max_len: int, n_max: int = 10, stream: Optional[int] = None):
        h = C.c_void_p()
        _check(lib().bild_state_create(pair.h, max_src, max_len, n_max, C.c_void_p(stream or 0), C.byref(h)),
               "bild_state_create")
        self.h, self.pair, self.max_len = h, pair, max_len

    def close(self):
        if self.h:
            lib().bild_state_destroy(self.h)
            self.h = None

    __del__ = close

    def encode(self, src):
        a = _i32(src)
        _check(lib().bild_encode(self.h, a.ctypes.data, len(a)), "bild_encode")

    def small_step(self, alpha_fb: float):
        tok, flag, pm = C.c_int32(), C.c_int32(), C.c_float()
        _check(lib().bild_small_step(self.h, alpha_fb, C.byref(tok), C.byref(flag), C.byref(pm)), "bild_small_step")
        return tok.value, flag.value, pm.value

    def large_verify(self, alpha_rb: float, draft=None):
        if draft is None:
            n, dptr, cap = 0, None, MAX_ROWS
        else:
            d = _i32(draft)
            n, dptr, cap = len(d), d.ctypes.data, len(d) + 1
        out = np.zeros(max(cap, 1), dtype=np.int32)
        nll = np.zeros(MAX_ROWS, dtype=np.float32)
        n_out, r = C.c_int32(), C.c_int32()
        _check(lib().bild_large_verify(self.h, dptr, n, alpha_rb, out.ctypes.data, C.byref(n_out), C.byref(r),
                                       nll.ctypes.data), "bild_large_verify")
        return out[:n_out.value].tolist(), r.value, nll

    def kv_truncate(self, which: int, pos: int):
        _check(lib().bild_kv_truncate(self.h, which, pos), "bild_kv_truncate")

    def set_sampling(self, top_p: float, u_small=None, u_large=None):
        """top_p <= 0 returns to argmax decoding."""
        if top_p <= 0:
            _check(lib().bild_set_sampling(self.h, float(top_p), None, None, 0), "bild_set_sampling")
            return
        a = np.ascontiguousarray(u_small, dtype=np.float32)
        b = np.ascontiguousarray(u_large, dtype=np.float32)
        _check(lib().bild_set_sampling(self.h, float(top_p), a.ctypes.data, b.ctypes.data, min(len(a), len(b))),
               "bild_set_sampling")

    def seq_truncate(self, n_keep: int):
        _check(lib().bild_seq_truncate(self.h, n_keep), "bild_seq_truncate")

    def set_acceptance(self, rule: int, u_accept=None):
        """rule: ACCEPT_THRESHOLD (the paper's rollback policy) or ACCEPT_REJECTION (needs set_sampling first)."""
        if u_accept is None:
            _check(lib().bild_set_acceptance(self.h, int(rule), None, 0), "bild_set_acceptance")
            return
        a = np.ascontiguousarray(u_accept, dtype=np.float32)
        _check(lib().bild_set_acceptance(self.h, int(rule), a.ctypes.data, len(a)), "bild_set_acceptance")

    def force_tokens(self, first: int, tokens, draft_start: int):
        a = _i32(tokens)
        _check(lib().bild_force_tokens(self.h, first, a.ctypes.data if len(a) else None, len(a), draft_start),
               "bild_force_tokens")

    def generate(self, src, alpha_fb: float, alpha_rb: float, max_new: int, eos: int = -1):
        """src=None continues from the encoded state without re-encoding."""
        a = _i32(src if src is not None else [])
        out = np.zeros(max(max_new, 1), dtype=np.int32)
        n, st = C.c_int32(), Stats()
        _check(lib().bild_generate(self.h, a.ctypes.data if src is not None else None, len(a), alpha_fb, alpha_rb, max_new, eos, out.ctypes.data,
                                   C.byref(n), C.byref(st)), "bild_generate")
        return out[:n.value].tolist(), st.as_dict()

    def greedy(self, which: int, src, max_new: int, eos: int = -1):
        a = _i32(src if src is not None else [])
        out = np.zeros(max(max_new, 1), dtype=np.int32)
        n = C.c_int32()
        _check(lib().bild_greedy(self.h, which, a.ctypes.data if src is not None else None, len(a), max_new, eos, out.ctypes.data, C.byref(n)),
               "bild_greedy")
        return out[:n.value].tolist()

    def lengths(self):
        v = [C.c_int32() for _ in range(4)]
        _check(lib().bild_get_lengths(self.h, *[C.byref(x) for x in v]), "bild_get_lengths")
        return dict(y_len=v[0].value, draft_start=v[1].value, len_small=v[2].value, len_large=v[3].value)

    def sequence(self):
        out = np.zeros(self.max_len + 1, dtype=np.int32)
        n = C.c_int32()
        _check(lib().bild_get_sequence(self.h, out.ctypes.data, len(out), C.byref(n)), "bild_get_sequence")
        return out[:n.value].tolist()

    def debug_enable_logits(self, enable: bool = True):
        _check(lib().bild_debug_enable_logits(self.h, int(enable)), "bild_debug_enable_logits")

    def debug_logits(self, which: int, row: int) -> np.ndarray:
        v = self.pair.large.cfg.vocab
        out = np.zeros(v, dtype=np.float32)
        _check(lib().bild_debug_logits(self.h, which, row, out.ctypes.data), "bild_debug_logits")
        return out

    def debug_kv(self, which: int, layer: int, is_v: bool, pos0: int, n: int) -> np.ndarray:
        """Cached keys or values of one decoder layer, rows pos0..pos0+n-1, as [n][heads*d_head] float32."""
        cfg = (self.pair.large if which == LARGE or self.pair.small is None else self.pair.small).cfg
        out = np.zeros((n, cfg.n_heads * cfg.d_head), dtype=np.float32)
        _check(lib().bild_debug_kv(self.h, which, layer, int(is_v), pos0, n, out.ctypes.data), "bild_debug_kv")
        return out

    def bench_pass(self, which: int, rows: int, reps: int) -> float:
        ms = C.c_float()
        _check(lib().bild_bench_pass(self.h, which, rows, reps, C.byref(ms)), "bild_bench_pass")
        return ms.value

    def bench_gemm(self, which: int, rows: int, reps: int) -> dict:
        ms, n, b = C.c_float(), C.c_int64(), C.c_int64()
        _check(lib().bild_bench_gemm(self.h, which, rows, reps, C.byref(ms), C.byref(n), C.byref(b)), "bild_bench_gemm")
        return dict(ms_per_pass=ms.value, launches=n.value, bytes=b.value)

    def pass_stages(self) -> int:
        n = C.c_int32()
        _check(lib().bild_pass_stages(self.h, C.byref(n)), "bild_pass_stages")
        return n.value

    def gemm_tally(self, reset: bool = False) -> dict:
        n, b = C.c_int64(), C.c_int64()
        _check(lib().bild_gemm_tally(self.h, C.byref(n), C.byref(b), int(reset)), "bild_gemm_tally")
        return dict(launches=n.value, bytes=b.value)

    def probe_stream(self, groups: int, kib_per_group: int, reps: int = 8) -> float:
        us = C.c_float()
        _check(lib().bild_probe_stream(self.h, groups, kib_per_group, reps, C.byref(us)), "bild_probe_stream")
        return us.value

    def probe_launch(self, reps: int = 2000) -> float:
        us = C.c_float()
        _check(lib().bild_probe_launch(self.h, reps, C.byref(us)), "bild_probe_launch")
        return us.value

    def probe_copy(self, nbytes: int, reps: int = 1):
        _check(lib().bild_probe_copy(self.h, nbytes, reps), "bild_probe_copy")

    def profile_begin(self, max_records: int = 65536):
        _check(lib().bild_profile_begin(self.h, max_records), "bild_profile_begin")

    def profile_end(self) -> dict:
        p = Profile()
        _check(lib().bild_profile_end(self.h, C.byref(p)), "bild_profile_end")
        out = {}
        for mi, mn in enumerate(("small", "large")):
            for ci, cn in enumerate(("layers", "lm_head")):
                out[f"{mn}.{cn}"] = dict(launches=p.launches[mi][ci], bytes=p.bytes[mi][ci], ms=p.ms[mi][ci])
        out["dropped"] = p.dropped
        return out

    def pass_bytes(self, which: int, t_cache: int, rows: int = 1) -> int:
        return int(lib().bild_pass_bytes(self.h, which, t_cache, rows))


def tile_matrix(src: np.ndarray, src_is_k_by_n: bool, dtype: int) -> np.ndarray:
    """Host re-layout of a matrix into the kernels' streaming tile order (bytes)."""
    a = np.ascontiguousarray(src, dtype=np.float32)
    k, n = a.shape if src_is_k_by_n else a.shape[::-1]
    nbytes = int(lib().bild_debug_tiled_bytes(n, k, dtype))
    if nbytes < 0:
        raise BildError(nbytes, "bild_debug_tiled_bytes")
    out = np.zeros(nbytes, dtype=np.uint8)
    _check(lib().bild_debug_tile_matrix(a.ctypes.data, int(src_is_k_by_n), n, k, dtype, out.ctypes.data), "bild_debug_tile_matrix")
    return out


def gemm_shape(n: int, k: int, rows: int, gated: bool = False, lm_head: bool = False, dtype: int = 1) -> dict:
    out = (C.c_int32 * 8)()
    _check(lib().bild_debug_gemm_shape(n, k, rows, int(gated), int(lm_head), dtype, out), "bild_debug_gemm_shape")
    keys = ("wk", "nwv", "rw", "kc", "blocks", "row_blocks", "lds", "lds_limit")
    return dict(zip(keys, [int(v) for v in out]))


def attn_shape(heads: int, d_head: int, rows: int, nkeys: int, max_splits: int = 8, dtype: int = 1) -> dict:
    out = (C.c_int32 * 4)()
    _check(lib().bild_debug_attn_shape(heads, d_head, rows, nkeys, max_splits, dtype, out), "bild_debug_attn_shape")
    return dict(zip(("splits", "defer", "waves", "lds"), [int(v) for v in out]))
