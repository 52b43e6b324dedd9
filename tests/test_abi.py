"""The C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments with error codes - without any GPU work."""
import ctypes as C
import os
import re

import pytest

import paper_2302_07863_amd as pkg
from paper_2302_07863_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("bild.h", "bild_bench.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(bild_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = pkg.lib()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(names) == b.exported_symbols()      # the binding covers the whole header


def test_error_strings():
    assert b.strerror(0) == "ok"
    for code in (b.EINVAL, b.ESTATE, b.ECAP, b.EHIP, b.ENOMEM):
        assert b.strerror(code) not in ("ok", "unknown error")
    assert b.strerror(-99) == "unknown error"


def _cfg(**kw):
    base = dict(n_enc_layers=1, n_dec_layers=1, d_model=64, n_heads=2, d_head=16, d_ff=96, act=0, pos=0, vocab=100,
                tied_head=1, dtype=0, cross_attn=1, bos=0, tie_shift=0, logit_scale=1.0, embed_scale=1.0,
                norm_eps=1e-6, rope_base=10000.0)
    base.update(kw)
    return b.ModelConfig(**base)


def test_tensor_count_follows_the_config():
    lib = pkg.lib()
    assert lib.bild_model_num_tensors(C.byref(_cfg())) == 1 + 1 + 1 + 8 + 13
    assert lib.bild_model_num_tensors(C.byref(_cfg(tied_head=0, act=1))) == 2 + 1 + 1 + 9 + 14
    assert lib.bild_model_num_tensors(C.byref(_cfg(n_enc_layers=0, cross_attn=0, act=2, pos=1))) == 1 + 1 + 9
    # relative-position models bring one bias table per stack
    assert lib.bild_model_num_tensors(C.byref(_cfg(pos=2, rel_max_dist=8))) == 1 + 1 + 1 + 2 + 8 + 13
    assert lib.bild_model_num_tensors(C.byref(_cfg(n_enc_layers=0, cross_attn=0, pos=2, rel_max_dist=8))) == 1 + 1 + 1 + 8
    import bild_inputs as bi
    for kw in (dict(pos=bi.POS_RELATIVE), dict(pos=bi.POS_RELATIVE, cross=False, tied=False)):
        for shape in (bi.toy_pair(**kw).large, bi.toy_pair(**kw).small):
            assert lib.bild_model_num_tensors(C.byref(pkg.config_from_shape(shape))) == len(bi.tensor_names(shape))


@pytest.mark.parametrize("kw", [dict(d_model=48), dict(d_ff=100), dict(d_head=12), dict(d_head=256), dict(act=3),
                                dict(pos=3), dict(pos=2), dict(pos=2, rel_max_dist=5000), dict(dtype=5), dict(vocab=0), dict(bos=100), dict(n_dec_layers=0),
                                dict(n_enc_layers=1, cross_attn=0), dict(tie_shift=-1), dict(rope_base=0.0)])
def test_bad_configs_are_rejected_before_any_device_work(kw):
    lib = pkg.lib()
    cfg = _cfg(**kw)
    assert lib.bild_model_num_tensors(C.byref(cfg)) == b.EINVAL
    h = C.c_void_p()
    ptrs = (C.c_void_p * 4)()
    assert lib.bild_model_create(C.byref(cfg), ptrs, 4, C.byref(h)) == b.EINVAL
    assert not h.value


def test_null_arguments():
    lib = pkg.lib()
    h = C.c_void_p()
    assert lib.bild_model_create(None, None, 0, C.byref(h)) == b.EINVAL
    cfg = _cfg()
    n = lib.bild_model_num_tensors(C.byref(cfg))
    ptrs = (C.c_void_p * n)()                    # all NULL tensors
    assert lib.bild_model_create(C.byref(cfg), ptrs, n, C.byref(h)) == b.EINVAL
    assert lib.bild_model_create(C.byref(cfg), ptrs, n - 1, C.byref(h)) == b.EINVAL
    assert lib.bild_pair_create(None, None, C.byref(h)) == b.EINVAL
    assert lib.bild_state_create(None, 8, 8, 10, None, C.byref(h)) == b.EINVAL
    assert lib.bild_encode(None, None, 0) == b.EINVAL
    t, f = C.c_int32(), C.c_int32()
    assert lib.bild_small_step(None, 0.5, C.byref(t), C.byref(f), None) == b.EINVAL
    assert lib.bild_large_verify(None, None, 0, 1.0, None, None, None, None) == b.EINVAL
    assert lib.bild_kv_truncate(None, 3, 0) == b.EINVAL
    assert lib.bild_seq_truncate(None, 1) == b.EINVAL
    assert lib.bild_force_tokens(None, 0, None, 0, 0) == b.EINVAL
    assert lib.bild_generate(None, None, 0, 0.5, 2.0, 4, -1, None, None, None) == b.EINVAL
    assert lib.bild_greedy(None, 1, None, 0, 4, -1, None, None) == b.EINVAL
    assert lib.bild_model_destroy(None) == b.EINVAL
    assert lib.bild_pair_destroy(None) == b.EINVAL
    assert lib.bild_state_destroy(None) == b.EINVAL
    assert lib.bild_pass_bytes(None, 1, 0, 1) == b.EINVAL


def test_product_code_never_imports_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2302_07863_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    text = open(os.path.join(ROOT, "bild_inputs", "generate.py")).read() + open(os.path.join(ROOT, "bild_inputs", "configs.py")).read()
    assert "oracle" not in text.replace("CPU oracle", "") or "import oracle" not in text
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2302_07863_amd" not in text and "ctypes" not in text, f
