"""GPU parity of the persistent pass kernel (opt-in, BILD_RESIDENT=1): the same oracle
comparisons as the default one-kernel-per-stage path, with few resident workgroups so
that stages loop over several units of work, and the barrier's give-up path."""
import pytest

import bild_inputs as bi
import oracle
import paper_2302_07863_amd as pkg
from tests import parity
from tests.test_gpu_parity import Rig, TOY_VARIANTS

pytestmark = pytest.mark.gpu


@pytest.fixture
def resident(monkeypatch):
    def set_(groups, spin=None):
        monkeypatch.setenv("BILD_RESIDENT", "1")
        monkeypatch.setenv("BILD_RESIDENT_G", str(groups))
        if spin is not None:
            monkeypatch.setenv("BILD_BARRIER_SPIN", str(spin))
    return set_


@pytest.mark.parametrize("name,groups", [("f32-relu-tied", 3), ("bf16-trunc-geglu", 8), ("bf16-rope-swiglu-deconly", 5),
                                         ("f32-wide", 16)])
def test_resident_toy_parity(resident, name, groups):
    resident(groups)
    R = Rig(bi.toy_pair(**TOY_VARIANTS[name]))
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
        st = R.state(R.cfg.max_new, nm)
        st.encode(R.src)
        worst = parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg)
        toks, stats = st.generate(R.src, fb, rb, R.cfg.max_new)
        res = parity.compare_generation(toks, stats, ref, fb, rb)
        print(name, groups, worst, res)


def test_resident_tiny_config(resident):
    resident(32)
    cfg = bi.tiny_pair()
    R = Rig(cfg)
    ref = oracle.bild_generate(R.req, cfg.alpha_fb, cfg.alpha_rb, cfg.n_max, cfg.max_new, keep_logits=True)
    st = R.state(cfg.max_new, cfg.n_max)
    st.encode(R.src)
    print(parity.teacher_forced(st, ref, R.n0, cfg.alpha_fb, cfg.alpha_rb, cfg))
    toks, stats = st.generate(R.src, cfg.alpha_fb, cfg.alpha_rb, cfg.max_new)
    print(parity.compare_generation(toks, stats, ref, cfg.alpha_fb, cfg.alpha_rb), stats)


def test_resident_barrier_gives_up_cleanly(resident, monkeypatch):
    """A barrier wait that runs out must end the kernel, surface as an error, and leave the
    library usable: the host forces the give-up path (limit -1), every workgroup exits."""
    resident(4, spin=-1)
    R = Rig(bi.toy_pair())
    st = R.state(R.cfg.max_new, 4)
    with pytest.raises(pkg.BildError) as e:
        st.generate(R.src, 0.5, 2.0, R.cfg.max_new)
    assert e.value.code == -4  # BILD_EHIP
    monkeypatch.delenv("BILD_BARRIER_SPIN")
    st2 = R.state(R.cfg.max_new, 4)
    ref = oracle.bild_generate(R.req, 0.5, 2.0, 4, R.cfg.max_new)
    toks, stats = st2.generate(R.src, 0.5, 2.0, R.cfg.max_new)
    parity.compare_generation(toks, stats, ref, 0.5, 2.0)


def test_plain_launches_without_graph_replay(monkeypatch):
    """BILD_NO_GRAPH=1 (the configuration profiles are taken in): every kernel launched directly, same results."""
    monkeypatch.setenv("BILD_NO_GRAPH", "1")
    R = Rig(bi.toy_pair(**TOY_VARIANTS["bf16-trunc-geglu"]))
    for fb, rb, nm in ((0.5, 2.0, 10), (0.2, 0.7, 3)):
        ref = oracle.bild_generate(R.req, fb, rb, nm, R.cfg.max_new, keep_logits=True)
        st = R.state(R.cfg.max_new, nm)
        st.encode(R.src)
        print(parity.teacher_forced(st, ref, R.n0, fb, rb, R.cfg))
        toks, stats = st.generate(R.src, fb, rb, R.cfg.max_new)
        print(parity.compare_generation(toks, stats, ref, fb, rb))
