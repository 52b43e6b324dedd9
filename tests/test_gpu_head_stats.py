"""bild_head_stats: the fused final norm + LM head + softmax statistics as a call of its own, on hidden rows the
caller holds on the device, against the oracle's head and policy quantities (Sections 3.2-3.4)."""
import numpy as np
import pytest

import bild_inputs as bi
import oracle
import paper_2302_07863_amd as pkg
from paper_2302_07863_amd import binding as b
from tests import parity
from tests.hipmem import DeviceArray

pytestmark = pytest.mark.gpu


def run_head_stats(model, x, targets, entry="bild_head_stats"):
    """x [rows][d] float32 numpy, targets [rows] int or None -> records of binding.ROW_STATS_DTYPE (numpy)."""
    xd = DeviceArray(np.ascontiguousarray(x, dtype=np.float32))
    td = DeviceArray(np.ascontiguousarray(targets, dtype=np.int32)) if targets is not None else None
    out = DeviceArray(nbytes=len(x) * b.ROW_STATS_DTYPE.itemsize)
    b.head_stats(model, xd.ptr.value, len(x), td.ptr.value if td is not None else None, out.ptr.value, None, entry)
    return out.to_host(b.ROW_STATS_DTYPE, len(x))


def check_against_oracle(shape, weights, x, targets, got, tol):
    m = oracle.Model(shape, weights)
    z = m.logits_from_hidden(np.asarray(x, dtype=np.float64))
    for t in range(len(x)):
        assert abs(float(got["zmax"][t]) - float(np.max(z[t]))) <= tol, t
        assert abs(float(got["lse"][t]) - oracle.policy.logsumexp(z[t])) <= tol, t
        assert int(got["argmax"][t]) == int(np.argmax(z[t])) or oracle.policy.top2_gap(z[t]) < parity.MARGIN, t
        if targets is None:
            assert np.isnan(got["z_target"][t])
        else:
            assert abs(float(got["z_target"][t]) - float(z[t][targets[t]])) <= tol, t
            # the two policy quantities built from the record
            assert abs(float(np.exp(got["zmax"][t] - got["lse"][t])) - oracle.policy.max_prob(z[t])) <= 2 * tol
            assert abs(float(got["lse"][t] - got["z_target"][t]) - oracle.policy.nll(z[t], int(targets[t]))) <= 2 * tol


@pytest.mark.parametrize("kw", [dict(), dict(dtype=bi.DT_BF16), dict(tied=False, vocab=1000, d=256, heads=3, d_head=32, d_ff=160),
                                dict(dtype=bi.DT_BF16, tied=False, vocab=40000)])
def test_head_stats_against_the_oracle(kw):
    cfg = bi.toy_pair(**kw)
    _, wl = bi.make_pair_weights(cfg)
    shape = cfg.large
    model = parity.make_gpu_model(shape, wl)
    rng = np.random.default_rng(11)
    tol = parity.logit_tol(cfg)
    for rows in (1, 3, 17, 32):
        x = rng.standard_normal((rows, shape.d)).astype(np.float32) * 3.0
        targets = rng.integers(0, shape.vocab, size=rows)
        check_against_oracle(shape, wl, x, targets, run_head_stats(model, x, targets), tol)
    x = rng.standard_normal((2, shape.d)).astype(np.float32)
    check_against_oracle(shape, wl, x, None, run_head_stats(model, x, None), tol)


def test_head_stats_t5_small_shape_and_errors():
    cfg = bi.t5_pair()
    ws, _ = bi.make_pair_weights(replace_large_with_small(cfg))
    shape = cfg.small
    model = parity.make_gpu_model(shape, ws)
    rng = np.random.default_rng(12)
    x = rng.standard_normal((11, shape.d)).astype(np.float32) * 2.0
    targets = rng.integers(0, shape.vocab, size=11)
    check_against_oracle(shape, ws, x, targets, run_head_stats(model, x, targets), parity.logit_tol(cfg))
    xd = DeviceArray(nbytes=40 * shape.d * 4)
    out = DeviceArray(nbytes=40 * 16)
    for rows, xp, op in ((0, xd.ptr.value, out.ptr.value), (33, xd.ptr.value, out.ptr.value), (4, 0, out.ptr.value),
                         (4, xd.ptr.value, 0), (4, xd.ptr.value + 4, out.ptr.value)):
        with pytest.raises(pkg.BildError) as e:
            b.head_stats(model, xp, rows, None, op)
        assert e.value.code == b.EINVAL


def replace_large_with_small(cfg):
    """A pair whose `large` is the small model's shape: weights of the small model alone, without drawing the large one."""
    from dataclasses import replace
    return replace(cfg, large=cfg.small)
