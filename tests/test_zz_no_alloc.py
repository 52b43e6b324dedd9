"""bild_head_stats_static (the entry point that allocates nothing) against bild_head_stats, through the C ABI:
two calls in a row, the second with a smaller input, both checked against the allocating entry point and the oracle."""
import numpy as np
import pytest

import bild_inputs as bi
import paper_2302_07863_amd as pkg
from paper_2302_07863_amd import binding as b
from tests import parity
from tests.test_gpu_head_stats import check_against_oracle, run_head_stats

pytestmark = pytest.mark.gpu


def _same(a, c):
    for f in ("zmax", "lse", "z_target"):
        assert np.array_equal(a[f], c[f], equal_nan=True), f
    assert np.array_equal(a["argmax"], c["argmax"])


@pytest.mark.parametrize("dtype", [bi.DT_F32, bi.DT_BF16])
def test_static_scratch_entry_point_matches_the_allocating_one(dtype):
    rng = np.random.default_rng(21)
    # first call: 17 rows on a vocabulary of 40000; second call: 3 rows on a vocabulary of 1000 (fewer workgroups,
    # fewer rows: whatever the first call left in the array must not show)
    big = bi.toy_pair(dtype=dtype, tied=False, vocab=40000)
    small = bi.toy_pair(dtype=dtype, tied=False, vocab=1000, d=256, heads=3, d_head=32, d_ff=160)
    models = []
    for cfg in (big, small):
        _, wl = bi.make_pair_weights(cfg)
        models.append((cfg, wl, parity.make_gpu_model(cfg.large, wl)))
    calls = []
    for (cfg, wl, model), rows in zip(models, (17, 3)):
        x = rng.standard_normal((rows, cfg.large.d)).astype(np.float32) * 3.0
        targets = rng.integers(0, cfg.large.vocab, size=rows)
        calls.append((cfg, wl, model, x, targets))
    got = [run_head_stats(model, x, targets, entry="bild_head_stats_static") for cfg, wl, model, x, targets in calls]
    for (cfg, wl, model, x, targets), g in zip(calls, got):
        _same(g, run_head_stats(model, x, targets))                      # bit for bit what the allocating call returns
        check_against_oracle(cfg.large, wl, x, targets, g, parity.logit_tol(cfg))
    # without targets, right after a call that had them
    cfg, wl, model, x, targets = calls[1]
    g = run_head_stats(model, x[:2], None, entry="bild_head_stats_static")
    assert np.all(np.isnan(g["z_target"]))
    _same(g, run_head_stats(model, x[:2], None))


def test_static_scratch_entry_point_rejects_bad_arguments():
    cfg = bi.toy_pair()
    _, wl = bi.make_pair_weights(cfg)
    model = parity.make_gpu_model(cfg.large, wl)
    from tests.hipmem import DeviceArray
    xd, out = DeviceArray(nbytes=40 * cfg.large.d * 4), DeviceArray(nbytes=40 * 16)
    for rows, xp, op in ((0, xd.ptr.value, out.ptr.value), (33, xd.ptr.value, out.ptr.value), (4, 0, out.ptr.value)):
        with pytest.raises(pkg.BildError) as e:
            b.head_stats(model, xp, rows, None, op, None, "bild_head_stats_static")
        assert e.value.code == b.EINVAL
