"""Shape accounting against what the paper prints (Table 2) and states
(Section 3.2 and the appendix's model analysis: a pass over n rows costs the
flops of n single-row passes but one weight load)."""
import os

import bild_inputs as bi

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table2_decoder_params.txt")


def _table2():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, layers, dim, ffn, params = line.split()
        rows[name] = (int(layers), int(dim), int(ffn), int(params))
    return rows


def test_table2_decoder_parameter_counts():
    gold = _table2()
    shapes = {}
    for pair in (bi.t5_pair(), bi.mt5_pair()):
        shapes[pair.small.name] = pair.small
        shapes[pair.large.name] = pair.large
    assert set(shapes) == set(gold)
    for name, (layers, dim, ffn, millions) in gold.items():
        s = shapes[name]
        assert (s.n_dec, s.d, s.d_ff) == (layers, dim, ffn)
        # the table mixes rounding and truncation (402.65M is printed as 402M)
        assert abs(s.decoder_params() / 1e6 - millions) < 1.0, (name, s.decoder_params())


def test_size_ratio_about_twenty():
    # Section 4.1: the two models of a pair differ in size by roughly a factor of 20.
    for pair in (bi.t5_pair(), bi.mt5_pair()):
        assert 14 < pair.large.decoder_params() / pair.small.decoder_params() < 20


def test_rows_cost_same_flops_but_one_weight_load():
    for pair in bi.PAIRS.values():
        m = pair().large
        n_src = pair().n_src
        t0, rows = 17, 11
        seq = sum(m.pass_flops(t0 + r, n_src, 1) for r in range(rows))
        assert m.pass_flops(t0, n_src, rows) == seq
        one = m.pass_bytes(t0, n_src, 1)
        many = m.pass_bytes(t0, n_src, rows)
        # only the K/V rows of the extra tokens are added; weights are read once
        assert many - one == m.elem_bytes * m.n_dec * 2 * m.inner * (rows - 1)
        assert many < 1.01 * one


def test_bytes_per_pass_match_the_configured_shapes():
    # decoder weights + LM head + self K/V at the end-of-generation length + cross K/V
    t5 = bi.t5_pair()
    assert abs(t5.small.pass_bytes(64, 512, 0) / 1e6 - 90.3) < 0.1
    assert abs(t5.large.pass_bytes(64, 512, 0) / 1e6 - 927.7) < 0.2
    mt5 = bi.mt5_pair()
    assert abs(mt5.small.pass_bytes(64, 64, 0) / 1e6 - 308.0) < 0.5
    assert abs(mt5.large.pass_bytes(64, 64, 0) / 1e6 - 1342.7) < 0.5


def test_generator_is_seeded_and_bf16_exact():
    import numpy as np
    cfg = bi.toy_pair(dtype=bi.DT_BF16, truncate=True)
    ws, wl = bi.make_pair_weights(cfg)
    ws2, wl2 = bi.make_pair_weights(cfg)
    for k in wl:
        assert np.array_equal(wl[k], wl2[k])
        if wl[k].ndim == 2:
            assert np.all((wl[k].view(np.uint32) & 0xFFFF) == 0), k     # bf16-representable
            assert abs(float(wl[k].std()) - 0.02) < 0.004
    assert np.array_equal(ws["dec.0.wq"], wl["dec.0.wq"][:cfg.small.d, :cfg.small.inner])
    assert np.array_equal(ws["emb"], wl["emb"][:, :cfg.small.d])
    src = bi.make_source(bi.t5_pair())
    assert src.min() >= 0 and src.max() < 32128 and len(src) == 512
    assert np.mean(src < 10) > 0.2          # Zipf: low ranks dominate


def test_bf16_value_rounding_matches_torch():
    import numpy as np
    import torch
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    a[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0]     # exact ties
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(bi.to_bf16_values(a), ref)
