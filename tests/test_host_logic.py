"""Host logic of the library, without a GPU: the weight re-layout against the documented tile order written
out independently in numpy, and invariants of the GEMM launch shapes over the shapes of every configuration."""
import numpy as np
import pytest

import bild_inputs as bi
from paper_2302_07863_amd import binding as b


def _bf16_bits(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def _expected_tiles(w_n_by_k, dtype):
    """Tile order from its description: tiles of 16 features x KT inputs, 1 KiB each, feature blocks outermost and
    tiles of a block contiguous along the inputs; lane l of a tile owns feature l % 16 and KT/4 consecutive inputs
    starting at (l // 16) * KT/4."""
    n, k = w_n_by_k.shape
    kt = 32 if dtype == bi.DT_BF16 else 16
    per = kt // 4
    tn = (n + 15) // 16
    padded = np.zeros((tn * 16, k), dtype=np.float32)
    padded[:n] = w_n_by_k
    t = padded.reshape(tn, 16, k // kt, 4, per)          # [block, feature, k tile, lane group, j]
    t = t.transpose(0, 2, 3, 1, 4)                          # [block, k tile, lane group, feature, j] = lanes in order
    flat = np.ascontiguousarray(t).reshape(-1)
    return _bf16_bits(flat).view(np.uint8) if dtype == bi.DT_BF16 else flat.view(np.uint8)


@pytest.mark.parametrize("dtype", [bi.DT_F32, bi.DT_BF16])
@pytest.mark.parametrize("n,k", [(16, 32), (40, 96), (200, 64), (33, 160)])
def test_tile_matrix_matches_the_documented_order(dtype, n, k):
    rng = np.random.default_rng(n * 1000 + k)
    w = rng.normal(size=(n, k)).astype(np.float32)
    want = _expected_tiles(w, dtype)
    assert np.array_equal(b.tile_matrix(w, False, dtype), want)
    assert np.array_equal(b.tile_matrix(np.ascontiguousarray(w.T), True, dtype), want)      # math layout [k][n]
    assert len(want) == ((n + 15) // 16) * (k // (32 if dtype == bi.DT_BF16 else 16)) * 1024


def _projections(shape):
    d, i, f = shape.d, shape.inner, shape.d_ff
    out = [(3 * i, d, False, False), (i, d, False, False), (d, i, False, False), (f, d, shape.gated, False),
           (d, f, False, False), (shape.vocab, d, False, True)]
    if shape.cross:
        out.append((2 * i, d, False, False))
    return out


@pytest.mark.parametrize("pair", sorted(bi.PAIRS))
def test_gemm_launch_shapes_are_consistent(pair):
    """Every projection of every configuration, for 1..32 rows and for row-block launches: the waves of a workgroup
    factor into input slices x feature groups, the feature-group workgroups cover every feature tile exactly once,
    the LDS request fits, and the staged chunk is a whole number of input tiles."""
    cfg = bi.PAIRS[pair]()
    for shape in (cfg.small, cfg.large):
        kt = 32 if shape.dtype == bi.DT_BF16 else 16
        for n, k, gated, head in _projections(shape):
            for rows in (1, 2, 3, 4, 7, 11, 16, 17, 32) + (() if head else (33, 512, 1000)):
                s = b.gemm_shape(n, k, rows, gated, head, shape.dtype)
                tiles = ((2 * n if gated else n) + 15) // 16
                if rows > 512:
                    # the dense-tile kernel: 64 rows x (4 waves x 4 feature tiles) per workgroup, chunks of 128 inputs
                    assert (s["wk"], s["nwv"], s["rw"], s["kc"]) == (1, 4, 4, 128)
                    assert (s["blocks"] - 1) * 16 < tiles <= s["blocks"] * 16 and s["row_blocks"] == (rows + 63) // 64
                    assert 2 * s["lds"] <= s["lds_limit"]          # two workgroups share a compute unit (registers)
                    continue
                assert s["nwv"] in (1, 2, 4, 8) and s["nwv"] % s["wk"] == 0, (n, k, rows, s)
                assert s["wk"] in (1, 2, 4, 8), (n, k, rows, s)   # the kernels cut the wave index by shifts
                # feature tiles per wave: 2 = gate and linear branch; 4 only for a very wide LM head at up to 16 rows
                assert s["rw"] == (2 if gated else (4 if head and rows <= 16 and tiles >= 8192 else 1))
                per_wg = (s["nwv"] // s["wk"]) * s["rw"]
                assert (s["blocks"] - 1) * per_wg < tiles <= s["blocks"] * per_wg, (n, k, rows, s)
                assert s["row_blocks"] == (rows + 31) // 32
                assert 0 < s["lds"] <= s["lds_limit"], (n, k, rows, s)
                assert s["kc"] % kt == 0 and s["kc"] >= kt
                assert s["wk"] <= max(1, min(s["kc"], k) // kt)


@pytest.mark.parametrize("pair", sorted(bi.PAIRS))
def test_attention_launch_shapes_are_consistent(pair):
    """Key splits stay within the partial buffers and the grid the kernels assume; partials are left to the consumer
    projection only in the range it merges (at most 8 splits and 16 rows, one (row, head) pair per thread of a 256-thread
    workgroup, a weight table of at most 4 KiB); the LDS request fits; a workgroup
    that is not split further streams at most about 160 KiB unless the split limits are exhausted."""
    cfg = bi.PAIRS[pair]()
    for shape in (cfg.small, cfg.large):
        esz = 2 if shape.dtype == bi.DT_BF16 else 4
        for nkeys in (1, 31, 64, 128, 512, 1024, 2048, 4096):
            for rows in (1, 2, 4, 5, 8, 9, 11, 16, 32, 33, 700):
                for max_splits in (8, 16, 64):
                    s = b.attn_shape(shape.heads, shape.d_head, rows, nkeys, max_splits, shape.dtype)
                    assert 1 <= s["splits"] <= max_splits and shape.heads * s["splits"] <= max(512, shape.heads)
                    assert s["splits"] & (s["splits"] - 1) == 0
                    if rows > 32:
                        assert s["splits"] == 1
                    if s["defer"]:
                        assert 1 < s["splits"] <= 8 and rows <= 16 and rows * shape.heads <= 256
                        assert rows * shape.heads * s["splits"] * 4 <= 4096
                    assert s["waves"] in (1, 2, 4, 8) and 0 < s["lds"] <= 128 * 1024
                    if min(rows, 32) <= 16 and shape.d_head <= 64:
                        assert s["waves"] >= 4      # q is staged in one piece per thread from 256 threads on
                    per_wg = nkeys * shape.d_head * 2 * esz / s["splits"]
                    if per_wg > 160 * 1024 and rows <= 32 and not s["defer"]:
                        assert s["splits"] * 2 > max_splits or shape.heads * s["splits"] * 2 > 512


def test_launch_shape_rules_at_their_boundaries():
    """The measured thresholds of the GEMM launch shapes: eight-wave workgroups once a thread of a four-wave workgroup
    would stage more than eight pieces (rows x inputs > 8192); single-row launches never field between one and two
    workgroups per compute unit; a very wide LM head takes four feature tiles per wave up to 16 rows."""
    assert b.gemm_shape(1024, 1024, 8)["nwv"] == 4 and b.gemm_shape(1024, 1024, 9)["nwv"] == 8
    assert b.gemm_shape(512, 512, 16)["nwv"] == 4 and b.gemm_shape(512, 512, 17)["nwv"] == 8
    one, two = b.gemm_shape(12288, 4096, 1), b.gemm_shape(12288, 4096, 2)
    assert one["blocks"] == 768 and one["nwv"] == 2 and two["blocks"] == 384 and two["nwv"] == 4
    for n, k in ((1024, 1024), (3072, 1024), (4096, 1024), (1024, 4096), (12288, 4096), (22016, 4096), (4096, 11008)):
        blocks = b.gemm_shape(n, k, 1)["blocks"]
        assert not 256 < blocks < 512, (n, k, blocks)
    wide = b.gemm_shape(250112, 512, 1, False, True)
    assert wide["rw"] == 4 and wide["blocks"] * wide["nwv"] * 4 >= 250112 // 16
    assert b.gemm_shape(250112, 512, 17, False, True)["rw"] == 1
    assert b.gemm_shape(32128, 1024, 1, False, True)["rw"] == 1


def test_debug_calls_reject_bad_arguments():
    lib = b.lib()
    assert lib.bild_debug_tiled_bytes(0, 32, 0) == b.EINVAL
    assert lib.bild_debug_tiled_bytes(16, 40, 1) == b.EINVAL
    assert lib.bild_debug_gemm_shape(16, 32, 0, 0, 0, 0, None) == b.EINVAL


def test_launch_shapes_of_ragged_widths_keep_a_power_of_two_of_input_slices():
    """Widths whose tile count is not a power of two (96 inputs = 6 fp32 tiles, 160 = 10) in row-block launches: the
    kernels split the wave index into (input slice, feature group) by shifts, so the slices must be a power of two."""
    for dtype, kt in ((bi.DT_F32, 16), (bi.DT_BF16, 32)):
        for k in (96, 160, 192, 320, 6 * kt, 10 * kt, 12 * kt):
            for n in (48, 96, 288, 1000, 4096):
                for rows in (1, 3, 16, 33, 40, 300):
                    s = b.gemm_shape(n, k, rows, False, False, dtype)
                    assert s["wk"] in (1, 2, 4, 8) and s["nwv"] in (1, 2, 4, 8) and s["nwv"] % s["wk"] == 0, (n, k, rows, s)
                    assert s["wk"] <= max(1, min(s["kc"], k) // kt), (n, k, rows, s)
