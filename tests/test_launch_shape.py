"""Host-side launch-shape logic (es_spmm_launch_info): runs without a GPU.
Checks the invariants the kernels rely on before anything is launched."""
import itertools

import pytest

import paper_2104_10716_amd as es


SHAPES = [(1, 0), (7, 20), (2708, 13518), (170_000, 2_370_240), (233_000, 113_134_823),
          (2_450_000, 119_569_270)]
WIDTHS = [1, 2, 3, 4, 5, 16, 17, 41, 48, 64, 100, 128, 130, 256, 512, 602, 1024, 1028, 5000]


def _check(info, N, F, backward):
    G, CH, V = info["lanes_per_row"], info["chunks_per_lane"], info["vector_width"]
    R, E = info["rows_per_wave"], info["edge_slots"]
    assert V in (1, 4) and CH in (1, 2, 4) and G in (4, 8, 16, 32, 64)
    if info["flattened"]:
        assert R * G in (64, 128) and E * G == 64         # a wave lays E or 2E rows end to end for its E slots
    else:
        assert R * G * E == 64 and E >= 1                 # a wave is R rows x E slots x G lanes
    assert info["loads_in_flight"] * CH == 8
    assert info["tile_slots_per_row"] * R == es.es_spmm_tile_slots(1)
    assert G * CH * V * info["grid_y"] >= F               # every column is covered ...
    assert G * CH * V * (info["grid_y"] - 1) < F          # ... by no more column blocks than needed
    rows_per_workgroup = 4 * R
    row_groups = info["grid_x"] - info["long_row_workgroups"]
    if info["column_ranges"] == 8 and not info["flattened"]:   # a wave serves 4 rows; two sweeps per launch
        rows_per_workgroup *= 4
        assert info["long_row_workgroups"] == row_groups
    assert row_groups % 8 == 0                            # one equal share per XCD
    assert row_groups * rows_per_workgroup >= N
    assert info["long_row_workgroups"] % 8 == 0
    assert info["long_row_threshold"] >= 64
    if backward:
        assert V == 1 and info["aligned"] == 0
    if V == 4 and not info["aligned"]:
        assert F >= 4


@pytest.mark.parametrize("backward", [False, True])
def test_shape_invariants_over_sizes_and_widths(backward):
    for (N, nnz), F, mode, W in itertools.product(SHAPES, WIDTHS, ("full", "bucket", "fastrand"),
                                                  (1, 16, 128, 2304)):
        for aligned in (True, False):
            info = es.es_spmm_launch_info(N, nnz, F, W, mode, aligned16=aligned, backward=backward)
            _check(info, N, F, backward)
            if not backward:
                expect_aligned = aligned and F % 4 == 0
                assert info["aligned"] == int(expect_aligned)
                assert info["vector_width"] == (4 if F >= 4 else 1)


def test_long_rows_are_only_possible_when_the_long_part_is_launched():
    for (N, nnz), F in itertools.product(SHAPES, (16, 64, 128, 41)):
        full = es.es_spmm_launch_info(N, nnz, F, 0, "full", opts=dict(column_partition=-1))
        assert full["long_row_workgroups"] > 0            # nnz is only a hint: never gated by it
        assert full["column_ranges"] == 1
        auto = es.es_spmm_launch_info(N, nnz, F, 0, "full")
        # the column-partitioned product sweeps its rows twice per launch (long pieces first)
        if auto["column_ranges"] == 8 and not auto["flattened"]:
            assert auto["long_row_workgroups"] * 2 == auto["grid_x"]
        for W in (1, 16, 128, 512):
            s = es.es_spmm_launch_info(N, nnz, F, W, "fastrand")
            assert s["long_row_threshold"] >= 512 and s["long_row_workgroups"] == 0
        big = es.es_spmm_launch_info(N, nnz, F, 2304, "bucket")
        assert (big["long_row_workgroups"] > 0) == (2304 > big["long_row_threshold"])


def test_options_are_honoured_and_clamped():
    base = es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket")
    info = es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket", opts=dict(rows_per_wave=64))
    assert info["lanes_per_row"] == 16 and info["rows_per_wave"] == 4      # lowered to fit G
    assert es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket", opts=dict(rows_per_wave=1))["rows_per_wave"] == 1
    info = es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket", opts=dict(long_row_threshold=7))
    assert info["long_row_threshold"] == 7 and info["long_row_workgroups"] > 0
    # options travel with the call: the next call without them sees the heuristic again
    assert es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket") == base
    assert base["long_row_workgroups"] == 0
    # an all-zero struct is the same as no struct
    assert es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket", opts={}) == base
    for bad in (dict(rows_per_wave=3), dict(rows_per_wave=-1), dict(lanes_per_row=12), dict(lanes_per_row=-2),
                dict(long_row_threshold=-4), dict(column_partition=-2)):
        with pytest.raises(es.EsSpmmError):
            es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket", opts=bad)


def test_option_grid_keeps_the_shape_invariants():
    for (N, nnz), F, mode in itertools.product(SHAPES[1:], (3, 16, 41, 64, 128, 256, 602), ("full", "fastrand")):
        for rpw, lanes, thr in itertools.product((0, 1, 8, 64), (0, -1, 4, 8, 32, 64), (0, 1, 100)):
            opts = dict(rows_per_wave=rpw, lanes_per_row=lanes, long_row_threshold=thr)
            for backward in (False, True):
                info = es.es_spmm_launch_info(N, nnz, F, 64, mode, backward=backward, opts=opts)
                assert info["long_row_threshold"] >= (thr if thr else 64)
                if thr and info["column_ranges"] == 1:
                    assert info["long_row_threshold"] == thr
                G, CH, V = info["lanes_per_row"], info["chunks_per_lane"], info["vector_width"]
                assert info["rows_per_wave"] * G * info["edge_slots"] == (64 * info["rows_per_wave"] if info["flattened"] else 64)
                assert G * CH * V * info["grid_y"] >= F
                groups = 4 if info["column_ranges"] == 8 and not info["flattened"] else 1
                assert (info["grid_x"] - info["long_row_workgroups"]) * 4 * info["rows_per_wave"] * groups >= N


def test_column_slicing_option_only_narrows():
    base = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket", opts=dict(lanes_per_row=-1))
    assert base["lanes_per_row"] == 32 and base["grid_y"] == 1
    sliced = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket", opts=dict(lanes_per_row=8))
    assert sliced["lanes_per_row"] == 8 and sliced["chunks_per_lane"] == 1 and sliced["grid_y"] == 4
    _check(sliced, 1000, 128, False)
    wide = es.es_spmm_launch_info(1000, 9000, 16, 8, "bucket", opts=dict(lanes_per_row=8))
    assert wide["lanes_per_row"] == 4 and wide["grid_y"] == 1           # already narrower than 8 lanes
    bwd = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket", backward=True, opts=dict(lanes_per_row=8))
    assert bwd["lanes_per_row"] == 64                                   # the transposed product ignores it


def test_column_partition_choice():
    """Dense graph whose eighth of X is near an L2: partitioned for the exact
    product and for wide FastRand, never for Bucket, never for sparse graphs or
    for tables far beyond the L2s; the option forces it either way."""
    dense = (233_000, 113_134_823)
    assert es.es_spmm_launch_info(*dense, 64, 0, "full")["column_ranges"] == 8
    assert es.es_spmm_launch_info(*dense, 64, 256, "fastrand")["column_ranges"] == 1      # only on request
    assert es.es_spmm_launch_info(*dense, 64, 256, "fastrand", opts=dict(column_partition=1))["column_ranges"] == 8
    assert es.es_spmm_launch_info(*dense, 64, 256, "bucket")["column_ranges"] == 1
    assert es.es_spmm_launch_info(*dense, 64, 256, "bucket", opts=dict(column_partition=1))["column_ranges"] == 1
    assert es.es_spmm_launch_info(*dense, 64, 0, "full", opts=dict(column_partition=-1))["column_ranges"] == 1
    assert es.es_spmm_launch_info(170_000, 2_370_240, 128, 0, "full")["column_ranges"] == 1      # 14 per row
    assert es.es_spmm_launch_info(2_450_000, 119_569_270, 128, 0, "full")["column_ranges"] == 1  # X far too big
    forced = es.es_spmm_launch_info(170_000, 2_370_240, 128, 0, "full", opts=dict(column_partition=1, kernel=1))
    assert forced["column_ranges"] == 8 and forced["long_row_workgroups"] * 2 == forced["grid_x"]
    assert forced["long_row_workgroups"] % 8 == 0 and forced["lanes_per_row"] == 16
    forced = es.es_spmm_launch_info(170_000, 2_370_240, 128, 0, "full", opts=dict(column_partition=1))
    assert forced["column_ranges"] == 8 and forced["flattened"] == 1 and forced["lanes_per_row"] == 8
    assert es.es_spmm_launch_info(100, 5000, 64, 0, "full", opts=dict(column_partition=1))["column_ranges"] == 1
    assert es.es_spmm_launch_info(*dense, 64, 0, "full", backward=True)["column_ranges"] == 1


def test_flattened_kernel_choice():
    """Without options the flattened kernel runs where narrow column slices pay:
    the partitioned product once a 64-column share outgrows an L2, and tables of
    0.3 GB and more with F >= 128; the row kernel everywhere else."""
    big = es.es_spmm_launch_info(2_450_000, 119_569_270, 128, 32, "fastrand")
    assert big["flattened"] == 1 and big["lanes_per_row"] == 8 and big["grid_y"] == 4 and big["rows_per_wave"] == 16
    exact = es.es_spmm_launch_info(2_450_000, 119_569_270, 128, 0, "full")
    assert exact["flattened"] == 1 and exact["rows_per_wave"] == 8            # one row per slot: evens the waves out
    row = es.es_spmm_launch_info(2_450_000, 119_569_270, 128, 32, "fastrand", opts=dict(kernel=1))
    assert row["flattened"] == 0 and row["lanes_per_row"] == 16
    dense = es.es_spmm_launch_info(233_000, 113_134_823, 64, 0, "full")
    assert dense["flattened"] == 1 and dense["column_ranges"] == 8 and dense["lanes_per_row"] == 8
    small = es.es_spmm_launch_info(58_250, 27_659_516, 64, 0, "full")
    assert small["flattened"] == 0 and small["column_ranges"] == 8 and small["lanes_per_row"] == 16
    assert es.es_spmm_launch_info(233_000, 113_134_823, 64, 64, "fastrand")["flattened"] == 0
    assert es.es_spmm_launch_info(233_000, 113_134_823, 256, 64, "fastrand")["flattened"] == 0   # 0.24 GB table
    assert es.es_spmm_launch_info(170_000, 2_370_240, 128, 16, "bucket")["flattened"] == 0
    assert es.es_spmm_launch_info(2_450_000, 119_569_270, 128, 32, "fastrand", backward=True)["flattened"] == 0
    # rows that do not tile 128-byte lines (F = 41, stride 41) keep the row kernel on whole rows
    odd = es.es_spmm_launch_info(233_000, 113_134_823, 41, 0, "full", aligned16=False)
    assert odd["flattened"] == 0 and odd["column_ranges"] == 8 and odd["lanes_per_row"] == 16


def test_flattened_kernel_option():
    for F, G in ((16, 4), (64, 16), (128, 32), (256, 64), (602, 64), (41, 16)):
        info = es.es_spmm_launch_info(100_000, 1_000_000, F, 16, "fastrand", aligned16=(F % 4 == 0),
                                      opts=dict(kernel=2, lanes_per_row=-1))
        assert info["flattened"] == 1 and info["lanes_per_row"] == G and info["chunks_per_lane"] == 1
        assert info["rows_per_wave"] == 128 // G and info["edge_slots"] == 64 // G   # sampled: two rows per slot
        assert info["grid_y"] == -(-F // (4 * G))
        _check(info, 100_000, F, False)
    assert es.es_spmm_launch_info(1000, 5000, 3, 2, "bucket", opts=dict(kernel=2))["flattened"] == 0    # F < 4
    assert es.es_spmm_launch_info(1000, 5000, 64, 2, "bucket", backward=True, opts=dict(kernel=2))["flattened"] == 0
    assert es.es_spmm_launch_info(1000, 5000, 64, 2, "bucket", opts=dict(kernel=1))["flattened"] == 0
    part = es.es_spmm_launch_info(10_000, 5_000_000, 64, 0, "full", opts=dict(kernel=2, column_partition=1))
    assert part["flattened"] == 1 and part["column_ranges"] == 8 and part["long_row_workgroups"] == 0
    fr = es.es_spmm_launch_info(10_000, 5_000_000, 64, 9, "fastrand", opts=dict(kernel=2, column_partition=1))
    assert fr["flattened"] == 0 and fr["column_ranges"] == 8                # FastRand pieces: the row form
    with pytest.raises(es.EsSpmmError):
        es.es_spmm_launch_info(1000, 5000, 64, 2, "bucket", opts=dict(kernel=3))


def test_bad_sizes_are_rejected():
    for kw in (dict(N=0), dict(F=0), dict(W=0), dict(mode=5), dict(nnz=-1), dict(ldx=3)):
        a = dict(N=10, nnz=20, F=4, W=2, mode="bucket", ldx=None)
        a.update(kw)
        with pytest.raises(es.EsSpmmError):
            es.es_spmm_launch_info(a["N"], a["nnz"], a["F"], a["W"], a["mode"], ldx=a["ldx"])
    # grids beyond what a launch can carry are refused, not truncated
    with pytest.raises(es.EsSpmmError):
        es.es_spmm_launch_info(2 ** 40, 0, 4, 1, "bucket")
