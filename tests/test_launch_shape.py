"""Host-side launch-shape logic (es_spmm_launch_info): runs without a GPU.
Checks the invariants the kernels rely on before anything is launched."""
import itertools

import pytest

import paper_2104_10716_amd as es


@pytest.fixture(autouse=True)
def _reset_overrides():
    es.es_spmm_set_rows_per_wave(0)
    es.es_spmm_set_long_row_threshold(0)
    es.es_spmm_set_lanes_per_row(0)
    yield
    es.es_spmm_set_rows_per_wave(0)
    es.es_spmm_set_long_row_threshold(0)
    es.es_spmm_set_lanes_per_row(0)


SHAPES = [(1, 0), (7, 20), (2708, 13518), (170_000, 2_370_240), (233_000, 113_134_823),
          (2_450_000, 119_569_270)]
WIDTHS = [1, 2, 3, 4, 5, 16, 17, 41, 48, 64, 100, 128, 130, 256, 512, 602, 1024, 1028, 5000]


def _check(info, N, F, backward):
    G, CH, V = info["lanes_per_row"], info["chunks_per_lane"], info["vector_width"]
    R, E = info["rows_per_wave"], info["edge_slots"]
    assert V in (1, 4) and CH in (1, 2, 4) and G in (4, 8, 16, 32, 64)
    assert R * G * E == 64 and E >= 1                     # a wave is R rows x E slots x G lanes
    assert info["loads_in_flight"] * CH == 8
    assert info["tile_slots_per_row"] * R == es.es_spmm_tile_slots(1)
    assert G * CH * V * info["grid_y"] >= F               # every column is covered ...
    assert G * CH * V * (info["grid_y"] - 1) < F          # ... by no more column blocks than needed
    rows_per_workgroup = 4 * R
    row_groups = info["grid_x"] - info["long_row_workgroups"]
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
        full = es.es_spmm_launch_info(N, nnz, F, 0, "full")
        assert full["long_row_workgroups"] > 0            # nnz is only a hint: never gated by it
        for W in (1, 16, 128, 512):
            s = es.es_spmm_launch_info(N, nnz, F, W, "fastrand")
            assert s["long_row_threshold"] >= 512 and s["long_row_workgroups"] == 0
        big = es.es_spmm_launch_info(N, nnz, F, 2304, "bucket")
        assert (big["long_row_workgroups"] > 0) == (2304 > big["long_row_threshold"])


def test_overrides_are_honoured_and_clamped():
    es.es_spmm_set_rows_per_wave(64)
    info = es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket")
    assert info["lanes_per_row"] == 16 and info["rows_per_wave"] == 4      # lowered to fit G
    es.es_spmm_set_rows_per_wave(1)
    assert es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket")["rows_per_wave"] == 1
    es.es_spmm_set_rows_per_wave(0)
    es.es_spmm_set_long_row_threshold(7)
    info = es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket")
    assert info["long_row_threshold"] == 7 and info["long_row_workgroups"] > 0
    es.es_spmm_set_long_row_threshold(0)
    assert es.es_spmm_launch_info(1000, 5000, 64, 8, "bucket")["long_row_workgroups"] == 0


def test_column_slicing_override_only_narrows():
    base = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket")
    assert base["lanes_per_row"] == 32 and base["grid_y"] == 1
    es.es_spmm_set_lanes_per_row(8)
    sliced = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket")
    assert sliced["lanes_per_row"] == 8 and sliced["chunks_per_lane"] == 1 and sliced["grid_y"] == 4
    _check(sliced, 1000, 128, False)
    wide = es.es_spmm_launch_info(1000, 9000, 16, 8, "bucket")          # already narrower than 8 lanes
    assert wide["lanes_per_row"] == 4 and wide["grid_y"] == 1
    bwd = es.es_spmm_launch_info(1000, 9000, 128, 8, "bucket", backward=True)
    assert bwd["lanes_per_row"] == 64                                   # the transposed product ignores it
    with pytest.raises(es.EsSpmmError):
        es.es_spmm_set_lanes_per_row(12)
    es.es_spmm_set_lanes_per_row(0)


def test_bad_sizes_are_rejected():
    for kw in (dict(N=0), dict(F=0), dict(W=0), dict(mode=5), dict(nnz=-1), dict(ldx=3)):
        a = dict(N=10, nnz=20, F=4, W=2, mode="bucket", ldx=None)
        a.update(kw)
        with pytest.raises(es.EsSpmmError):
            es.es_spmm_launch_info(a["N"], a["nnz"], a["F"], a["W"], a["mode"], ldx=a["ldx"])
    # grids beyond what a launch can carry are refused, not truncated
    with pytest.raises(es.EsSpmmError):
        es.es_spmm_launch_info(2 ** 40, 0, 4, 1, "bucket")
