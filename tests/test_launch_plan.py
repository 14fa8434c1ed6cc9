"""Host logic of the launch plan (row blocks, partitions per launch, record form, feature sweeps), through the
C ABI's host-only query; no GPU is touched."""
import pytest

import paper_2207_04606_amd as sptir
from paper_2207_04606_amd import build as sptir_build


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if sptir_build.is_stale():
        sptir_build.build()
    sptir.load_library()


SOCIAL = dict(n_rows=232965, n_cols=232965, stored_slots=165316912, n_col_parts=16)   # the largest configuration
MEDIUM = dict(n_rows=169343, n_cols=169343, stored_slots=1389517, n_col_parts=4)
TINY = dict(n_rows=2708, n_cols=2708, stored_slots=11753, n_col_parts=1)


def test_largest_configuration_runs_in_rounds():
    # a partition's 128-byte column of X is 14,561 rows x 128 B = 1.86 MB: one fits an XCD's L2, two do not, and
    # with ~700 stored slots per row that locality is worth keeping: every list sweeps all 16 partitions in order
    # and the lists run in rounds, Y written once
    p = sptir.sptir_launch_plan(feat=128, **SOCIAL)
    assert p == dict(row_block=128, parts_per_launch=16, n_launches=1, compact_stream=1, n_feature_tiles=4,
                     tiles_per_sweep=4, n_sweeps=1, rounds=1, full_rows=0)
    # asked for explicitly, the older plan: a launch per partition, each reading back the Y of the one before
    p = sptir.sptir_launch_plan(feat=128, options={"rounds": 2}, **SOCIAL)
    assert (p["row_block"], p["parts_per_launch"], p["n_launches"], p["rounds"]) == (64, 1, 16, 0)
    # the same when the pieces that would stay in the lists are long (the caller's knowledge of the matrix, or
    # the builder's own histogram): nothing keeps the wavefronts of a round in step, and with long pieces that
    # costs more than the round trips of Y
    p = sptir.sptir_launch_plan(feat=128, options={"light_piece_len": 37}, **SOCIAL)
    assert (p["parts_per_launch"], p["n_launches"], p["rounds"]) == (1, 16, 0)
    p = sptir.sptir_launch_plan(feat=128, options={"light_piece_len": 8}, **SOCIAL)
    assert p["rounds"] == 1
    # naming the partitions per launch implies it
    p = sptir.sptir_launch_plan(feat=128, options={"parts_per_launch": 1}, **SOCIAL)
    assert (p["parts_per_launch"], p["n_launches"], p["rounds"]) == (1, 16, 0)


def test_wide_y_is_swept_in_groups_of_feature_tiles_without_rounds():
    # Y of 232,965 x 256 floats is 239 MB, more than the memory-side cache keeps between launches: two sweeps of
    # four tiles; 512 columns: four sweeps
    old = {"rounds": 2}
    assert sptir.sptir_launch_plan(feat=256, options=old, **SOCIAL)["tiles_per_sweep"] == 4
    assert sptir.sptir_launch_plan(feat=256, options=old, **SOCIAL)["n_sweeps"] == 2
    assert sptir.sptir_launch_plan(feat=512, options=old, **SOCIAL)["n_sweeps"] == 4
    # 132,534 rows x 256 floats = 136 MB stays in one sweep, x 512 takes two of eight tiles
    protein = dict(n_rows=132534, n_cols=132534, stored_slots=56233393, n_col_parts=8)
    assert sptir.sptir_launch_plan(feat=256, options=old, **protein)["n_sweeps"] == 1
    p = sptir.sptir_launch_plan(feat=512, options=old, **protein)
    assert (p["tiles_per_sweep"], p["n_sweeps"]) == (8, 2)
    # a tile count that does not split into fours is not swept
    assert sptir.sptir_launch_plan(feat=320, options=old, **SOCIAL)["n_sweeps"] == 1
    # in rounds Y never makes a round trip; there a sweep is what keeps its share of X (232,965 rows x 128 floats
    # = 119 MB) within half of the memory-side cache
    assert sptir.sptir_launch_plan(feat=128, **SOCIAL)["n_sweeps"] == 1
    p = sptir.sptir_launch_plan(feat=256, **SOCIAL)
    assert (p["rounds"], p["tiles_per_sweep"], p["n_sweeps"]) == (1, 4, 2)
    assert sptir.sptir_launch_plan(feat=512, **SOCIAL)["n_sweeps"] == 4
    small_x = dict(n_rows=60000, n_cols=60000, stored_slots=30000000, n_col_parts=16)
    p = sptir.sptir_launch_plan(feat=512, options={"rounds": 1}, **small_x)   # 60,000 x 512 floats = 123 MB
    assert (p["tiles_per_sweep"], p["n_sweeps"]) == (16, 1)
    assert sptir.sptir_launch_plan(feat=512, **protein)["rounds"] == 1      # (piece lengths unknown to the query)


def test_few_feature_tiles_take_smaller_row_blocks():
    assert sptir.sptir_launch_plan(feat=32, **SOCIAL)["row_block"] == 32
    assert sptir.sptir_launch_plan(feat=64, **SOCIAL)["row_block"] == 64


def test_low_degree_graphs_run_as_one_launch():
    # 8 stored slots per row do not pay for a read-modify-write of Y per partition
    p = sptir.sptir_launch_plan(feat=128, **MEDIUM)
    assert (p["parts_per_launch"], p["n_launches"], p["rounds"]) == (4, 1, 0)
    p = sptir.sptir_launch_plan(feat=64, **TINY)
    assert (p["n_launches"], p["n_sweeps"]) == (1, 1)
    assert p["row_block"] == 8          # 2,708 rows: small blocks, or the chip does not fill


def test_many_columns_fall_back_to_wide_records():
    # a compact record holds a column in 20 bits (heavy lists cross partitions, so it is the absolute column)
    for c in (1, 2, 4, 9):
        assert sptir.sptir_launch_plan(700, 2_500_000, 20000, c, 4)["compact_stream"] == 0
    assert sptir.sptir_launch_plan(700, 1 << 20, 20000, 2, 4)["compact_stream"] == 1
    assert sptir.sptir_launch_plan(700, (1 << 20) + 1, 20000, 2, 4)["compact_stream"] == 0


def test_build_options_steer_the_plan():
    p = sptir.sptir_launch_plan(feat=128, options={"row_block": 128, "parts_per_launch": 4}, **SOCIAL)
    assert (p["row_block"], p["parts_per_launch"], p["n_launches"], p["rounds"]) == (128, 4, 4, 0)
    # more rows than a compact record can address
    assert sptir.sptir_launch_plan(feat=128, options={"row_block": 256}, **SOCIAL)["compact_stream"] == 0
    assert sptir.sptir_launch_plan(feat=128, options={"wide_stream": 1}, **SOCIAL)["compact_stream"] == 0
    p = sptir.sptir_launch_plan(feat=256, options={"rounds": 2, "sweep_kb": 1024}, **SOCIAL)
    assert p["tiles_per_sweep"] == 4
    # rounds can be forced on a graph that would not choose them
    p = sptir.sptir_launch_plan(feat=128, options={"rounds": 1}, **MEDIUM)
    assert (p["rounds"], p["parts_per_launch"], p["n_launches"]) == (1, 4, 1)
    # the feature size hint sizes the row blocks: the query takes it from feat unless told otherwise
    assert sptir.sptir_launch_plan(feat=128, options={"feat_hint": 32}, **SOCIAL)["row_block"] == 32


def test_full_rows_are_never_chosen_but_can_be_asked_for():
    # a wavefront per 512-byte run of a row of X measured slower than 128-byte tiles bound to XCDs on every
    # workload, low-degree ones included, so no size chooses it
    for sizes in (SOCIAL, MEDIUM, TINY):
        assert sptir.sptir_launch_plan(feat=128, **sizes)["full_rows"] == 0
    p = sptir.sptir_launch_plan(feat=128, options={"full_rows": 1}, **MEDIUM)
    assert (p["full_rows"], p["row_block"], p["n_feature_tiles"]) == (1, 16, 1)     # 16 rows x 512 B of LDS
    p = sptir.sptir_launch_plan(feat=256, options={"full_rows": 1}, **MEDIUM)
    assert (p["full_rows"], p["n_feature_tiles"]) == (1, 2)
    # the 128-float tile needs feat to be a multiple of 128: otherwise the usual tiles, on the small row blocks
    p = sptir.sptir_launch_plan(feat=96, options={"full_rows": 1}, **MEDIUM)
    assert (p["full_rows"], p["row_block"], p["n_feature_tiles"]) == (1, 16, 3)
    # ... and row blocks of at most 64 rows (4 wavefronts x rows x 512 bytes of LDS): beyond that, the usual tiles
    p = sptir.sptir_launch_plan(feat=128, options={"full_rows": 1, "row_block": 64}, **MEDIUM)
    assert (p["row_block"], p["n_feature_tiles"]) == (64, 1)
    p = sptir.sptir_launch_plan(feat=128, options={"full_rows": 1, "row_block": 128}, **MEDIUM)
    assert (p["row_block"], p["n_feature_tiles"]) == (128, 4)


def test_invalid_arguments():
    for args in ((-1, 5, 5, 1, 4), (5, -1, 5, 1, 4), (5, 5, -1, 1, 4), (5, 5, 5, 0, 4), (5, 5, 5, 1, 0)):
        with pytest.raises(sptir.SptirError):
            sptir.sptir_launch_plan(*args)
    assert sptir.load_library().sptir_launch_plan(5, 5, 5, 1, 4, None, None) == 1


def test_sddmm_partition_rule():
    # one partition's rows of Yt should fit 2.5 MB: 232,965 x 512 B needs 46 partitions -> 48 (multiple of 8)
    assert sptir.sptir_sddmm_default_col_parts(232965, 232965, 114615892, 128) == 48
    assert sptir.sptir_sddmm_default_col_parts(232965, 232965, 114615892, 32) == 8     # 12 wanted: nearest is 8
    assert sptir.sptir_sddmm_default_col_parts(232965, 232965, 114615892, 256) == 88
    assert sptir.sptir_sddmm_default_col_parts(232965, 232965, 114615892, 0) == 48     # hint 0 stands for 128
    assert sptir.sptir_sddmm_default_col_parts(132534, 132534, 39756333, 32) == 8      # 7 wanted
    # 7 entries per row cannot be cut into pieces of 4: CSR order
    assert sptir.sptir_sddmm_default_col_parts(169343, 169343, 1166243, 128) == 1
    # Yt fits L2 whole
    assert sptir.sptir_sddmm_default_col_parts(2708, 2708, 10556, 64) == 1
    assert sptir.sptir_sddmm_default_col_parts(3000, 3000, 3000 * 400, 128) == 1
    assert sptir.sptir_sddmm_default_col_parts(0, 5, 0, 128) == 1
