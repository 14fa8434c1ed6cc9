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


def test_largest_configuration_takes_one_launch_per_partition():
    # a partition's 128-byte column of X is 14,561 rows x 128 B = 1.86 MB: one fits an XCD's L2, two do not
    p = sptir.sptir_launch_plan(feat=128, **SOCIAL)
    assert p == dict(row_block=64, parts_per_launch=1, n_launches=16, compact_stream=1, n_feature_tiles=4,
                     tiles_per_sweep=4, n_sweeps=1)


def test_wide_y_is_swept_in_groups_of_feature_tiles():
    # Y of 232,965 x 256 floats is 239 MB, more than the memory-side cache keeps between launches: two sweeps of
    # four tiles; 512 columns: four sweeps
    assert sptir.sptir_launch_plan(feat=256, **SOCIAL)["tiles_per_sweep"] == 4
    assert sptir.sptir_launch_plan(feat=256, **SOCIAL)["n_sweeps"] == 2
    assert sptir.sptir_launch_plan(feat=512, **SOCIAL)["n_sweeps"] == 4
    # 132,534 rows x 256 floats = 136 MB stays in one sweep, x 512 takes two of eight tiles
    protein = dict(n_rows=132534, n_cols=132534, stored_slots=56233393, n_col_parts=8)
    assert sptir.sptir_launch_plan(feat=256, **protein)["n_sweeps"] == 1
    p = sptir.sptir_launch_plan(feat=512, **protein)
    assert (p["tiles_per_sweep"], p["n_sweeps"]) == (8, 2)
    # a tile count that does not split into fours is not swept
    assert sptir.sptir_launch_plan(feat=320, **SOCIAL)["n_sweeps"] == 1


def test_few_feature_tiles_take_smaller_row_blocks():
    assert sptir.sptir_launch_plan(feat=32, **SOCIAL)["row_block"] == 32
    assert sptir.sptir_launch_plan(feat=64, **SOCIAL)["row_block"] == 64


def test_low_degree_graphs_run_as_one_launch():
    # 8 stored slots per row do not pay for a read-modify-write of Y per partition
    p = sptir.sptir_launch_plan(feat=128, **MEDIUM)
    assert (p["parts_per_launch"], p["n_launches"]) == (4, 1)
    p = sptir.sptir_launch_plan(feat=64, **TINY)
    assert (p["n_launches"], p["n_sweeps"]) == (1, 1)
    assert p["row_block"] == 8          # 2,708 rows: small blocks, or the chip does not fill


def test_many_columns_fall_back_to_wide_records():
    # more than 2^20 columns in one partition do not fit the compact record
    assert sptir.sptir_launch_plan(700, 2_500_000, 20000, 1, 4)["compact_stream"] == 0
    assert sptir.sptir_launch_plan(700, 2_500_000, 20000, 2, 4)["compact_stream"] == 0
    p = sptir.sptir_launch_plan(700, 2_500_000, 20000, 4, 4)
    assert (p["compact_stream"], p["parts_per_launch"]) == (1, 1)
    p = sptir.sptir_launch_plan(700, 2_500_000, 20000, 9, 4)
    assert p["compact_stream"] == 1 and p["parts_per_launch"] * 277_778 <= 1 << 20


def test_environment_knobs(monkeypatch):
    monkeypatch.setenv("SPTIR_ROW_BLOCK", "128")
    monkeypatch.setenv("SPTIR_PARTS_PER_PHASE", "4")
    p = sptir.sptir_launch_plan(feat=128, **SOCIAL)
    assert (p["row_block"], p["parts_per_launch"], p["n_launches"]) == (128, 4, 4)
    monkeypatch.setenv("SPTIR_ROW_BLOCK", "256")       # more rows than a compact record can address
    assert sptir.sptir_launch_plan(feat=128, **SOCIAL)["compact_stream"] == 0
    monkeypatch.delenv("SPTIR_ROW_BLOCK")
    monkeypatch.setenv("SPTIR_WIDE_STREAM", "1")
    assert sptir.sptir_launch_plan(feat=128, **SOCIAL)["compact_stream"] == 0
    monkeypatch.delenv("SPTIR_WIDE_STREAM")
    monkeypatch.delenv("SPTIR_PARTS_PER_PHASE")
    monkeypatch.setenv("SPTIR_SWEEP_MB", "1")
    assert sptir.sptir_launch_plan(feat=256, **SOCIAL)["tiles_per_sweep"] == 4


def test_invalid_arguments():
    for args in ((-1, 5, 5, 1, 4), (5, -1, 5, 1, 4), (5, 5, -1, 1, 4), (5, 5, 5, 0, 4), (5, 5, 5, 1, 0)):
        with pytest.raises(sptir.SptirError):
            sptir.sptir_launch_plan(*args)
    assert sptir.load_library().sptir_launch_plan(5, 5, 5, 1, 4, None) == 1


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
