"""What sptir_spmm actually reads is not the canonical hyb arrays (those are compared with the oracle bit for
bit) but a stream derived from them: chunk lists per (launch, row block) and the sequence of heavy pieces.  This
test exports that stream through the C ABI, decodes it on the host from its documented record format alone
(include/sptir.h, SPTIR_PLAN_STREAM) and checks that every non-zero of A occurs in it exactly once, with its row,
column and value, that no other slot claims to hold an entry, and that the hand-over flags close every row piece.
The expected triplets come from the CSR input, not from the GPU."""
import numpy as np
import pytest

import workloads
from gpu_helpers import upload

pytestmark = pytest.mark.gpu

CHUNK = 64
QUAD = 4 * CHUNK


def ragged(seed, n_rows, n_cols, max_deg, long_rows, one_value_per_row=False):
    rng = np.random.default_rng(seed)
    deg = np.minimum(rng.geometric(0.12, n_rows), max_deg)
    deg[rng.random(n_rows) < 0.1] = 0
    for r in rng.choice(n_rows, size=long_rows, replace=False):
        deg[r] = rng.integers(max_deg // 3, max_deg + 1)
    w = workloads.random_csr(n_rows, n_cols, np.minimum(deg, n_cols), seed, 4)
    if one_value_per_row:
        w.values[:] = np.repeat(rng.standard_normal(n_rows).astype(np.float32), np.diff(w.indptr))
    return w


class Stream:
    """The exported stream, cut into chunks of 64 slots: column words, value bits (or None), row words (or None)."""

    def __init__(self, sptir, hyb, info):
        self.compact = bool(info["compact_stream"])
        self.unit = bool(info["values_per_row"])
        arrays = (2 if self.compact else 3) - (1 if self.unit else 0)
        words = sptir.sptir_hyb_array(hyb, "plan_stream")
        assert words.size == (info["n_work_items"] + info["n_heavy_items"]) * CHUNK * arrays
        quads = words.reshape(-1, arrays, QUAD)
        per_chunk = lambda a: a.reshape(-1, CHUNK)
        self.col_word = per_chunk(quads[:, 0, :])
        self.val_bits = None if self.unit else per_chunk(quads[:, 1, :])
        self.row_word = None if self.compact else per_chunk(quads[:, arrays - 1, :])

    def chunk(self, k):
        """(kind, hand_over, per-slot: real, column field, row field, hand-over flag, value bits) of chunk k;
        kind 0 is a padding chunk."""
        cw = self.col_word[k].astype(np.int64) & 0xFFFFFFFF
        vb = None if self.unit else self.val_bits[k]
        if self.compact:
            if (cw == 0xF0000000).all():
                return 0, False, None, None, None, None, None
            kind = int((cw[0] >> 28) & 7)
            assert ((cw >> 28) & 7 == kind).all(), "all slots of a chunk name its kind"
            real = ((cw >> 27) & 1).astype(bool)
            flag = ((cw >> 31) & 1).astype(bool)
            return kind, bool(flag[0]), real, cw & 0xFFFFF, (cw >> 20) & 127, flag, vb
        rw = self.row_word[k].astype(np.int64)
        if (rw == -1).all() and (cw == 0).all():
            return 0, False, None, None, None, None, None
        real = (rw >= 0) & (((rw >> 23) & 1) == 0)
        kinds = (rw[rw >= 0] >> 16) & 63
        kind = int(kinds[0])
        assert (kinds == kind).all()
        flag = (rw >= 0) & (((rw >> 22) & 1) == 1)
        hand = bool(flag[np.argmax(rw >= 0)])
        return (3 if kind == 3 else 7), hand, real, cw, np.where(rw >= 0, rw & 0xFFFF, 0), flag, vb


def decode(sptir, hyb, info, w):
    """All (row, column, value bits) triplets the stream holds, plus structural checks."""
    st = Stream(sptir, hyb, info)
    n_rb, n_launch, rb = info["n_row_blocks"], info["n_phases"], info["row_block"]
    span = info["parts_per_launch"] * info["part_width"]
    ptr = sptir.sptir_hyb_array(hyb, "plan_rb_chunk_ptr")
    order = sptir.sptir_hyb_array(hyb, "plan_rb_order")
    assert ptr[0] == 0 and ptr[-1] == info["n_work_items"] and (np.diff(ptr) >= 0).all() and (np.diff(ptr) % 4 == 0).all()
    for l in range(n_launch):      # the launch order is a permutation of the row blocks, longest list first
        o = order[l * n_rb:(l + 1) * n_rb]
        assert np.array_equal(np.sort(o), np.arange(n_rb))
        lens = np.diff(ptr[l * n_rb:(l + 1) * n_rb + 1])[o]
        assert (np.diff(lens) <= 0).all()
    row_val = sptir.sptir_hyb_array(hyb, "plan_row_val") if st.unit else None
    rows, cols, vals = [], [], []

    def emit(r, c, v):
        rows.append(r); cols.append(c); vals.append(v)

    # ---- the chunk lists
    for l in range(n_launch):
        col0 = l * span if st.compact else 0
        for b in range(n_rb):
            open_piece = {}     # queue -> row of the piece it is in the middle of
            wide_row = None     # row of the piece cut wide that is in the middle
            for k in range(int(ptr[l * n_rb + b]), int(ptr[l * n_rb + b + 1])):
                kind, hand, real, cf, rf, flag, vb = st.chunk(k)
                if kind == 0:
                    continue
                if kind == 3:
                    assert wide_row is None, "a queue chunk inside a piece cut wide"
                    for q in range(8):
                        for j in range(8):
                            s = 8 * q + j
                            if not real[s]:
                                assert not flag[s]
                                continue
                            r = b * rb + int(rf[s])
                            assert open_piece.get(q, r) == r, "a queue changed rows without a hand-over"
                            open_piece[q] = r
                            emit(r, col0 + int(cf[s]), None if vb is None else int(vb[s]))
                            if flag[s]:
                                del open_piece[q]
                else:
                    r = b * rb + int(rf[0])
                    assert real[0] and (wide_row is None or wide_row == r)
                    n_real = int(real.sum())
                    assert real[:n_real].all(), "the entries of a wide chunk come first"
                    for s in range(n_real):
                        emit(r, col0 + int(cf[s]), None if vb is None else int(vb[s]))
                    wide_row = None if hand else r
            assert not open_piece and wide_row is None, "a list ended inside a row piece"

    # ---- the heavy sequence
    if info["n_heavy_pieces"] > 0:
        first_slot = sptir.sptir_hyb_array(hyb, "plan_hlist_first_slot")
        slot_ptr = sptir.sptir_hyb_array(hyb, "plan_row_slot_ptr")
        slots = sptir.sptir_hyb_array(hyb, "plan_row_slots")
        heavy_rows = sptir.sptir_hyb_array(hyb, "plan_heavy_rows")
        n_partial = info["n_heavy_pieces"] + info["n_heavy_lists"]
        owner = np.full(n_partial, -1, dtype=np.int64)
        has = np.flatnonzero(np.diff(slot_ptr) > 0)
        assert np.array_equal(has, heavy_rows)
        for r in heavy_rows:
            mine = slots[slot_ptr[r]:slot_ptr[r + 1]]
            assert (owner[mine] == -1).all(), "a partial-sum row is added to two rows of Y"
            owner[mine] = r
        base = info["n_work_items"]
        written = np.zeros(n_partial, dtype=bool)
        for wl in range(info["n_heavy_lists"]):
            cur = int(first_slot[wl])
            per_list = info["heavy_list_items"]
            for k in range(base + per_list * wl, min(base + per_list * (wl + 1), base + info["n_heavy_items"])):
                kind, hand, real, cf, rf, flag, vb = st.chunk(k)
                if kind == 0:
                    continue
                assert kind == 7
                end = int(rf[0]) if hand else CHUNK
                for s in range(CHUNK):
                    if not real[s]:
                        continue
                    pr = cur if s <= end else cur + 1
                    assert owner[pr] >= 0, "an entry is summed into a partial-sum row that no row of Y takes"
                    emit(int(owner[pr]), int(cf[s]), None if vb is None else int(vb[s]))
                if hand:
                    written[cur] = True
                    cur += 1
            written[cur] = True          # what is left at the end of the list
        assert written[owner >= 0].all(), "a row of Y takes a partial-sum row that nothing writes"
    rows = np.array(rows, dtype=np.int64); cols = np.array(cols, dtype=np.int64)
    if st.unit:
        vals = row_val[rows].view(np.int32).astype(np.int64)
    else:
        vals = np.array(vals, dtype=np.int64)
    return rows, cols, vals


@pytest.mark.parametrize("options", [
    None, {"rounds": 1}, {"rounds": 1, "heavy_len": 64}, {"rounds": 1, "heavy_len": 20, "wide_stream": 1},
    {"rounds": 2, "parts_per_launch": 1}, {"rounds": 2, "parts_per_launch": 2, "heavy_len": 200, "wide_stream": 1},
    {"row_block": 8, "heavy_len": 100}, {"keep_values": 1, "rounds": 1}])
@pytest.mark.parametrize("one_value_per_row", [False, True])
def test_stream_holds_every_non_zero_exactly_once(gpu_lib, options, one_value_per_row):
    sptir = gpu_lib
    w = ragged(11, 900, 1100, 700, 6, one_value_per_row)
    d = upload(w)
    c, k = 3, 5
    hyb = sptir.sptir_hyb_build_ex(w.n_rows, w.n_cols, d.indptr, d.indices, d.values, c, k, options)
    info = sptir.sptir_hyb_info(hyb)
    assert info["values_per_row"] == int(one_value_per_row and not (options or {}).get("keep_values"))
    rows, cols, vals = decode(sptir, hyb, info, w)
    want_rows = np.repeat(np.arange(w.n_rows, dtype=np.int64), np.diff(w.indptr))
    want_key = want_rows * w.n_cols + w.indices
    got_key = rows * w.n_cols + cols
    assert got_key.size == want_key.size, f"{got_key.size} entries in the stream, {want_key.size} non-zeros in A"
    o = np.argsort(got_key, kind="stable")
    assert np.array_equal(got_key[o], want_key), "the stream's (row, column) pairs are not those of A"
    assert np.array_equal(vals[o], w.values.view(np.int32).astype(np.int64)), "a value differs"
    if (options or {}).get("heavy_len"):
        lens = np.diff(w.indptr)
        assert info["n_heavy_pieces"] > 0 or lens.max() <= options["heavy_len"]
