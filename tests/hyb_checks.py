"""Checks of a set of hyb(c,k) arrays against what Section 4.2.1 fixes.

These do not rebuild the format: they read the arrays back (decode) and test
the properties that, together, leave exactly one valid layout:
 - dropping pads and merging the remainder gives back A's non-zeros exactly;
 - an ELL row of bucket i holds l real entries with 2^(i-1) < l <= 2^i;
 - bucket (p,i) only holds columns of partition p; rows ascend inside a bucket;
 - pads are +0.0f (bit pattern 0) and repeat the last real column;
 - remainder pieces are longer than 2^k and ordered by (partition, row).
"""
import numpy as np

ARRAY_NAMES = ("bucket_row_ptr", "bucket_slot_ptr", "ell_row", "ell_col", "ell_val",
               "rem_part_ptr", "rem_row", "rem_ptr", "rem_col", "rem_val")


def load_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = vals
    return out


def decode_and_check(h, n_rows, n_cols, indptr, indices, values):
    """Raises AssertionError on any violated property; returns stats."""
    c, k = h.c, h.k
    w = -(-n_cols // c)
    assert h.w == w
    B = c * (k + 1)
    assert h.bucket_row_ptr.shape == (B + 1,) and h.bucket_slot_ptr.shape == (B + 1,)
    assert h.bucket_row_ptr[0] == 0 and h.bucket_slot_ptr[0] == 0
    assert h.bucket_row_ptr[-1] == h.ell_row.shape[0]
    assert h.bucket_slot_ptr[-1] == h.ell_col.shape[0] == h.ell_val.shape[0]
    val_bits = h.ell_val.view(np.uint32)
    triplets = []          # (row, col, value bits)
    seen = set()           # (row, partition) pairs
    pads = 0
    for b in range(B):
        p, i = divmod(b, k + 1)
        width = 1 << i
        r0, r1 = int(h.bucket_row_ptr[b]), int(h.bucket_row_ptr[b + 1])
        s0, s1 = int(h.bucket_slot_ptr[b]), int(h.bucket_slot_ptr[b + 1])
        assert r1 >= r0 and s1 - s0 == (r1 - r0) * width
        rows = h.ell_row[r0:r1]
        assert (np.diff(rows) > 0).all(), "rows must ascend inside a bucket"
        if r1 > r0:
            assert rows.min() >= 0 and rows.max() < n_rows
        cols = h.ell_col[s0:s1].reshape(r1 - r0, width)
        bits = val_bits[s0:s1].reshape(r1 - r0, width)
        assert ((cols >= p * w) & (cols < min((p + 1) * w, n_cols))).all(), "column outside its partition"
        for q in range(r1 - r0):
            row = int(rows[q])
            assert (row, p) not in seen
            seen.add((row, p))
            l = 1
            while l < width and cols[q, l] > cols[q, l - 1]:
                l += 1
            assert (width >> 1) < l <= width or (i == 0 and l == 1), "row piece in the wrong bucket"
            assert (cols[q, l:] == cols[q, l - 1]).all(), "pad must repeat the last real column"
            assert (bits[q, l:] == 0).all(), "pad value must be +0.0f"
            pads += width - l
            for j in range(l):
                triplets.append((row, int(cols[q, j]), int(bits[q, j])))
    assert h.rem_part_ptr.shape == (c + 1,) and h.rem_part_ptr[0] == 0
    M = h.rem_row.shape[0]
    assert h.rem_part_ptr[-1] == M and h.rem_ptr.shape == (M + 1,)
    assert h.rem_ptr[0] == 0 if M >= 0 else True
    assert h.rem_ptr[-1] == h.rem_col.shape[0] == h.rem_val.shape[0]
    rem_bits = h.rem_val.view(np.uint32)
    for p in range(c):
        m0, m1 = int(h.rem_part_ptr[p]), int(h.rem_part_ptr[p + 1])
        assert (np.diff(h.rem_row[m0:m1]) > 0).all(), "remainder rows must ascend inside a partition"
        for m in range(m0, m1):
            row = int(h.rem_row[m])
            a, e = int(h.rem_ptr[m]), int(h.rem_ptr[m + 1])
            assert e - a > (1 << k), "remainder piece must be longer than 2^k"
            assert (row, p) not in seen
            seen.add((row, p))
            seg = h.rem_col[a:e]
            assert (np.diff(seg) > 0).all()
            assert seg[0] >= p * w and seg[-1] < min((p + 1) * w, n_cols)
            for j in range(a, e):
                triplets.append((row, int(h.rem_col[j]), int(rem_bits[j])))
    # reconstruction: the stored real entries are exactly A's non-zeros
    rows_of = np.repeat(np.arange(n_rows), np.diff(indptr))
    want = sorted(zip(rows_of.tolist(), np.asarray(indices).tolist(),
                      np.asarray(values, dtype=np.float32).view(np.uint32).tolist()))
    assert sorted(triplets) == want, "hyb does not reconstruct A"
    nnz = len(want)
    assert h.ell_col.shape[0] - pads + h.rem_col.shape[0] == nnz
    return dict(pads=pads, nnz=nnz, slots=int(h.ell_col.shape[0]), rem_nnz=int(h.rem_col.shape[0]))


def assert_same_hyb(got, want):
    """Bit-exact comparison of two sets of hyb arrays."""
    for name in ARRAY_NAMES:
        a, b = getattr(got, name), getattr(want, name)
        assert a.dtype == b.dtype, (name, a.dtype, b.dtype)
        assert a.shape == b.shape, (name, a.shape, b.shape)
        if a.dtype == np.float32:
            a, b = a.view(np.uint32), b.view(np.uint32)
        if not np.array_equal(a, b):
            bad = np.flatnonzero(a != b)
            raise AssertionError(f"{name}: {bad.size} mismatches, first at {bad[0]}: {a[bad[0]]} vs {b[bad[0]]}")
