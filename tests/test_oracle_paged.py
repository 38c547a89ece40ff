"""Pin of the oracle's paged-cache gather against numpy indexing, on the two common page layouts."""
import numpy as np

from oracle import ta_oracle as ora


def test_paged_gather_equals_numpy_indexing_on_both_layouts():
    rng = np.random.default_rng(4)
    pages, ps, H, d, n = 23, 16, 3, 8, 150
    table = rng.permutation(pages)[: (n + ps - 1) // ps].astype(np.int32)
    pos = np.arange(n)
    # layout A: [pages][page_size][heads][d]
    poolA = rng.integers(0, 65536, (pages, ps, H, d)).astype(np.uint16)
    # layout B: [pages][heads][page_size][d]
    poolB = np.ascontiguousarray(poolA.transpose(0, 2, 1, 3))
    for h in range(H):
        ref = poolA[table[pos // ps], pos % ps, h]
        gotA = ora.paged_gather(poolA, table, n, ps, ps * H * d, H * d, d, h, d)
        gotB = ora.paged_gather(poolB, table, n, ps, H * ps * d, d, ps * d, h, d)
        assert np.array_equal(gotA, ref) and np.array_equal(gotB, ref)
    # a dense cache is the special case of an identity table
    dense = rng.integers(0, 65536, (4 * ps, d)).astype(np.uint16)
    got = ora.paged_gather(dense, np.arange(4, dtype=np.int32), 4 * ps - 3, ps, ps * d, d, 0, 0, d)
    assert np.array_equal(got, dense[: 4 * ps - 3])


def test_paged_scatter_equals_numpy_assignment_and_inverts_the_gather():
    """Rows written to slots 0..cnt-1 of a paged cache (compaction into the page pool; the slots of a
    generation-step cache kept in pages): numpy fancy-index assignment on both page layouts, nothing
    else in the pool changes, and gathering the slots back returns the rows."""
    rng = np.random.default_rng(9)
    pages, ps, H, d = 19, 16, 3, 8
    for cnt in (1, 16, 45, 129):
        table = rng.permutation(pages)[: (cnt + ps - 1) // ps].astype(np.int32)
        slot = np.arange(cnt)
        poolA = rng.integers(0, 65536, (pages, ps, H, d)).astype(np.uint16)
        poolB = np.ascontiguousarray(poolA.transpose(0, 2, 1, 3))
        for h in range(H):
            rows = rng.integers(0, 65536, (cnt, d)).astype(np.uint16)
            wantA = poolA.copy()
            wantA[table[slot // ps], slot % ps, h] = rows
            ora.paged_scatter(poolA, rows, table, ps, ps * H * d, H * d, d, h)
            ora.paged_scatter(poolB, rows, table, ps, H * ps * d, d, ps * d, h)
            assert np.array_equal(poolA, wantA)
            assert np.array_equal(poolB, wantA.transpose(0, 2, 1, 3))
            assert np.array_equal(ora.paged_gather(poolA, table, cnt, ps, ps * H * d, H * d, d, h, d), rows)
