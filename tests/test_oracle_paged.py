"""Pins of the oracle's paged-layout helpers (CPU only): closed forms of the page count,
uniqueness and order of the assignment, failure cases, and that scattering a pruned cache
into pages and reading it back through the block tables is the identity."""
import numpy as np
import pytest

from oracle import kvzap_oracle as O


def test_page_count_closed_form():
    P = 16
    assert [O.pages_needed(n, P) for n in (0, 1, 15, 16, 17, 32, 33)] == [0, 1, 1, 1, 2, 2, 3]
    assert O.pages_needed(0, P, reserve_rows=1) == 1
    assert O.pages_needed(16, P, reserve_rows=16) == 2
    for n in range(0, 200):
        for P in (16, 32, 128):
            c = O.pages_needed(n, P)
            assert c * P >= n and (c == 0 or (c - 1) * P < n)


def test_assignment_is_first_fit_in_order():
    lengths = np.array([[5, 0, 40], [16, 17, 1]])
    free = [7, 3, 9, 11, 2, 30, 31, 4, 8, 100]
    table, used, ok = O.assign_pages(lengths, 16, free, max_pages=4)
    assert ok and used == 1 + 0 + 3 + 1 + 2 + 1
    flat = [int(x) for row in table for x in row if x >= 0]
    assert flat == free[:used]                      # list order, heads in (b,h) order
    assert len(set(flat)) == len(flat)
    assert [int((row >= 0).sum()) for row in table] == [1, 0, 3, 1, 2, 1]
    assert (table[1] == -1).all()                   # an empty head owns nothing


def test_assignment_fails_atomically():
    lengths = np.array([[20, 20]])
    t, used, ok = O.assign_pages(lengths, 16, [1, 2, 3], max_pages=4)      # needs 4 pages
    assert not ok and used == 0 and (t == -1).all()
    t, used, ok = O.assign_pages(lengths, 16, list(range(10)), max_pages=1)  # 2 per head
    assert not ok and used == 0 and (t == -1).all()


@pytest.mark.parametrize("P", [16, 32, 64])
def test_paged_round_trip_of_a_pruned_cache(P):
    rng = np.random.default_rng(P)
    B, H, T, D, w = 2, 3, 150, 8, 10
    S = rng.standard_normal((B, H, T))
    K = rng.integers(0, 65536, (B, H, T, D)).astype(np.uint16)
    res = O.prune(S, 0.3, w, K, K)
    rows = [res.K_out[res.offsets[i]:res.offsets[i + 1]] for i in range(B * H)]
    n_pages = sum(O.pages_needed(r.shape[0], P) for r in rows)
    free = list(rng.permutation(n_pages + 5))
    table, used, ok = O.assign_pages(res.lengths, P, free, max_pages=T // P + 1)
    assert ok and used == n_pages
    pool = O.scatter_to_pages(rows, table, P, n_pages + 5, D)
    for i, r in enumerate(rows):
        back = O.gather_from_pages(pool, table[i], r.shape[0], P)
        assert np.array_equal(back, r)
        # position by position, from the definition: row j lives at (table[j // P], j % P)
        for j in (0, r.shape[0] // 2, r.shape[0] - 1):
            assert np.array_equal(pool[table[i, j // P], j % P], r[j])
    # pages not assigned stay untouched
    untouched = sorted(set(range(n_pages + 5)) - {int(x) for x in table.reshape(-1) if x >= 0})
    assert (pool[untouched] == 0).all()


def test_extend_is_assign_when_nothing_is_owned():
    rng = np.random.default_rng(5)
    lengths = rng.integers(0, 300, (3, 4))
    free = list(rng.permutation(200))
    t0 = np.full((12, 24), -1, np.int32)
    t, counts, used, ok = O.extend_pages(lengths, np.zeros(12, np.int32), t0, 16, free)
    ta, useda, oka = O.assign_pages(lengths, 16, free, 24)
    assert ok and oka and used == useda
    assert np.array_equal(t, ta)
    assert counts.tolist() == [O.pages_needed(int(x), 16) for x in lengths.reshape(-1)]


def test_extend_appends_only_what_is_missing():
    lengths = np.array([[16, 17, 40]])
    counts = np.array([1, 1, 5], np.int32)                  # the last head owns more than it needs
    table = np.array([[7, -1, -1, -1, -1, -1], [8, -1, -1, -1, -1, -1], [1, 2, 3, 4, 5, -1]], np.int32)
    t, c, used, ok = O.extend_pages(lengths, counts, table, 16, [50, 51, 52], reserve_rows=1)
    # 16+1 -> 2 pages, 17+1 -> 2 pages, 40+1 -> 3 pages (already 5)
    assert ok and used == 2 and c.tolist() == [2, 2, 5]
    assert t.tolist() == [[7, 50, -1, -1, -1, -1], [8, 51, -1, -1, -1, -1], [1, 2, 3, 4, 5, -1]]
    # growing token by token with reserve 1 never leaves a head without room for the next row
    counts = np.zeros(1, np.int32); table = np.full((1, 10), -1, np.int32); free = list(range(100, 110))
    used_total = 0
    for n in range(0, 100):
        table, counts, used, ok = O.extend_pages(np.array([[n]]), counts, table, 16, free[used_total:], 1)
        assert ok
        used_total += used
        assert counts[0] * 16 >= n + 1
    assert used_total == 7 and table[0, :7].tolist() == free[:7]


def test_extend_fails_atomically():
    table = np.array([[3, -1]], np.int32)
    t, c, used, ok = O.extend_pages(np.array([[40]]), np.array([1], np.int32), table, 16, [9, 10])
    assert not ok and used == 0 and np.array_equal(t, table) and c.tolist() == [1]   # needs 3 > width 2
    t, c, used, ok = O.extend_pages(np.array([[30]]), np.array([1], np.int32), table, 16, [])
    assert not ok and np.array_equal(t, table)
