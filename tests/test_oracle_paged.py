"""Pins for the oracle's model of the paged layout (pages = the blocks of Sec. 4.2).

The model is pinned to hand-worked examples typed out below, to numpy indexing of
the same rows held contiguously, and to the invariants a page pool must keep.
"""
import numpy as np

import oracle as orc


def _fill(pc, seg, n, rng, scatter):
    """Give `seg` n rows on pages taken from the free stack (top first, or a random
    free page when `scatter`); returns the rows as a contiguous array."""
    k = rng.integers(0, 65536, size=(n, pc.D), dtype=np.uint16)
    v = rng.integers(0, 65536, size=(n, pc.D), dtype=np.uint16)
    for p in range((n + pc.P - 1) // pc.P):
        if scatter:
            j = int(rng.integers(0, pc.free_count))
            pc.free_stack[[j, pc.free_count - 1]] = pc.free_stack[[pc.free_count - 1, j]]
        pc.free_count -= 1
        page = int(pc.free_stack[pc.free_count])
        pc.table[seg, p] = page
        lo, hi = p * pc.P, min((p + 1) * pc.P, n)
        pc.k_pool[page, :hi - lo] = k[lo:hi]
        pc.v_pool[page, :hi - lo] = v[lo:hi]
        pc.pos_pool[page, :hi - lo] = np.arange(lo, hi)
    pc.len[seg] = n
    return k, v


def _conserved(pc):
    owned = pc.owned_pages()
    free = pc.free_stack[:pc.free_count].tolist()
    assert sorted(owned + free) == list(range(pc.num_pages))      # every page exactly once


def test_hand_worked_round():
    # P = 2, one segment of 7 rows on pages [5, 3, 8, 1] (the last holds one row), pool of 10
    pc = orc.PagedCache(nseg=1, P=2, max_pages=6, num_pages=10, D=1)
    pc.table[0, :4] = [5, 3, 8, 1]
    pc.len[0] = 7
    pc.free_stack[:6] = [9, 7, 6, 4, 2, 0]
    pc.free_count = 6
    for r in range(7):
        pc.k_pool[pc.table[0, r // 2], r % 2, 0] = 100 + r
        pc.v_pool[pc.table[0, r // 2], r % 2, 0] = 200 + r
        pc.pos_pool[pc.table[0, r // 2], r % 2] = r
    # keep logical pages 1 and 3 (rows 2, 3 and the short last page, row 6)
    pc.evict([0], [[1, 3]])
    assert pc.table[0, :4].tolist() == [3, 1, 5, 8]           # kept, then evicted, ascending
    assert pc.len[0] == 3
    assert pc.free_count == 8 and pc.free_stack[:8].tolist() == [9, 7, 6, 4, 2, 0, 5, 8]
    k, v = pc.rows(0)
    assert k[:, 0].tolist() == [102, 103, 106] and v[:, 0].tolist() == [202, 203, 206]
    assert pc.positions(0).tolist() == [2, 3, 6]
    # the next row fills the short page; the one after needs a page: the top of the stack (8)
    assert pc.append([0], np.array([[111]], np.uint16), np.array([[211]], np.uint16), [7]) == []
    assert pc.len[0] == 4 and pc.free_count == 8 and pc.table[0, :2].tolist() == [3, 1]
    assert pc.append([0], np.array([[112]], np.uint16), np.array([[212]], np.uint16), [8]) == []
    assert pc.len[0] == 5 and pc.free_count == 7 and pc.table[0, :3].tolist() == [3, 1, 8]
    assert pc.rows(0)[0][:, 0].tolist() == [102, 103, 106, 111, 112]
    assert pc.positions(0).tolist() == [2, 3, 6, 7, 8]
    # keep only the full first page: the last kept page is not the segment's last, so it counts P rows
    pc.evict([0], [[0]])
    assert pc.len[0] == 2 and pc.table[0, :3].tolist() == [3, 1, 8]
    assert pc.free_stack[:pc.free_count].tolist() == [9, 7, 6, 4, 2, 0, 5, 1, 8]


def test_logical_rows_equal_contiguous_indexing():
    rng = np.random.default_rng(40)
    P, D = 4, 3
    pc = orc.PagedCache(nseg=3, P=P, max_pages=12, num_pages=40, D=D)
    lens = [37, 16, 5]
    flat = [_fill(pc, s, lens[s], rng, scatter=True) for s in range(3)]
    _conserved(pc)
    for s in range(3):
        k, v = pc.rows(s)
        assert k.tobytes() == flat[s][0].tobytes() and v.tobytes() == flat[s][1].tobytes()
    kept = [[0, 2, 3, 7, 9], [1, 3], [1]]                       # segment 0 and 2 keep their short last page
    pc.evict([0, 1, 2], kept)
    _conserved(pc)
    for s in range(3):
        rows = np.concatenate([np.arange(b * P, min((b + 1) * P, lens[s])) for b in kept[s]])
        k, v = pc.rows(s)
        assert k.tobytes() == flat[s][0][rows].tobytes() and v.tobytes() == flat[s][1][rows].tobytes()
        assert pc.positions(s).tolist() == rows.tolist()
        # the same thing the contiguous layout's block compaction produces
        assert k.tobytes() == orc.compact_rows(flat[s][0], kept[s], block=P).tobytes()
    assert pc.len.tolist() == [4 * 4 + 1, 8, 1]


def test_release_and_grant_order():
    # two segments evict in one call: pages go on the stack segment by segment, ascending logical page;
    # three segments then ask for a page in one call: the lowest segment gets the top of the stack
    pc = orc.PagedCache(nseg=3, P=2, max_pages=4, num_pages=9, D=1)
    pc.table[0, :3] = [0, 1, 2]; pc.len[0] = 6
    pc.table[1, :3] = [3, 4, 5]; pc.len[1] = 6
    pc.table[2, :1] = [6];       pc.len[2] = 2
    pc.free_stack[:2] = [8, 7]; pc.free_count = 2
    pc.evict([0, 1], [[1], [0, 2]])
    assert pc.free_stack[:5].tolist() == [8, 7, 0, 2, 4] and pc.free_count == 5
    assert pc.len.tolist() == [2, 4, 2]
    row = np.zeros((3, 1), np.uint16)
    assert pc.append([0, 1, 2], row, row) == []
    assert [int(pc.table[0, 1]), int(pc.table[1, 2]), int(pc.table[2, 1])] == [4, 2, 0]
    assert pc.free_count == 2 and pc.free_stack[:2].tolist() == [8, 7]
    _conserved(pc)


def test_pool_exhaustion_and_capacity():
    pc = orc.PagedCache(nseg=3, P=2, max_pages=2, num_pages=3, D=1)
    row = np.ones((3, 1), np.uint16)
    assert pc.append([0, 1, 2], row, row) == []                  # three pages handed out: 0, 1, 2
    assert pc.table[:, 0].tolist() == [0, 1, 2] and pc.free_count == 0
    assert pc.append([0, 1, 2], row, row) == []                  # second row of each first page
    assert pc.append([0, 1, 2], row, row) == [0, 1, 2]           # the pool is empty: nobody grows
    assert pc.len.tolist() == [2, 2, 2] and pc.table[:, 1].tolist() == [-1, -1, -1]
    pc.evict([1], [[]])                                          # segment 1 gives its page back
    assert pc.len[1] == 0 and pc.free_count == 1
    assert pc.append([0, 2], row[:2], row[:2]) == [2]            # one page for two askers: the lower segment wins
    assert pc.len.tolist() == [3, 0, 2]
    assert pc.append([0], row[:1], row[:1]) == []
    assert pc.append([0], row[:1], row[:1]) == [0]               # at capacity (2 pages of 2 rows)
    assert pc.len[0] == 4


def test_rounds_of_evict_and_grow_keep_the_pool_consistent():
    rng = np.random.default_rng(41)
    P, D, nseg = 4, 2, 5
    pc = orc.PagedCache(nseg=nseg, P=P, max_pages=16, num_pages=60, D=D)
    mirror = []
    for s in range(nseg):
        k, v = _fill(pc, s, int(rng.integers(20, 50)), rng, scatter=True)
        mirror.append((k, v))
    for rnd in range(4):
        kept = []
        for s in range(nseg):
            N = pc.pages_in_use(s)
            kk = np.sort(rng.permutation(N)[:max(1, N // 2)]).tolist()
            kept.append(kk)
            n = mirror[s][0].shape[0]
            rows = np.concatenate([np.arange(b * P, min((b + 1) * P, n)) for b in kk])
            mirror[s] = (mirror[s][0][rows], mirror[s][1][rows])
        pc.evict(range(nseg), kept)
        _conserved(pc)
        for step in range(9):
            nk = rng.integers(0, 65536, size=(nseg, D), dtype=np.uint16)
            nv = rng.integers(0, 65536, size=(nseg, D), dtype=np.uint16)
            assert pc.append(range(nseg), nk, nv) == []
            mirror = [(np.vstack([mirror[s][0], nk[s:s + 1]]), np.vstack([mirror[s][1], nv[s:s + 1]]))
                      for s in range(nseg)]
        _conserved(pc)
        for s in range(nseg):
            k, v = pc.rows(s)
            assert k.tobytes() == mirror[s][0].tobytes() and v.tobytes() == mirror[s][1].tobytes()
