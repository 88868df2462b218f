"""Plain model of the paged cache layout (blocks of the eviction policy = pages,
Sec. 4.2: whole blocks are kept or evicted, which is what a paged cache can
do by editing a page table instead of moving rows).

TEST INFRASTRUCTURE ONLY -- see the header of ``ngc_oracle.c``.

State, all numpy:
  k_pool, v_pool  uint16 [num_pages][P][D]   bf16 bit patterns
  pos_pool        int32  [num_pages][P]
  table           int32  [nseg][max_pages]   physical page of each logical page
  len             int32  [nseg]              rows in use
  free_stack      int32  [num_pages], free_count: ids of the pages nobody owns

Definitions (one call acts on a list of segments in ascending order):
  evict   logical pages `kept` (ascending) of a segment survive: the new table is
          the old entries of the kept pages in order, then the old entries of the
          evicted pages in ascending logical order, then the rest unchanged; the
          new length is P * (K - 1) + rows of the last kept page (short only if it
          is the segment's last page).  After every segment is done, the evicted
          pages are pushed on the free stack segment by segment, ascending.
  append  every segment whose length is a multiple of P (and below capacity)
          needs a page; the r-th such segment gets free_stack[count - 1 - r]
          (none, table entry -1, if r >= count); count drops by the number of
          pages handed out.  Then every segment writes its new row at row `len`
          of its logical space and adds one to `len`; a segment at capacity or
          without a page is skipped and reported.
"""
from __future__ import annotations

import numpy as np


class PagedCache:
    def __init__(self, nseg: int, P: int, max_pages: int, num_pages: int, D: int):
        self.nseg, self.P, self.max_pages, self.num_pages, self.D = nseg, P, max_pages, num_pages, D
        self.k_pool = np.zeros((num_pages, P, D), np.uint16)
        self.v_pool = np.zeros((num_pages, P, D), np.uint16)
        self.pos_pool = np.zeros((num_pages, P), np.int32)
        self.table = np.full((nseg, max_pages), -1, np.int32)
        self.len = np.zeros(nseg, np.int32)
        self.free_stack = np.arange(num_pages - 1, -1, -1, dtype=np.int32)   # pops hand out 0, 1, 2, ...
        self.free_count = num_pages

    # ---- views -------------------------------------------------------------
    def pages_in_use(self, seg: int) -> int:
        return (int(self.len[seg]) + self.P - 1) // self.P

    def rows(self, seg: int):
        """Logical K and V rows [len][D] of a segment."""
        n = int(self.len[seg])
        k = np.zeros((n, self.D), np.uint16)
        v = np.zeros((n, self.D), np.uint16)
        for r in range(n):
            page = int(self.table[seg, r // self.P])
            k[r] = self.k_pool[page, r % self.P]
            v[r] = self.v_pool[page, r % self.P]
        return k, v

    def positions(self, seg: int) -> np.ndarray:
        n = int(self.len[seg])
        return np.array([self.pos_pool[int(self.table[seg, r // self.P]), r % self.P] for r in range(n)], np.int32)

    # ---- append ------------------------------------------------------------
    def append(self, segs, k_rows, v_rows, pos=None):
        """k_rows[i], v_rows[i] (uint16 [D]) go to segs[i]; pos[i] optional.  Returns the
        segments that were skipped."""
        segs = list(segs)
        assert segs == sorted(segs)
        cap = self.max_pages * self.P
        need = [s for s in segs if self.len[s] % self.P == 0 and self.len[s] < cap]
        count = self.free_count
        for r, s in enumerate(need):
            self.table[s, self.len[s] // self.P] = self.free_stack[count - 1 - r] if r < count else -1
        self.free_count = max(count - len(need), 0)
        skipped = []
        for i, s in enumerate(segs):
            n = int(self.len[s])
            if n >= cap:
                skipped.append(s)
                continue
            page = int(self.table[s, n // self.P])
            if page < 0:
                skipped.append(s)
                continue
            self.k_pool[page, n % self.P] = k_rows[i]
            self.v_pool[page, n % self.P] = v_rows[i]
            if pos is not None:
                self.pos_pool[page, n % self.P] = pos[i]
            self.len[s] = n + 1
        return skipped

    # ---- evict -------------------------------------------------------------
    def evict(self, segs, kept_lists):
        """kept_lists[i]: ascending logical pages of segs[i] that survive."""
        segs = list(segs)
        assert segs == sorted(segs)
        freed_all = []
        for s, kept in zip(segs, kept_lists):
            kept = [int(t) for t in kept]
            n = int(self.len[s])
            N = self.pages_in_use(s)
            assert kept == sorted(set(kept)) and all(0 <= t < N for t in kept)
            old = self.table[s].copy()
            gone = [t for t in range(N) if t not in set(kept)]
            new = [old[t] for t in kept] + [old[t] for t in gone]
            self.table[s, :N] = new
            if kept:
                last_rows = n - (N - 1) * self.P if kept[-1] == N - 1 else self.P
                self.len[s] = (len(kept) - 1) * self.P + last_rows
            else:
                self.len[s] = 0
            freed_all.append([int(old[t]) for t in gone])
        for freed in freed_all:
            for page in freed:
                self.free_stack[self.free_count] = page
                self.free_count += 1

    # ---- invariants ----------------------------------------------------------
    def owned_pages(self):
        return [int(self.table[s, i]) for s in range(self.nseg) for i in range(self.pages_in_use(s))]
