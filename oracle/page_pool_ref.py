"""Reference model of the KV page pool (test infrastructure only): free pages, reference counts,
fork and copy-on-write, with the rules stated at marl_page_pool_* in include/marl_decode.h (the
paper's Parallel Sampling, Section 5.1, shares a prompt's pages between its samples and leaves
the mechanism to the inference backend).  Plain Python; rows are Python lists."""
from typing import List, Optional, Tuple

PAGE = 16
OK, INVALID, NO_PAGES = 0, -1, -3


class PagePoolRef:
    def __init__(self, num_pages: int):
        self.count = [0] * num_pages
        self.free = list(range(num_pages - 1, -1, -1))   # pops 0, 1, 2, ...; released pages go on top

    def _in_use(self, page: int) -> bool:
        return 0 <= page < len(self.count) and self.count[page] > 0

    def alloc(self, n: int) -> Tuple[int, Optional[List[int]]]:
        if n > len(self.free):
            return NO_PAGES, None
        pages = [self.free.pop() for _ in range(n)]
        for p in pages:
            self.count[p] = 1
        return OK, pages

    def retain(self, pages) -> int:
        if not all(self._in_use(p) for p in pages):
            return INVALID
        for p in pages:
            self.count[p] += 1
        return OK

    def release(self, pages) -> int:
        if not all(self._in_use(p) for p in pages):
            return INVALID
        if any(list(pages).count(p) > self.count[p] for p in set(pages)):
            return INVALID
        for p in pages:
            self.count[p] -= 1
            if self.count[p] == 0:
                self.free.append(p)
        return OK

    def fork(self, parent_row, length: int) -> Tuple[int, Optional[List[int]]]:
        n = -(-length // PAGE)
        rc = self.retain(parent_row[:n])
        return (rc, list(parent_row[:n])) if rc == OK else (rc, None)

    def prepare_append(self, row: List[int], max_pages: int, length: int) -> Tuple[int, int, int]:
        """Edits `row` in place; returns (status, copy_src, copy_dst)."""
        if length < 0 or length >= max_pages * PAGE:
            return INVALID, -1, -1
        slot = length // PAGE
        if length % PAGE == 0:
            if not self.free:
                return NO_PAGES, -1, -1
            page = self.free.pop()
            self.count[page] = 1
            if slot < len(row):
                row[slot] = page
            else:
                assert slot == len(row)
                row.append(page)
            return OK, -1, -1
        old = row[slot]
        if not self._in_use(old):
            return INVALID, -1, -1
        if self.count[old] == 1:
            return OK, -1, -1
        if not self.free:
            return NO_PAGES, -1, -1
        fresh = self.free.pop()
        self.count[fresh] = 1
        self.count[old] -= 1
        row[slot] = fresh
        return OK, old, fresh

    def drop(self, row, length: int) -> int:
        return self.release(row[: -(-length // PAGE)])
