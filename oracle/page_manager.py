"""Model of the paged KV-manager's bookkeeping -- TEST INFRASTRUCTURE ONLY.

Plain Python sets and lists, written from Algorithm 1 (Reserve: a sequence of length len owns
n = ceil(len / P) blocks, missing ones are popped from the free list) and Sec. III-B (pages are
returned as soon as a sequence ends; sequences with the same prefix may map the same pages).
Which free page a reservation receives is not fixed by the paper, so the model hands out abstract
page tokens of its own; tests compare what IS fixed -- block counts, the number of free pages,
reference counts and which (sequence, block) pairs share a page -- and check the rest for validity.
The GPU library shares no code with this file.
"""
from __future__ import annotations


class OutOfPages(Exception):
    pass


class PageManagerModel:
    def __init__(self, num_pages: int, page_size: int, max_seqs: int, max_blocks: int, pow2_growth: bool = False):
        assert page_size > 0 and page_size & (page_size - 1) == 0
        self.num_pages = num_pages
        self.page_size = page_size
        self.max_blocks = max_blocks
        self.pow2_growth = pow2_growth                      # Sec. IV "Memory Utilization": power-of-two allocations
        self.free = set(range(num_pages))
        self.rows = [[] for _ in range(max_seqs)]          # rows[s][b] = page token

    # Algorithm 1, Reserve
    def reserve(self, seq: int, length: int) -> None:
        n = -(-length // self.page_size)                    # ceil(len / P)
        if n > self.max_blocks:
            raise ValueError("more blocks than the table holds")
        have = len(self.rows[seq])
        if n <= have:
            return
        if n - have > len(self.free):
            raise OutOfPages()
        want = n
        if self.pow2_growth:                                # capacity = next power of two, as far as pages last
            want = 1
            while want < n:
                want *= 2
            want = min(want, self.max_blocks, have + len(self.free))
        for _ in range(want - have):
            self.rows[seq].append(self.free.pop())

    def refcount(self, page: int) -> int:
        return sum(row.count(page) for row in self.rows)

    # Sec. III-B: a finished sequence gives its pages back at once; a shared page stays while referenced
    def release(self, seq: int) -> None:
        row, self.rows[seq] = self.rows[seq], []
        for page in row:
            if self.refcount(page) == 0:
                self.free.add(page)

    # Sec. III-B / Sec. I-A: identical prefixes map the same physical pages (whole pages only)
    def share_prefix(self, dst: int, src: int, prefix_tokens: int) -> None:
        nb = prefix_tokens // self.page_size
        if dst == src or self.rows[dst] or nb > len(self.rows[src]):
            raise ValueError("bad share")
        self.rows[dst] = list(self.rows[src][:nb])

    # a write into a shared page first gives the writer a private copy
    def make_writable(self, seq: int, position: int) -> bool:
        b = position // self.page_size
        page = self.rows[seq][b]
        if self.refcount(page) <= 1:
            return False
        if not self.free:
            raise OutOfPages()
        self.rows[seq][b] = self.free.pop()
        return True

    def num_free(self) -> int:
        return len(self.free)

    def num_blocks(self, seq: int) -> int:
        return len(self.rows[seq])

    def sharing(self):
        """Partition of the mapped (seq, block) pairs by page: a sorted list of sorted groups."""
        groups = {}
        for s, row in enumerate(self.rows):
            for b, page in enumerate(row):
                groups.setdefault(page, []).append((s, b))
        return sorted(sorted(g) for g in groups.values())
