"""CPU oracle: reference page allocation for per-candidate suffix KV.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The shared prefix is one block outside the pool.  Each candidate's suffix tokens go
to fixed-size pages taken from a free list.  Rule: before a decode step appends one
token per candidate, candidates are visited in ascending index; one whose suffix
length is a multiple of the page size takes the page at the head of the free list.
"""
from __future__ import annotations

import numpy as np


def page_tables(n_cands: int, n_steps: int, page_tokens: int, free_list) -> np.ndarray:
    """Page table after n_steps lock-step decode steps: [n_cands][ceil(n_steps/page_tokens)]."""
    free = list(free_list)
    n_pages = -(-n_steps // page_tokens)
    table = -np.ones((n_cands, max(n_pages, 1)), dtype=np.int32)
    head = 0
    for t in range(n_steps):                  # suffix length before the append is t
        if t % page_tokens == 0:
            for b in range(n_cands):
                table[b, t // page_tokens] = free[head]
                head += 1
    return table[:, :n_pages] if n_pages else table[:, :0]


def slot_of(table: np.ndarray, b: int, j: int, page_tokens: int):
    """(page id, offset in page) of candidate b's j-th suffix token."""
    return int(table[b, j // page_tokens]), j % page_tokens


class PagePool:
    """The same rule with candidates that leave early: the free list is a queue.  A candidate
    that is dropped gives its pages back to the tail of the queue (candidates in ascending index,
    each one's pages in the order it took them); at a page boundary only the candidates still
    decoding are visited.  Written event by event so that a test can replay a call sequence."""

    def __init__(self, n_cands: int, page_tokens: int, free_list):
        self.free = list(free_list)
        self.page_tokens = page_tokens
        self.alive = list(range(n_cands))
        self.pages = {b: [] for b in range(n_cands)}
        self.length = 0                                  # common suffix length

    def append(self, n_tokens: int = 1):
        """n_tokens lock-step appends; raises MemoryError (state untouched by the failing append)
        if a boundary needs more pages than the queue holds."""
        for _ in range(n_tokens):
            if self.length % self.page_tokens == 0:
                if len(self.free) < len(self.alive):
                    raise MemoryError("page pool exhausted")
                for b in self.alive:
                    self.pages[b].append(self.free.pop(0))
            self.length += 1

    def drop(self, ids):
        for b in sorted(ids):
            self.alive.remove(b)
            self.free.extend(self.pages[b])
            self.pages[b] = []

    def table(self, b: int):
        return list(self.pages[b])
