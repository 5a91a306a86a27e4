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
    """The same rule with candidates that leave early and candidates of different lengths: the
    free list is a queue.  Appends happen token index by token index; at every index the
    candidates that still have a token to append are visited in ascending order, and one whose
    own suffix length is a multiple of the page size takes the page at the head of the queue.  A
    candidate that is dropped gives its pages back to the tail of the queue (candidates in
    ascending index, each one's pages in the order it took them).  A candidate that pauses
    keeps its pages and its length and takes no part in the appends until it resumes (back into
    the ascending order).  Written event by event so that a test can replay a call sequence."""

    def __init__(self, n_cands: int, page_tokens: int, free_list):
        self.free = list(free_list)
        self.page_tokens = page_tokens
        self.alive = list(range(n_cands))
        self.paused = []
        self.pages = {b: [] for b in range(n_cands)}
        self.lens = {b: 0 for b in range(n_cands)}

    @property
    def length(self):
        """Longest suffix among the candidates still decoding."""
        return max(self.lens[b] for b in self.alive)

    def append_each(self, counts):
        """counts[i] tokens for the i-th candidate still decoding.  Raises MemoryError, with the
        pool untouched, if the queue cannot serve the whole call."""
        counts = list(counts)
        assert len(counts) == len(self.alive)
        free, lens, taken = list(self.free), dict(self.lens), {b: [] for b in self.alive}
        for j in range(max(counts)):
            for i, b in enumerate(self.alive):
                if j >= counts[i]:
                    continue
                if lens[b] % self.page_tokens == 0:
                    if not free:
                        raise MemoryError("page pool exhausted")
                    taken[b].append(free.pop(0))
                lens[b] += 1
        self.free, self.lens = free, lens
        for b in self.alive:
            self.pages[b].extend(taken[b])

    def append(self, n_tokens: int = 1):
        """n_tokens lock-step appends, one call each (a failing one leaves the pool as the last
        successful one left it)."""
        for _ in range(n_tokens):
            self.append_each([1] * len(self.alive))

    def drop(self, ids):
        for b in sorted(ids):
            self.alive.remove(b)
            self.free.extend(self.pages[b])
            self.pages[b] = []

    def pause(self, ids):
        for b in sorted(ids):
            self.alive.remove(b)
            self.paused.append(b)

    def resume(self, ids):
        for b in sorted(ids):
            self.paused.remove(b)
            self.alive.append(b)
        self.alive.sort()

    def table(self, b: int):
        return list(self.pages[b])
