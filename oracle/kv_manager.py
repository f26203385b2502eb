"""Block manager of the paged KV pool.  TEST INFRASTRUCTURE ONLY.

A trajectory keeps its blocks across tool calls and preemption (paper Sec. 4.2:
an evicted request's cache is kept) and gives them back when it finishes, so
the manager is only an allocator of 16-token blocks.  The discipline is a
stack: a fresh manager hands out 0, 1, 2, ...; free() pushes ids in the order
given; alloc() pops, most recently freed first.  Every call is all-or-nothing.

Blocks can have several holders: the samples of one prompt name the prompt's
blocks in their tables (Sec. 7, 16 samples per prompt; the prefix-cache hits of
Sec. 2.3).  alloc() gives a block one holder, retain() adds one, free() takes
one away, and the block returns to the stack when the last holder has freed it
(in the order of the free() call that did so).  A list names a block at most once.
"""
from __future__ import annotations

OK, E_INVAL, E_NOMEM = 0, -1, -2


class KVManager:
    def __init__(self, n_blocks: int):
        self.n_blocks = int(n_blocks)
        self.stack = list(range(self.n_blocks - 1, -1, -1))
        self.is_free = [True] * self.n_blocks
        self.holders = [0] * self.n_blocks

    def num_free(self) -> int:
        return len(self.stack)

    def alloc(self, n: int):
        """Returns (code, ids)."""
        if n < 0:
            return E_INVAL, []
        if n > len(self.stack):
            return E_NOMEM, []
        ids = [self.stack.pop() for _ in range(n)]
        for i in ids:
            self.is_free[i] = False
            self.holders[i] = 1
        return OK, ids

    def retain(self, ids) -> int:
        """One more holder for every listed block (all must be held)."""
        ids = [int(i) for i in ids]
        seen = set()
        for i in ids:
            if i < 0 or i >= self.n_blocks or self.is_free[i] or i in seen:
                return E_INVAL
            seen.add(i)
        for i in ids:
            self.holders[i] += 1
        return OK

    def free(self, ids) -> int:
        ids = [int(i) for i in ids]
        seen = set()
        for i in ids:
            if i < 0 or i >= self.n_blocks or self.is_free[i] or i in seen:
                return E_INVAL
            seen.add(i)
        for i in ids:
            self.holders[i] -= 1
            if self.holders[i] == 0:
                self.is_free[i] = True
                self.stack.append(i)
        return OK
