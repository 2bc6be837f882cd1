"""Exact definition of the paged KV block allocator (TEST INFRASTRUCTURE ONLY).

Section 4.5.1 / 4.4 of the paper: blocks are allocated per request, the number of blocks a
prompt needs follows from its length alone, the ids are handed to the prefill side, and the
blocks are released when the request ends.  The discipline chosen here (the paper names
none) is a LIFO free stack: a fresh pool hands out 0,1,2,...; a released request's blocks are
pushed in reverse table order, so the next allocation receives them in the original order.
A request only ever grows; a failed allocation changes nothing.
"""
from __future__ import annotations

from typing import Dict, List


class NoBlocks(Exception):
    pass


class KVAllocator:
    def __init__(self, n_blocks: int, block: int = 16):
        self.block = block
        self.n_blocks = n_blocks
        self.free: List[int] = list(range(n_blocks - 1, -1, -1))  # pop() yields 0,1,2,...
        self.owned: Dict[int, List[int]] = {}

    def alloc(self, req_id: int, n_tokens_total: int) -> List[int]:
        need = (n_tokens_total + self.block - 1) // self.block
        have = self.owned.get(req_id, [])
        extra = need - len(have)
        if extra > len(self.free):
            raise NoBlocks()
        if extra > 0:
            have = have + [self.free.pop() for _ in range(extra)]
        self.owned[req_id] = have
        return list(have)

    def release(self, req_id: int) -> None:
        for b in reversed(self.owned.pop(req_id)):
            self.free.append(b)

    def n_free(self) -> int:
        return len(self.free)
