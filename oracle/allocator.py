"""CPU oracle for the unified KV pool's block allocator and block tables.

TEST INFRASTRUCTURE ONLY (see oracle/attention.py).  Follows the paper's
"Unified Memory Manager": one paged pool shared by the prefill and the decode
worker, accessed through per-request block tables; an allocation is the three
steps query-utilisation / get-blocks / update-utilisation done as one atomic
operation.  Here each call IS that atomic operation (single-threaded model);
concurrent callers of the real library are compared by replaying their logged
operations in the order of the sequence numbers the library handed out.

The paper fixes no block-selection policy.  The reading pinned for both sides:

* the free list is a stack whose first pops are 0, 1, 2, ...;
* reserve(req, n_tokens) grows the request's table to ceil(n_tokens / P) blocks,
  popping one block at a time; it is all-or-nothing (too few free blocks: error,
  nothing changes); a request that already owns enough blocks is a no-op;
* free(req) pushes the request's blocks back last-to-first, so re-reserving the
  same size at once returns the same table;
* every successful mutating call gets the next operation sequence number
  (starting at 1); a failed call consumes none and changes nothing.
"""
from __future__ import annotations

from typing import Dict, List


class PoolExhausted(Exception):
    pass


class BlockAllocator:
    def __init__(self, num_pages: int, page_tokens: int):
        if num_pages <= 0 or page_tokens <= 0:
            raise ValueError("bad pool geometry")
        self.num_pages = num_pages
        self.page_tokens = page_tokens
        self.free_stack: List[int] = list(range(num_pages - 1, -1, -1))  # pop() -> 0, 1, 2, ...
        self.tables: Dict[int, List[int]] = {}
        self.used = 0            # the "memory utilisation" the paper's lock protects
        self.op_seq = 0

    # -- the atomic allocation: query, get, update in one step
    def reserve(self, req_id: int, n_tokens_total: int) -> int:
        if n_tokens_total <= 0:
            raise ValueError("n_tokens_total must be positive")
        table = self.tables.get(req_id, [])
        need = -(-n_tokens_total // self.page_tokens) - len(table)
        if need > 0:
            if self.num_pages - self.used < need:        # query
                raise PoolExhausted(f"need {need}, free {self.num_pages - self.used}")
            table = table + [self.free_stack.pop() for _ in range(need)]   # get
            self.used += need                            # update
        self.tables[req_id] = table
        self.op_seq += 1
        return self.op_seq

    def free(self, req_id: int) -> int:
        if req_id not in self.tables:
            raise KeyError(req_id)
        table = self.tables.pop(req_id)
        for b in reversed(table):
            self.free_stack.append(b)
        self.used -= len(table)
        self.op_seq += 1
        return self.op_seq

    def block_table(self, req_id: int) -> List[int]:
        return list(self.tables[req_id])

    @property
    def n_free(self) -> int:
        return len(self.free_stack)

    def state(self):
        """Hashable snapshot of everything the allocator owns."""
        return (tuple(self.free_stack), tuple(sorted((r, tuple(t)) for r, t in self.tables.items())),
                self.used, self.op_seq)

    def replay(self, ops) -> None:
        """Execute ("reserve", req, n_tokens) / ("free", req, _) tuples in the given order."""
        for op, req, n in ops:
            if op == "reserve":
                self.reserve(req, n)
            elif op == "free":
                self.free(req)
            else:
                raise ValueError(op)
