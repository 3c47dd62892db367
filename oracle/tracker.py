"""The paper's own next-accessed-iteration tracker, for tiny inputs.  TEST INFRASTRUCTURE.

Section 3.4, "Tracking Next Accessed Iteration": the node x iteration access matrix is kept
in a CSR-like pair (iters, ptr).  iters lists, node after node, the iterations that access
the node in ascending order; ptr[v] points at the entry that tells when v is accessed next.
The first entry of every node's run carries a mark in its top bit, and one dummy entry
holding the largest value of the datatype closes the array.  Advancing past the end of a
node's run lands on a marked entry (the next node's head, or the dummy), which is how the
tracker notices that the node is never accessed again: it then points the node at the dummy.

This exists only to check that ``oracle.next_use`` (a backward scan) and the structure the
paper describes agree; plain Python lists, O(total accesses).
"""
from __future__ import annotations

MARK = 1 << 31
DUMMY = (1 << 32) - 1
NEVER = 0x7FFFFFFF


class NextAccessTracker:
    def __init__(self, num_nodes, ids_list):
        # pass 1: appearances per node, then a running sum with a zero put in front and
        # the last element dropped gives the start of every node's run
        count = [0] * num_nodes
        for ids in ids_list:
            for v in ids:
                count[v] += 1
        running, total = [], 0
        for c in count:
            total += c
            running.append(total)
        ptr = [0] + running[:-1]
        # pass 2: write the iteration numbers, bumping ptr as a write cursor
        iters = [0] * total
        for i, ids in enumerate(ids_list):
            for v in ids:
                iters[ptr[v]] = i
                ptr[v] += 1
        # every cursor now sits where the next node's run starts: shift back by one node
        ptr = [0] + ptr[:-1]
        iters.append(DUMMY)
        for v in range(num_nodes):
            if count[v]:
                iters[ptr[v]] |= MARK
        self.iters, self.ptr, self.count = iters, ptr, count
        self.dummy_index = len(iters) - 1

    def next_access(self, v):
        """Iteration at which v is accessed next (before any advance: its first access)."""
        if self.ptr[v] == self.dummy_index:
            return NEVER
        return self.iters[self.ptr[v]] & ~MARK

    def advance(self, ids):
        """Account for one iteration that accesses ``ids`` (distinct)."""
        for v in ids:
            self.ptr[v] += 1
            if self.iters[self.ptr[v]] & MARK:
                self.ptr[v] = self.dummy_index
