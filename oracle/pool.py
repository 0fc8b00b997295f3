"""Oracle of the virtual weight tensor's page accounting (test infrastructure).

Paper Sec. 4.2: a virtual weight tensor is one contiguous virtual range of
P = M + N*E_max expert-sized slots; physical pages of fixed size back only the
slots that hold a loaded expert; a page that an expert range fills only partly is
shared with the neighbouring range and released when its last user is unloaded
(sub-page allocation with reference counting).  Sec. 3.1: adapter sparsity S_i and
memory fragmentation F_mem.
"""
from __future__ import annotations

from collections import Counter
from fractions import Fraction


def pages_of_range(slot0: int, n: int, expert_bytes: int, page_bytes: int) -> range:
    """Pages touched by slots [slot0, slot0+n): start_addr = base + slot0*expert_size (Sec. 4.2)."""
    if n <= 0:
        return range(0)
    b0 = slot0 * expert_bytes
    b1 = (slot0 + n) * expert_bytes            # exclusive
    return range(b0 // page_bytes, (b1 - 1) // page_bytes + 1)


class VirtualTensorPages:
    """Reference-counted page table of one virtual weight tensor."""

    def __init__(self, P: int, expert_bytes: int, page_bytes: int):
        self.P, self.expert_bytes, self.page_bytes = P, expert_bytes, page_bytes
        self.refs: Counter = Counter()
        self.loaded: dict[int, int] = {}        # slot0 -> n

    def load(self, slot0: int, n: int) -> list[int]:
        """Returns the pages newly mapped by this load."""
        if slot0 < 0 or n < 0 or slot0 + n > self.P:
            raise ValueError("slot range outside the virtual tensor")
        new = []
        for q in pages_of_range(slot0, n, self.expert_bytes, self.page_bytes):
            if self.refs[q] == 0:
                new.append(q)
            self.refs[q] += 1
        self.loaded[slot0] = n
        return new

    def unload(self, slot0: int) -> list[int]:
        """Returns the pages unmapped (their last user left)."""
        n = self.loaded.pop(slot0)
        freed = []
        for q in pages_of_range(slot0, n, self.expert_bytes, self.page_bytes):
            self.refs[q] -= 1
            if self.refs[q] == 0:
                del self.refs[q]
                freed.append(q)
        return freed

    def mapped_pages(self) -> list[int]:
        return sorted(self.refs)

    def mapped_bytes(self) -> int:
        return len(self.refs) * self.page_bytes

    def shared_pages(self) -> list[int]:
        return sorted(q for q, c in self.refs.items() if c > 1)


def adapter_sparsity(e_per_layer) -> Fraction:
    """S_i = sum_l (E_i - e_i^(l)) / (L * E_i),  E_i = max_l e_i^(l)   (Sec. 3.1)."""
    e = [int(v) for v in e_per_layer]
    L, E_i = len(e), max(e)
    return Fraction(sum(E_i - v for v in e), L * E_i)


def fragmentation_factor(M: int, N: int, E_max: int, e) -> Fraction:
    """F_mem = L*(M + N*E_max) / sum_l (M + sum_i e_i^(l))   (Sec. 3.1).  e[l][i], ints or Fractions."""
    L = len(e)
    used = sum(M + sum(Fraction(v) for v in row) for row in e)
    return Fraction(L * (M + N * E_max)) / used
