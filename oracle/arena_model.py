"""Pure-Python model of the KV-arena bookkeeping -- TEST INFRASTRUCTURE ONLY.

The paper defines two allocator counters (Section 2.2): *reserved* memory, what
has been taken from the driver, and *allocated* memory, what live tensors
occupy; fragmentation (Section 3, first paragraph; Appendix B) is their
difference at the moment the allocator has to go back to the driver.  A cache
arena that is taken from the driver once and handed out in fixed pages has
exact values for all of these, and this model states them with lists and
integers only:

* pages are popped from the head of a free list that starts as
  `initial_free_order` (identity if not given);
* a sequence id may appear once per append call;
* a sequence needs a new page exactly when its length is a multiple of the
  page size; tokens of one call are placed sequence by sequence in call order,
  token by token;
* an append that would need more pages than are free, or would push a sequence
  past `max_pages_per_seq`, fails as a whole and changes nothing;
* freeing a sequence pushes its pages to the tail of the free list in logical
  order; reset restores the initial free order and clears every length;
* reserved bytes never change after creation; allocated bytes are pages in use
  times page bytes, for K and V together.

It shares no code with the library's host bookkeeping; tests replay the same
call trace through both and compare page tables, lengths, free lists and stats
bit for bit.
"""
from __future__ import annotations

from typing import List, Optional, Sequence


class ArenaModelError(Exception):
    """kind is 'invalid' or 'oom', mirroring the library's status codes."""

    def __init__(self, kind: str, msg: str = ""):
        super().__init__(f"{kind}: {msg}")
        self.kind = kind


class ArenaModel:
    def __init__(self, max_seqs: int, n_kv_heads: int, head_dim: int, page_tokens: int,
                 n_pages: int, max_pages_per_seq: int, elem_bytes: int = 2,
                 initial_free_order: Optional[Sequence[int]] = None):
        if min(max_seqs, n_kv_heads, head_dim, page_tokens, n_pages, max_pages_per_seq) <= 0:
            raise ArenaModelError("invalid", "non-positive dimension")
        self.max_seqs = max_seqs
        self.n_kv_heads = n_kv_heads
        self.head_dim = head_dim
        self.page_tokens = page_tokens
        self.n_pages = n_pages
        self.max_pages_per_seq = max_pages_per_seq
        self.elem_bytes = elem_bytes
        if initial_free_order is None:
            order = list(range(n_pages))
        else:
            order = [int(p) for p in initial_free_order]
            if sorted(order) != list(range(n_pages)):
                raise ArenaModelError("invalid", "initial_free_order is not a permutation")
        self._initial = order
        self.reset()

    # -- state -------------------------------------------------------------
    def reset(self) -> None:
        self.free: List[int] = list(self._initial)
        self.seq_lens: List[int] = [0] * self.max_seqs
        self.pages: List[List[int]] = [[] for _ in range(self.max_seqs)]
        self.peak_pages_in_use = 0

    def page_table(self, fill: int = -1) -> List[List[int]]:
        """Dense [max_seqs][max_pages_per_seq] table; unused entries = fill."""
        return [row + [fill] * (self.max_pages_per_seq - len(row)) for row in self.pages]

    # -- operations --------------------------------------------------------
    def append(self, seq_ids: Sequence[int], n_new: Sequence[int]) -> List[tuple]:
        """Returns, for every appended token in call order, (seq, logical_pos,
        page, slot)."""
        if len(seq_ids) != len(n_new):
            raise ArenaModelError("invalid", "length mismatch")
        seen = set()
        need = 0
        P = self.page_tokens
        for s, n in zip(seq_ids, n_new):
            if not (0 <= s < self.max_seqs) or n < 0 or s in seen:
                raise ArenaModelError("invalid", "bad or repeated sequence id, or bad count")
            seen.add(s)
            cur = self.seq_lens[s]
            if (cur + n + P - 1) // P > self.max_pages_per_seq:
                raise ArenaModelError("invalid", "sequence exceeds max_pages_per_seq")
            need += (cur + n + P - 1) // P - (cur + P - 1) // P
        if need > len(self.free):
            raise ArenaModelError("oom", f"need {need} pages, {len(self.free)} free")
        placed = []
        for s, n in zip(seq_ids, n_new):
            for _ in range(n):
                pos = self.seq_lens[s]
                if pos % self.page_tokens == 0:
                    self.pages[s].append(self.free.pop(0))
                placed.append((s, pos, self.pages[s][pos // self.page_tokens],
                               pos % self.page_tokens))
                self.seq_lens[s] = pos + 1
        self.peak_pages_in_use = max(self.peak_pages_in_use, self.n_pages - len(self.free))
        return placed

    def free_seq(self, seq_id: int) -> None:
        if not (0 <= seq_id < self.max_seqs):
            raise ArenaModelError("invalid", "bad sequence id")
        self.free.extend(self.pages[seq_id])
        self.pages[seq_id] = []
        self.seq_lens[seq_id] = 0

    # -- the paper's counters ---------------------------------------------
    @property
    def page_bytes(self) -> int:
        """Bytes of one K page (a V page is the same size)."""
        return self.n_kv_heads * self.page_tokens * self.head_dim * self.elem_bytes

    def stats(self) -> dict:
        in_use = self.n_pages - len(self.free)
        token_bytes = 2 * self.n_kv_heads * self.head_dim * self.elem_bytes
        return {
            "reserved_bytes": 2 * self.n_pages * self.page_bytes,
            "allocated_bytes": 2 * in_use * self.page_bytes,
            "live_token_bytes": sum(self.seq_lens) * token_bytes,
            "pages_free": len(self.free),
            "pages_in_use": in_use,
            "peak_pages_in_use": self.peak_pages_in_use,
            "live_seqs": sum(1 for n in self.seq_lens if n > 0),
        }
