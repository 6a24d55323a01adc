"""Pure-Python model of a caching device allocator -- TEST INFRASTRUCTURE ONLY.

The paper attributes RLHF's memory peaks to the caching allocator under the
frameworks it studies (Section 2.2, Appendix A): freed blocks stay in a pool,
requests are served from the pool when a cached block is large enough and from
the driver otherwise, and phases with different request sizes leave blocks that
later requests cannot reuse.  Its counters (Section 2.2): *reserved* = taken
from the driver, *allocated* = held by live tensors; *fragmentation*
(Section 3 first paragraph, Appendix B) = reserved - allocated sampled at the
moment the allocator goes to the driver; the overhead it reports (Section 3.1)
is the fragmentation present when reserved memory peaks.  `empty_cache()`
(Appendix A) returns every cached segment that holds no live block.

The paper does not spell out the pool policy.  This model takes the policy that
the allocator's public documentation describes, stated with lists and integers:

* a request is rounded up to a multiple of 512 bytes (at least 512);
* rounded sizes up to 1 MiB belong to the small pool, larger ones to the large
  pool; a block never changes pool;
* a request takes the smallest free block of its pool that is large enough
  (ties: the lowest segment number, then the lowest offset);
* if there is none, one segment comes from the driver: 2 MiB for the small
  pool; for the large pool 20 MiB if the rounded size is below 10 MiB, else
  the size rounded up to a multiple of 2 MiB.  Fragmentation is sampled right
  before reserved memory grows;
* the chosen block is split when the remainder is at least 512 bytes (small
  pool) or more than 1 MiB (large pool); the request gets the low part, the
  remainder stays free;
* a freed block merges with free neighbours of the same segment;
* allocated memory counts block sizes (what the request occupies after
  rounding and a remainder too small to split off).

It shares no code with the library's C++ simulator; tests replay the same
traces through both and compare every counter.
"""
from __future__ import annotations

from typing import Dict, List

KIB = 1024
MIB = 1024 * 1024
ROUND = 512
SMALL_LIMIT = MIB            # rounded sizes <= this use the small pool
SMALL_SEGMENT = 2 * MIB
LARGE_SEGMENT = 20 * MIB
LARGE_DIRECT = 10 * MIB      # rounded sizes >= this get a segment of their own size
LARGE_ROUND = 2 * MIB
SPLIT_SMALL = 512            # split when remainder >= this
SPLIT_LARGE = MIB            # split when remainder > this


class CachingAllocatorModel:
    def __init__(self):
        # a segment is a list of blocks ordered by offset: dicts offset/size/free
        self.segments: List[dict] = []
        self.live: Dict[int, tuple] = {}          # handle -> (segment index, block dict)
        self.next_handle = 1
        self.reserved = 0
        self.allocated = 0
        self.peak_reserved = 0
        self.peak_allocated = 0
        self.driver_allocations = 0
        self.driver_frees = 0
        self.last_fragmentation = 0
        self.peak_fragmentation = 0
        self.fragmentation_at_peak_reserved = 0

    @staticmethod
    def rounded(nbytes: int) -> int:
        if nbytes <= 0:
            raise ValueError("size must be positive")
        return max(ROUND, (nbytes + ROUND - 1) // ROUND * ROUND)

    def malloc(self, nbytes: int) -> int:
        size = self.rounded(nbytes)
        small = size <= SMALL_LIMIT
        best = None
        for si, seg in enumerate(self.segments):
            if seg is None or seg["small"] != small:
                continue
            for blk in seg["blocks"]:
                if blk["free"] and blk["size"] >= size:
                    if best is None or blk["size"] < best[1]["size"]:
                        best = (si, blk)
        if best is None:
            if small:
                seg_size = SMALL_SEGMENT
            elif size < LARGE_DIRECT:
                seg_size = LARGE_SEGMENT
            else:
                seg_size = (size + LARGE_ROUND - 1) // LARGE_ROUND * LARGE_ROUND
            frag = self.reserved - self.allocated
            self.last_fragmentation = frag
            self.peak_fragmentation = max(self.peak_fragmentation, frag)
            self.reserved += seg_size
            self.driver_allocations += 1
            if self.reserved > self.peak_reserved:
                self.peak_reserved = self.reserved
                self.fragmentation_at_peak_reserved = frag
            blk = {"offset": 0, "size": seg_size, "free": True}
            self.segments.append({"small": small, "size": seg_size, "blocks": [blk]})
            best = (len(self.segments) - 1, blk)
        si, blk = best
        rest = blk["size"] - size
        if (small and rest >= SPLIT_SMALL) or (not small and rest > SPLIT_LARGE):
            blocks = self.segments[si]["blocks"]
            at = blocks.index(blk)
            blocks.insert(at + 1, {"offset": blk["offset"] + size, "size": rest, "free": True})
            blk["size"] = size
        blk["free"] = False
        self.allocated += blk["size"]
        self.peak_allocated = max(self.peak_allocated, self.allocated)
        h = self.next_handle
        self.next_handle += 1
        self.live[h] = (si, blk)
        return h

    def free(self, handle: int) -> None:
        si, blk = self.live.pop(handle)          # KeyError on an unknown handle
        self.allocated -= blk["size"]
        blk["free"] = True
        blocks = self.segments[si]["blocks"]
        at = blocks.index(blk)
        if at + 1 < len(blocks) and blocks[at + 1]["free"]:
            blk["size"] += blocks[at + 1]["size"]
            del blocks[at + 1]
        if at > 0 and blocks[at - 1]["free"]:
            blocks[at - 1]["size"] += blk["size"]
            del blocks[at]

    def empty_cache(self) -> None:
        for si, seg in enumerate(self.segments):
            if seg is not None and len(seg["blocks"]) == 1 and seg["blocks"][0]["free"]:
                self.reserved -= seg["size"]
                self.driver_frees += 1
                self.segments[si] = None          # indices of other segments stay valid

    def stats(self) -> dict:
        segs = [s for s in self.segments if s is not None]
        return dict(reserved_bytes=self.reserved, allocated_bytes=self.allocated,
                    peak_reserved_bytes=self.peak_reserved, peak_allocated_bytes=self.peak_allocated,
                    driver_allocations=self.driver_allocations, driver_frees=self.driver_frees,
                    last_fragmentation_bytes=self.last_fragmentation,
                    peak_fragmentation_bytes=self.peak_fragmentation,
                    fragmentation_at_peak_reserved_bytes=self.fragmentation_at_peak_reserved,
                    n_segments=len(segs),
                    n_free_blocks=sum(1 for s in segs for b in s["blocks"] if b["free"]))
