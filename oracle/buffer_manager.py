"""CPU oracle for the dynamic buffer manager (EET, arXiv 2104.12470, Section 3.2).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file; it shares no code with
the library and does not import it.

What it models.  Section 3.2 keeps a list of buffers.  A developer requests a buffer of a given size
and marks it idle when it is no longer needed.  A request is served from the list under two rules:

  * within a module, an idle buffer is reused only when its size is identical to the request
    (no fragmentation);
  * across modules, an idle buffer is reused when the request is not larger than the buffer
    (no duplicated allocation);

otherwise a new buffer is created.  The sum of the sizes of all buffers ever created is the
"total buffer size" of Section 3.2.

Readings taken where the paper is silent (its decision figure is not reproduced in the text):
  * a buffer belongs to the module that used it last (the creator at first); "within" / "across" compares
    that module with the requester's;
  * the list is scanned in creation order and the first idle buffer that satisfies its rule is taken
    (first fit, not best fit);
  * memory is never returned: buffers are carved one after the other out of one arena that is sized in
    advance (Section 3.1 allocates the maximum up front), each rounded up to an alignment unit; a request
    that does not fit in what is left of the arena fails and changes nothing;
  * a request of zero bytes, and the release of something that is not a buffer in use, are errors.

Pinned by tests/test_buffer_manager.py: a hand-worked request/release scenario (tests/golden/
buffer_manager_scenario.txt, every decision derived by hand from the two rules), the total of Section 3.2,
b*p*(6h + n*p), reproduced by the request sequence of an unfused layer, invariants (live buffers never
overlap, a replayed sequence creates nothing new), and planted mistakes (first fit regardless of module,
exact match only, best fit) that the scenario must catch.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple


class BufferError(Exception):
    pass


@dataclass
class _Buffer:
    offset: int
    size: int
    module: int
    idle: bool


class BufferManagerOracle:
    def __init__(self, arena_bytes: int, align: int = 256):
        self.arena_bytes = int(arena_bytes)
        self.align = int(align)
        self.buffers: List[_Buffer] = []
        self.footprint = 0              # bytes of all buffers created so far
        self.counts = {"requests": 0, "same_size": 0, "larger": 0, "created": 0}

    def _round(self, n: int) -> int:
        return (n + self.align - 1) // self.align * self.align

    def request(self, nbytes: int, module: int) -> Tuple[int, str]:
        """-> (byte offset of the buffer in the arena, how it was obtained)."""
        if nbytes <= 0:
            raise BufferError("request of zero bytes")
        size = self._round(int(nbytes))
        for buf in self.buffers:                      # list order = creation order
            if not buf.idle:
                continue
            if buf.module == module:
                if buf.size == size:                  # within a module: identical size only
                    buf.idle = False
                    self.counts["requests"] += 1
                    self.counts["same_size"] += 1
                    return buf.offset, "same_size"
            elif size <= buf.size:                    # across modules: any idle buffer that is large enough
                how = "same_size" if size == buf.size else "larger"
                buf.idle, buf.module = False, module
                self.counts["requests"] += 1
                self.counts[how] += 1
                return buf.offset, how
        if self.footprint + size > self.arena_bytes:
            raise BufferError("arena exhausted")
        buf = _Buffer(self.footprint, size, module, False)
        self.buffers.append(buf)
        self.footprint += size
        self.counts["requests"] += 1
        self.counts["created"] += 1
        return buf.offset, "created"

    def release(self, offset: int) -> None:
        for buf in self.buffers:
            if buf.offset == offset:
                if buf.idle:
                    raise BufferError("buffer is already idle")
                buf.idle = True
                return
        raise BufferError("not a buffer of this manager")

    def live(self) -> List[Tuple[int, int]]:
        return [(b.offset, b.size) for b in self.buffers if not b.idle]
