"""Oracle of the window bookkeeping (Sec. 4.2: sink / retrieved / recent / denoising regions of the
sliding window; Sec. 5.1: 18 latent frames = 3 + 9 + 3 + 3) -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Plain Python, written as a literal simulation: explicit lists say which generated chunk lives in
which region at every step, so the arithmetic of the library's planner can be checked against
"what must be where".  The paper fixes the four regions and their sizes; the physical placement
(ring of chunk slots, slot reuse in the retrieved region) is bookkeeping the paper leaves open and is
this build's own: parity unpinned against the authors' code, pinned by the invariants in
tests/test_oracle_window.py.
"""
from collections import deque


class RollingWindow:
    """Logical content of the window while chunks 0, 1, 2, ... are generated.

    sink_chunks chunks stay forever; the ring holds the chunk being denoised and the
    recent_chunks chunks before it; a chunk pushed out of the ring goes to the store and gets the
    next store id (ids count evictions, oldest first)."""

    def __init__(self, sink_chunks, recent_chunks):
        self.sink_chunks, self.recent_chunks = sink_chunks, recent_chunks
        self.sink, self.ring, self.store = [], deque(), []
        # physical ring: slot index -> chunk living there (None = never written)
        self.ring_slots = [None] * (recent_chunks + 1)

    def step(self, c):
        """Chunk c starts denoising.  Returns (region, slot, evicted_chunk or None)."""
        if c < self.sink_chunks:
            self.sink.append(c)
            return "sink", c, None
        evicted = None
        if len(self.ring) == self.recent_chunks + 1:
            evicted = self.ring.popleft()
            self.store.append(evicted)
        self.ring.append(c)
        # the slot of the evicted chunk is the free one; before the ring is full, the next unused one
        slot = self.ring_slots.index(evicted) if evicted is not None else self.ring_slots.index(None)
        self.ring_slots[slot] = c
        return "ring", slot, evicted


def update_slots(slot_ids, ids, R, valid):
    """In-place refresh of the retrieved region (R slots, one stored chunk each).

    slot_ids: chunk id per slot before the call (-1 = empty); ids: the chunks wanted now, in
    rank order; valid(id) says whether an id may be placed.  Wanted ids that are invalid or repeat an
    earlier one are dropped; n = number left.  Afterwards exactly slots 0..n-1 are used.  A chunk that
    is wanted and already sits in a slot stays where it is (the first such slot, should a corrupt
    table name it twice); the wanted chunks not yet resident take
    the remaining slots below n in ascending slot order, in rank order.  If a resident wanted chunk
    sits in a slot >= n the region is rebuilt (slot j <- j-th wanted chunk).
    Returns (new_slot_ids, fetched) with fetched = [(slot, id), ...] in slot order."""
    want = []
    for i in ids:
        if valid(i) and i not in want:
            want.append(i)
    want = want[:R]
    n = len(want)
    kept = {s: slot_ids[s] for s in range(R)
            if slot_ids[s] >= 0 and slot_ids[s] in want and slot_ids[s] not in slot_ids[:s]}
    new = [-1] * R
    if any(s >= n for s in kept):
        for j, i in enumerate(want):
            new[j] = i
        fetched = [(j, want[j]) for j in range(n) if slot_ids[j] != want[j]]
        return new, fetched
    for s, i in kept.items():
        new[s] = i
    resident = set(kept.values())
    incoming = [i for i in want if i not in resident]
    free = [s for s in range(n) if s not in kept]
    assert len(incoming) == len(free)
    fetched = []
    for s, i in zip(free, incoming):
        new[s] = i
        fetched.append((s, i))
    return new, fetched
