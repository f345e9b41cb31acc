"""TEST INFRASTRUCTURE ONLY -- plain, slow model of the paged activation store.

Follows Sec. 3.4 ("Dynamic Activation Storage Control", "Page Allocation", "Page Table
Maintenance", "Dynamic Memory Budget") and Algorithm 3 with plain Python lists: the ordered
indices are rebuilt by a full sort on every query (what Sec. 4.3.2 "Memory Management"
calls the sorting-based approach), free space is found by scanning the sorted allocations.
Only tests/, __graft_entry__.smoke() and bench.py's CPU leg may import this module; it shares
no code with the C++ store.

Readings (the paper gives the listing and prose only):
  * An activation is described by the candidate widths it can be stored at (widest first),
    and for each of them its packed size in bytes and its time cost (integer nanoseconds).
  * Projected usage: UsedMem = sum over activations that are planned or allocated of
    pages(size at the current width) * page_bytes; UsedTime likewise.  Over budget means
    UsedMem > B_mem or UsedTime > B_time.
  * Tighter constraint = the one with the smaller remaining proportion (B - Used) / B
    (ties: memory).  An infinite time budget has remaining proportion 1.
  * The listing's SelectMax picks the activation that goes first: the one with the SMALLEST
    importance per byte (memory index) or per nanosecond (time index); ties by smaller id.
  * UpdateSize = step to the next narrower candidate width; an activation already at its
    narrowest width is evicted instead.  Evict = width 0, pages (if any) freed.
  * The reduction loop runs after the new activation has been inserted (so that it is
    counted), in both blocks of Algorithm 3.
  * Only activations that are not allocated yet can change size (their data does not exist
    yet); an allocated victim is evicted, whichever index chose it.
  * Storage is a contiguous run of pages, the lowest one that fits (first fit).  The arena
    starts empty and grows by `step_bytes` whenever nothing fits, up to floor(B_mem / page).
    If nothing fits at full size, allocated activations are evicted in memory-index order
    until a run fits; if none is left the new activation is evicted.
  * A smaller memory budget first runs the reduction loop, then shrinks the arena by whole
    steps until it is within the budget; allocations beyond the new end move to the first
    fit below it (the move is reported) or are evicted.
"""

PLANNED, ALLOCATED, EVICTED, RELEASED = 0, 1, 2, 3


class _Act:
    __slots__ = ("id", "widths", "bytes", "time", "w", "importance", "state", "offset", "pages")


class PageStoreOracle:
    def __init__(self, page_bytes, mem_budget_bytes, time_budget_ns, step_bytes):
        assert page_bytes > 0 and mem_budget_bytes > 0 and step_bytes >= page_bytes
        assert step_bytes % page_bytes == 0
        assert time_budget_ns is None or time_budget_ns > 0
        self.P = page_bytes
        self.B_mem = mem_budget_bytes
        self.B_time = time_budget_ns           # None = unlimited
        self.step_pages = step_bytes // page_bytes
        self.capacity = 0                      # pages
        self.acts = {}
        self.used_mem = 0                      # bytes (whole pages)
        self.used_time = 0                     # ns
        self.evicted_log = []                  # ids whose stored data was dropped

    # -- helpers --------------------------------------------------------------------------
    def _pages(self, a):
        return -(-a.bytes[a.w] // self.P)

    def _limit(self):
        return self.B_mem // self.P

    def _live(self):
        return [a for a in self.acts.values() if a.state in (PLANNED, ALLOCATED)]

    def _over(self):
        return self.used_mem > self.B_mem or (self.B_time is not None and self.used_time > self.B_time)

    def _tighter(self):
        r_mem = float(self.B_mem - self.used_mem) / float(self.B_mem)
        r_time = 1.0 if self.B_time is None else float(self.B_time - self.used_time) / float(self.B_time)
        return "mem" if r_mem <= r_time else "time"

    def _key(self, a, which):
        return a.importance / float(a.bytes[a.w] if which == "mem" else a.time[a.w])

    def _victim(self, which, candidates):
        order = sorted(candidates, key=lambda a: (self._key(a, which), a.id))   # full sort, every time
        return order[0] if order else None

    def _uncount(self, a):
        self.used_mem -= self._pages(a) * self.P
        self.used_time -= a.time[a.w]

    def _count(self, a):
        self.used_mem += self._pages(a) * self.P
        self.used_time += a.time[a.w]

    def _evict(self, a):
        self._uncount(a)
        if a.state == ALLOCATED:
            self.evicted_log.append(a.id)
        a.state, a.offset, a.pages = EVICTED, -1, 0

    def _reduce(self):
        while self._over():
            which = self._tighter()
            v = self._victim(which, self._live())
            if v is None:
                break
            if which == "mem" and v.state == PLANNED and v.w + 1 < len(v.widths):
                self._uncount(v)
                v.w += 1
                self._count(v)
            else:
                self._evict(v)

    def _first_fit(self, need):
        while True:
            pos = 0
            for a in sorted((a for a in self.acts.values() if a.state == ALLOCATED), key=lambda a: a.offset):
                if min(a.offset, self.capacity) - pos >= need:     # a gap ends at the arena's end
                    return pos
                pos = a.offset + a.pages
            if self.capacity - pos >= need:
                return pos
            if self.capacity >= self._limit():
                return None
            self.capacity = min(self.capacity + self.step_pages, self._limit())

    # -- Algorithm 3, first block: one activation of the pre-iteration estimation ------------
    def add(self, act_id, widths, bytes_per_width, time_per_width, moving_avg_importance):
        assert act_id not in self.acts and len(widths) >= 1
        assert len(widths) == len(bytes_per_width) == len(time_per_width)
        assert all(b > 0 for b in bytes_per_width) and all(t > 0 for t in time_per_width)
        a = _Act()
        a.id, a.widths, a.bytes, a.time = act_id, list(widths), list(bytes_per_width), list(time_per_width)
        a.w, a.importance, a.state, a.offset, a.pages = 0, float(moving_avg_importance), PLANNED, -1, 0
        self.acts[act_id] = a
        self._count(a)
        self._reduce()

    # -- Algorithm 3, second block: one activation arrives in the forward pass -----------------
    def receive(self, act_id, importance):
        """Returns (bits, offset_bytes, size_bytes); bits 0 = not stored."""
        a = self.acts[act_id]
        if a.state == EVICTED:
            return (0, -1, 0)
        assert a.state == PLANNED
        a.importance = float(importance)
        self._reduce()
        if a.state == EVICTED:
            return (0, -1, 0)
        need = self._pages(a)
        off = self._first_fit(need)
        while off is None:
            v = self._victim("mem", [b for b in self.acts.values() if b.state == ALLOCATED])
            if v is None:
                self._evict(a)
                return (0, -1, 0)
            self._evict(v)
            off = self._first_fit(need)
        a.state, a.offset, a.pages = ALLOCATED, off, need
        return (a.widths[a.w], off * self.P, a.bytes[a.w])

    def release(self, act_id):
        a = self.acts[act_id]
        assert a.state == ALLOCATED
        self._uncount(a)
        a.state, a.offset, a.pages = RELEASED, -1, 0

    def reset(self):
        """New iteration: forgets every activation; the arena keeps its size."""
        self.acts, self.used_mem, self.used_time, self.evicted_log = {}, 0, 0, []

    # -- Sec. 3.4 "Dynamic Memory Budget" ----------------------------------------------------------
    def set_mem_budget(self, mem_budget_bytes):
        """Returns the list of moves (id, from_offset_bytes, to_offset_bytes, size_bytes)."""
        assert mem_budget_bytes > 0
        self.B_mem = mem_budget_bytes
        self._reduce()
        while self.capacity > self._limit():
            self.capacity = max(self.capacity - self.step_pages, 0)
        moves = []
        beyond = sorted((a for a in self.acts.values()
                         if a.state == ALLOCATED and a.offset + a.pages > self.capacity), key=lambda a: a.offset)
        for a in beyond:
            old = a.offset
            a.state = PLANNED                      # its pages are free while a new place is sought
            off = self._first_fit(a.pages)
            if off is None:
                a.state = ALLOCATED
                self._evict(a)
            else:
                a.state, a.offset = ALLOCATED, off
                if off != old:
                    moves.append((a.id, old * self.P, off * self.P, a.bytes[a.w]))
        return moves

    def set_time_budget(self, time_budget_ns):
        assert time_budget_ns is None or time_budget_ns > 0
        self.B_time = time_budget_ns
        self._reduce()

    # -- queries ---------------------------------------------------------------------------------
    def query(self, act_id):
        """(state, bits, offset_bytes, size_bytes)"""
        a = self.acts[act_id]
        if a.state in (EVICTED, RELEASED):
            return (a.state, 0, -1, 0)
        return (a.state, a.widths[a.w], a.offset * self.P if a.state == ALLOCATED else -1, a.bytes[a.w])

    def pop_evicted(self):
        out, self.evicted_log = self.evicted_log, []
        return out

    def capacity_bytes(self):
        return self.capacity * self.P
