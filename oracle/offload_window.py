"""Oracle of the dynamic-offloading window.  TEST INFRASTRUCTURE ONLY.

Follows the paper's section 5.3, "Dynamic Offloading": the engine keeps a queue of free
pages; only a window of them is duplicated to CPU memory.  Three pointers walk the queue:
start (head of the free region), current (pages before it are already offloaded), end
(pages before it are scheduled for offloading).  Positions here are absolute counts of
pages that have ever entered the free region, so the pointers only move right.

Readings taken where the section leaves things open:
  - freed pages join the tail; the end pointer follows the tail until end - start reaches
    the configured window;
  - a query may take n pages only if all n lie before the current pointer; otherwise it
    stalls and takes none (the section: "the allocation must stall until the current
    pointer moves right enough to cover the required pages");
  - when pages are taken, the end pointer moves forward by their number (state 3);
  - a stalled request for more pages than the window covers pushes the end pointer to
    start + n (the section's example: one duplicated page, a query needing three, both
    pointers must advance by two more pages);
  - offloading proceeds in queue order, so the current pointer moves one page at a time.

Pinned in tests/test_oracle_offload_window.py by the section's own example and by
invariants; parity against printed values is otherwise unpinned (the figure is absent).
"""

INIT, IN_PROGRESS, STEADY = 1, 2, 4     # the section's states 1, 2 and 4; 3 is the move made by take()


class OffloadWindowOracle:
    def __init__(self, window):
        assert window >= 1
        self.window = window
        self.pages = []          # every page that ever entered the free region, in order
        self.start = 0
        self.current = 0
        self.end = 0

    @property
    def tail(self):
        return len(self.pages)

    def release(self, page):
        """The engine frees a page."""
        self.pages.append(page)
        if self.end - self.start < self.window:
            self.end = min(self.start + self.window, self.tail)

    def scheduled(self):
        """Pages waiting to be offloaded, in order."""
        return self.pages[self.current:self.end]

    def offloaded(self, n=1):
        """n more pages have reached CPU memory."""
        assert self.current + n <= self.end
        self.current += n

    def take(self, n):
        """A query asks for n free pages: the pages, or None if it must stall."""
        if n > self.tail - self.start:
            return None                      # not that many free pages at all
        if n > self.current - self.start:
            self.end = max(self.end, min(self.start + n, self.tail))
            return None
        got = self.pages[self.start:self.start + n]
        self.start += n
        self.end = min(self.end + n, self.tail)
        return got

    def state(self):
        if self.current == self.end:
            return STEADY
        return INIT if self.current == self.start else IN_PROGRESS
