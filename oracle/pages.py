"""Oracle page-allocator model (test infrastructure).

The paper appends observation tokens to a trajectory's context (Section 2.3.2,
Update step) but says nothing about storage.  The rule modelled here makes page
indices a pure function of the call sequence: a trajectory with n tokens holds
ceil(n / page_tokens) pages; a new page is always the lowest-numbered free page;
pages may be shared (fork) and return to the free set when their last holder lets go.
"""


class PageAllocator:
    def __init__(self, n_pages: int):
        self.n_pages = n_pages
        self.refcount = [0] * n_pages
        self._lo = 0          # every page below _lo is in use (scan shortcut only)

    def n_free(self) -> int:
        return sum(1 for c in self.refcount if c == 0)

    def take_lowest(self) -> int:
        for i in range(self._lo, self.n_pages):     # deliberately a linear scan
            if self.refcount[i] == 0:
                self.refcount[i] = 1
                self._lo = i + 1
                return i
        raise RuntimeError("no free page")

    def share(self, page: int):
        assert self.refcount[page] > 0
        self.refcount[page] += 1

    def drop(self, page: int):
        assert self.refcount[page] > 0
        self.refcount[page] -= 1
        if self.refcount[page] == 0:
            self._lo = min(self._lo, page)
