"""Oracle: paged KV-cache page table (the serving stack the method sits on
keeps KV in fixed-size pages; Sec. 4.1 builds on such a paged cache).

TEST INFRASTRUCTURE ONLY (see package docstring).

Policy (part of the boundary's contract so tables can be compared bit for
bit): pages are numbered 0..n_pages-1; an allocation of n tokens takes the
ceil(n / page_tokens) lowest-numbered free pages in ascending order; freeing
returns a request's pages to the free set.  Token t of a request lives in page
table[t // page_tokens] at slot t % page_tokens.
"""


class PageTable:
    def __init__(self, n_pages, page_tokens=16):
        self.n_pages = n_pages
        self.page_tokens = page_tokens
        self.free = [True] * n_pages
        self.tables = {}

    def n_free(self):
        return sum(self.free)

    def alloc(self, req_id, n_tokens):
        if req_id in self.tables or n_tokens < 0:
            raise ValueError("bad alloc")
        need = -(-n_tokens // self.page_tokens)
        if need > self.n_free():
            raise MemoryError("out of pages")
        got = []
        p = 0
        while len(got) < need:
            if self.free[p]:
                self.free[p] = False
                got.append(p)
            p += 1
        self.tables[req_id] = got
        return list(got)

    def release(self, req_id):
        for p in self.tables.pop(req_id):
            self.free[p] = True

    def table(self, req_id):
        return list(self.tables[req_id])

    def slot(self, req_id, token):
        """Global slot index (page * page_tokens + slot) of a token."""
        return (self.tables[req_id][token // self.page_tokens] * self.page_tokens
                + token % self.page_tokens)
