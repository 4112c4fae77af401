"""CPU oracle of the paged (block-table) KV cache reindex (TEST INFRASTRUCTURE, not the product).

The reorder step of Alg. 1 / App. C asks that, after resampling, particle k's cache hold what its ancestor's held.
The plain definition is the dense row gather (`reference.gather_kv`); this module reaches the same LOGICAL content
by copying page numbers instead of cache bytes, with copy-on-write when a shared page is appended to.  It is pinned
to the dense definition in the CPU tests.  Plain numpy and Python loops, no blocking; it shares no code with the
HIP library and imports nothing from it.

Layout and rules (the HIP library follows the same rules so that tables can be compared bit for bit):
  * positions are stored in pages of P positions; row r's page for positions [j*P, (j+1)*P) is table[r, j]
    (-1 while unused).  M = ceil(S/P) columns.
  * prompt b owns the page numbers [b*Q, (b+1)*Q), Q = N*M: prompts never share pages, and Q pages always suffice
    because at most N*M distinct pages can be referenced.
  * a page is free iff its reference count is 0.  Rows that need a new page take the free pages of their prompt in
    increasing page order, the rows in increasing row order.
  * reindex: table[k, :] = old table[anc[k], :] for resampled prompts; reference counts recounted.
  * before position pos is written, every row must own table[r, pos // P] exclusively: at a page start every row
    takes a new page; otherwise, of the rows that share a page, the lowest row keeps it and each of the others takes
    a new page and receives a copy of the positions already filled (pos % P of them).
"""
import numpy as np


class PagedKV:
    def __init__(self, B, N, H, S, D, P, n_tensors, dtype=np.uint16):
        self.B, self.N, self.H, self.S, self.D, self.P = B, N, H, S, D, P
        self.R = B * N
        self.M = (S + P - 1) // P
        self.Q = N * self.M
        self.pool = [np.zeros((B * self.Q, H, P, D), dtype) for _ in range(n_tensors)]
        self.table = np.full((self.R, self.M), -1, np.int32)
        self.refcnt = np.zeros(B * self.Q, np.int32)
        self.len = 0                      # positions appended so far (the same for every row)
        self.copied_positions = 0         # statistics: positions copied by copy-on-write, summed over rows

    def reset(self, len0):
        """The state after len0 positions were appended with no resampling in between (contents left as they are)."""
        self.table[:] = -1
        self.refcnt[:] = 0
        self.len = 0
        for pos in range(len0):
            self.prepare_append(pos)

    # -- allocation -------------------------------------------------------------------------------------------
    def _free_pages(self, b):
        lo = b * self.Q
        return (lo + np.nonzero(self.refcnt[lo:lo + self.Q] == 0)[0]).tolist()

    def prepare_append(self, pos):
        """Makes table[r, pos // P] exclusively owned by every row r.  Returns (slot[R], [(src_page, dst_page)])."""
        assert pos == self.len and pos < self.S
        j, o = divmod(pos, self.P)
        copies = []
        for b in range(self.B):
            rows = range(b * self.N, (b + 1) * self.N)
            if o == 0:
                needy = list(rows)
            else:
                seen, needy = set(), []
                for r in rows:
                    p = int(self.table[r, j])
                    if p in seen:
                        needy.append(r)
                    seen.add(p)
            free = self._free_pages(b)
            assert len(free) >= len(needy)
            for r, dst in zip(needy, free):
                if o > 0:
                    src = int(self.table[r, j])
                    for ten in self.pool:
                        ten[dst, :, :o, :] = ten[src, :, :o, :]
                    copies.append((src, dst))
                    self.copied_positions += o
                self.table[r, j] = dst
            for r in rows:
                self.refcnt[self.table[r, j]] = 1
        self.len = pos + 1
        return self.table[:, j].copy(), copies

    def write(self, pos, new):
        """What the decoder does after prepare_append(pos): new[ten] is [R, H, D], stored at position pos."""
        j, o = divmod(pos, self.P)
        for ten, x in zip(self.pool, new):
            for r in range(self.R):
                ten[self.table[r, j], :, o, :] = x[r]

    # -- reorder by ancestors ---------------------------------------------------------------------------------
    def reindex(self, anc, resampled):
        ncol = (self.len + self.P - 1) // self.P
        old = self.table.copy()
        for b in range(self.B):
            if not resampled[b]:
                continue
            lo = b * self.Q
            self.refcnt[lo:lo + self.Q] = 0
            for k in range(b * self.N, (b + 1) * self.N):
                self.table[k, :ncol] = old[anc[k], :ncol]
                for j in range(ncol):
                    self.refcnt[self.table[k, j]] += 1

    # -- inspection -------------------------------------------------------------------------------------------
    def logical(self, ten):
        """Dense [R, H, len, D] view of tensor `ten` read through the table."""
        out = np.zeros((self.R, self.H, self.len, self.D), self.pool[ten].dtype)
        for r in range(self.R):
            for pos in range(self.len):
                j, o = divmod(pos, self.P)
                out[r, :, pos, :] = self.pool[ten][self.table[r, j], :, o, :]
        return out
