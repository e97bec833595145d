"""Plain model of the KV page manager's bookkeeping (paper Sec. III-C, "Memory management": one page pool
shared by the prefill and the decode side under a mutex; what a finished prefill wrote is marked read-only so
decode can use it at once; events order the two sides so that decode never reads partly written KV, and - the
same rule seen from the other side - a page is not written for a new owner while an old reader may still read
it).  TEST INFRASTRUCTURE ONLY: the library's manager (C++) shares no code with this file, and only tests may
import it.

The paper names the mechanisms but no interface; the operations below are this build's reading of them:
  open / close            a session's lifetime; close returns its pages
  reserve(s, n)           room for n more tokens after those reserved so far, in whole pages, ALL OR NOTHING:
                          if the free pages or the session's row (max_pages) cannot cover it nothing changes
  seal(s)                 everything reserved so far becomes read-only ("sealed"); positions below the sealed
                          length are never handed out again, and a page is sealed once all its slots are
  commit(s, stream)       seal + remember that the writer's work on `stream` must finish first
  acquire(s, stream)      a reader on `stream`: must it wait for the writer? (not if same stream / finished)
  release(s, stream)      the reader's work on `stream` up to now uses the session's pages
  close(s)                returns what must be waited for (writer's commit, every released reader) BEFORE the
                          pages go back
WHICH free page a reservation gets is left open (any choice is correct); the model takes the smallest numbers,
and tests compare with the library only what does not depend on the choice.

Pins (tests/test_pager_model_pins.py): a sequence worked by hand; conservation and disjoint ownership after
every step of random walks; all-or-nothing on both limits; monotone starts (a start never lies below the sealed
length); page states by position; the wait sets of close in each ordering of commit / acquire / release /
finish; planted mistakes in a copy of this file, each caught.  The paper gives no trace of its manager: parity
with the authors' implementation is unpinned.
"""
from __future__ import annotations

FREE, WRITABLE, SEALED = 0, 1, 2


class NoSpace(Exception):
    pass


class Session:
    def __init__(self):
        self.reserved = 0          # tokens handed out
        self.sealed = 0            # tokens read-only
        self.pages = []            # physical pages in logical order
        self.writer = None         # (stream, ticket) of the last commit, while it may still be running
        self.readers = {}          # stream -> ticket of the last release on that stream, while it may still be running


class PagerModel:
    def __init__(self, num_pages: int, page_size: int, max_sessions: int, max_pages: int):
        if min(num_pages, page_size, max_sessions, max_pages) <= 0:
            raise ValueError("all sizes must be positive")
        self.P, self.ps, self.S, self.row = num_pages, page_size, max_sessions, max_pages
        self.free = set(range(num_pages))
        self.sessions = {}
        self.issued = {}           # stream -> tickets issued on it (work enqueued)
        self.done = {}             # stream -> tickets finished

    # ---- streams: work is a counter per stream; `finish` lets everything enqueued so far complete ----
    def _ticket(self, stream):
        self.issued[stream] = self.issued.get(stream, 0) + 1
        return self.issued[stream]

    def finish(self, stream):
        self.done[stream] = self.issued.get(stream, 0)

    def _running(self, stream, ticket):
        return self.done.get(stream, 0) < ticket

    # ---- sessions ----
    def open(self) -> int:
        for s in range(self.S):
            if s not in self.sessions:
                self.sessions[s] = Session()
                return s
        raise NoSpace("all sessions are open")

    def reserve(self, s: int, n: int) -> int:
        x = self.sessions[s]
        if n < 0:
            raise ValueError("negative token count")
        want_pages = -(-(x.reserved + n) // self.ps)
        more = want_pages - len(x.pages)
        if want_pages > self.row or more > len(self.free):
            raise NoSpace("not enough free pages or row capacity")      # nothing was changed
        for _ in range(more):
            pg = min(self.free)
            self.free.remove(pg)
            x.pages.append(pg)
        start = x.reserved
        x.reserved += n
        return start

    def seal(self, s: int) -> None:
        x = self.sessions[s]
        x.sealed = x.reserved

    def commit(self, s: int, stream) -> None:
        x = self.sessions[s]
        x.writer = (stream, self._ticket(stream))
        x.sealed = x.reserved

    def acquire(self, s: int, stream):
        """Returns (sealed length, whether the reader's stream has to wait for the writer)."""
        x = self.sessions[s]
        wait = False
        if x.writer is not None:
            wstream, ticket = x.writer
            if not self._running(wstream, ticket):
                x.writer = None
            elif wstream != stream:
                wait = True
        return x.sealed, wait

    def release(self, s: int, stream) -> None:
        self.sessions[s].readers[stream] = self._ticket(stream)

    def close(self, s: int):
        """Returns the set of (stream, ticket) that had to finish before the pages were returned."""
        x = self.sessions.pop(s)
        waits = set()
        if x.writer is not None:
            waits.add(x.writer)
        for stream, ticket in x.readers.items():
            waits.add((stream, ticket))
        for stream, ticket in waits:                    # waiting lets that work finish
            self.done[stream] = max(self.done.get(stream, 0), ticket)
        self.free.update(x.pages)
        return waits

    # ---- views ----
    def lengths(self, s: int):
        x = self.sessions[s]
        return {"reserved": x.reserved, "sealed": x.sealed, "pages": len(x.pages)}

    def page_state(self, page: int) -> int:
        for x in self.sessions.values():
            if page in x.pages:
                i = x.pages.index(page)
                return SEALED if (i + 1) * self.ps <= x.sealed else WRITABLE
        return FREE

    def owned(self):
        return {pg: s for s, x in self.sessions.items() for pg in x.pages}
