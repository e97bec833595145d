"""Pins for oracle/pager_model.py, the plain model of the page manager's bookkeeping (paper Sec. III-C, memory
management), and the library's manager against it.  The model is pinned by a sequence worked by hand, by
properties that must hold after every step whatever pages are chosen, and by planted mistakes."""
import importlib.util
import os
import random

import pytest

from oracle import pager_model as M
from paper_2603_10342_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))


def check_invariants(m):
    owned = {}
    for s, x in m.sessions.items():
        assert 0 <= x.sealed <= x.reserved <= len(x.pages) * m.ps               # sealed below reserved below capacity
        assert len(x.pages) == -(-x.reserved // m.ps) or (x.reserved == 0 and not x.pages) or len(x.pages) * m.ps - x.reserved < m.ps
        assert len(x.pages) <= m.row
        for pg in x.pages:
            assert pg not in owned and pg not in m.free                           # one owner, never also free
            owned[pg] = s
    assert len(owned) + len(m.free) == m.P                                        # conservation


def test_sequence_worked_by_hand():
    # pool of 6 pages of 4 tokens, rows of 4 pages, 2 sessions.  Worked on paper from the operations' definitions.
    m = M.PagerModel(6, 4, 2, 4)
    a = m.open()
    assert m.reserve(a, 5) == 0 and m.lengths(a) == {"reserved": 5, "sealed": 0, "pages": 2}      # ceil(5/4) = 2
    m.seal(a)                                               # 5 tokens: page 0 is full, page 1 has 3 open slots
    assert [m.page_state(p) for p in m.sessions[a].pages] == [M.SEALED, M.WRITABLE]
    assert m.reserve(a, 3) == 5 and m.lengths(a)["pages"] == 2                                      # 8 tokens fill 2 pages
    m.commit(a, "pre")
    assert m.lengths(a)["sealed"] == 8 and [m.page_state(p) for p in m.sessions[a].pages] == [M.SEALED, M.SEALED]
    assert m.acquire(a, "dec") == (8, True)                 # other stream, writer still running: wait
    assert m.acquire(a, "pre") == (8, False)                # the writer's own stream is ordered already
    b = m.open()
    with pytest.raises(M.NoSpace):
        m.reserve(b, 17)                                    # 5 pages wanted: a row holds 4 (and only 4 are free)
    assert m.lengths(b) == {"reserved": 0, "sealed": 0, "pages": 0} and len(m.free) == 4
    assert m.reserve(b, 16) == 0 and not m.free             # exactly a row, and the last free pages
    with pytest.raises(M.NoSpace):
        m.reserve(a, 1)                                     # a third page for a: its row has room, the pool has none
    assert m.lengths(a) == {"reserved": 8, "sealed": 8, "pages": 2}
    with pytest.raises(M.NoSpace):
        m.open()                                            # both sessions are open
    assert m.close(b) == set() and len(m.free) == 4
    assert m.reserve(a, 1) == 8                             # decode's next token starts at the sealed length
    assert [m.page_state(p) for p in m.sessions[a].pages] == [M.SEALED, M.SEALED, M.WRITABLE] and len(m.free) == 3
    m.release(a, "dec")
    m.finish("pre")                                         # the prefill's kernels are done
    assert m.acquire(a, "dec") == (8, False)                # nothing left to wait for
    held = list(m.sessions[a].pages)
    assert m.close(a) == {("dec", 1)}                       # only the released reader is still in flight
    assert len(m.free) == 6 and all(m.page_state(p) == M.FREE for p in held)


def test_close_waits_for_exactly_what_may_still_touch_the_pages():
    m = M.PagerModel(8, 4, 2, 4)
    s = m.open()
    m.reserve(s, 6)
    m.commit(s, "w")
    m.acquire(s, "r1"); m.release(s, "r1")
    m.acquire(s, "r2"); m.release(s, "r2")
    m.release(s, "r1")                                      # a later launch on r1: its newest ticket counts
    assert m.close(s) == {("w", 1), ("r1", 2), ("r2", 1)}
    s = m.open()
    m.reserve(s, 6)
    m.commit(s, "w")
    m.finish("w")
    assert m.acquire(s, "r1") == (6, False)
    assert m.close(s) == set()                              # an unreleased reader is invisible; the writer is done


def test_random_walks_keep_the_invariants_and_reserve_is_all_or_nothing():
    for seed in range(5):
        rnd = random.Random(seed)
        m = M.PagerModel(60, 8, 6, 12)
        for _ in range(1500):
            op = rnd.random()
            if op < 0.12 and len(m.sessions) < m.S:
                m.open()
            elif op < 0.2 and m.sessions:
                m.close(rnd.choice(list(m.sessions)))
            elif op < 0.75 and m.sessions:
                s = rnd.choice(list(m.sessions))
                x = m.sessions[s]
                before = (x.reserved, x.sealed, list(x.pages), set(m.free))
                n = rnd.choice([0, 1, 3, 8, 9, 40])
                try:
                    start = m.reserve(s, n)
                    assert start == before[0] >= x.sealed and x.pages[:len(before[2])] == before[2]
                except M.NoSpace:
                    assert (x.reserved, x.sealed, x.pages, m.free) == before
                    need = -(-(before[0] + n) // m.ps)
                    assert need > m.row or need - len(before[2]) > len(before[3])   # refused only for a reason
            elif m.sessions:
                s = rnd.choice(list(m.sessions))
                (m.seal if rnd.random() < 0.5 else (lambda q: m.commit(q, rnd.choice("ab"))))(s)
            check_invariants(m)


MUTANTS = [
    ("want_pages = -(-(x.reserved + n) // self.ps)", "want_pages = (x.reserved + n) // self.ps", "floor instead of ceiling"),
    ("if want_pages > self.row or more > len(self.free):", "if more > len(self.free):", "row capacity ignored"),
    ("if want_pages > self.row or more > len(self.free):", "if want_pages > self.row:", "takes pages that are not free"),
    ("        start = x.reserved\n", "        start = x.sealed\n", "start below what was handed out"),
    ("        self.free.update(x.pages)\n", "", "close loses the pages"),
    ("return SEALED if (i + 1) * self.ps <= x.sealed else WRITABLE", "return SEALED if i * self.ps < x.sealed else WRITABLE", "partly sealed page called sealed"),
    ("            elif wstream != stream:\n                wait = True", "            else:\n                wait = True", "waits on its own stream"),
    ("        for stream, ticket in x.readers.items():\n            waits.add((stream, ticket))\n", "", "close forgets the readers"),
    ("        x.writer = (stream, self._ticket(stream))\n        x.sealed = x.reserved", "        x.writer = (stream, self._ticket(stream))", "commit does not seal"),
]


@pytest.mark.parametrize("old,new,what", MUTANTS)
def test_planted_mistakes_are_caught(old, new, what, tmp_path):
    src = open(os.path.join(os.path.dirname(HERE), "oracle", "pager_model.py")).read()
    assert src.count(old) == 1, what
    path = tmp_path / "mutant.py"
    path.write_text(src.replace(old, new))
    spec = importlib.util.spec_from_file_location("mutant", path)
    mut = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mut)
    global M
    keep = M
    M = mut
    try:
        with pytest.raises((AssertionError, KeyError, ValueError)):
            test_sequence_worked_by_hand()
            test_close_waits_for_exactly_what_may_still_touch_the_pages()
            test_random_walks_keep_the_invariants_and_reserve_is_all_or_nothing()
    finally:
        M = keep


def test_library_manager_equals_the_model_on_a_random_walk():
    """Everything that does not depend on WHICH page is chosen: results of every call (starts, refusals, sealed
    lengths), lengths, page counts, page states by logical position, conservation."""
    rnd = random.Random(10342)
    P, ps, S, row = 200, 16, 12, 24
    p, m = B.Pager(P, ps, S, row), M.PagerModel(P, ps, S, row)
    ids = {}                                            # library session id -> model session id
    for step in range(3000):
        op = rnd.random()
        if op < 0.15 and len(ids) < S:
            ids[p.open()] = m.open()
        elif op < 0.25 and ids:
            s = rnd.choice(list(ids))
            p.close(s)
            m.close(ids.pop(s))
        elif op < 0.8 and ids:
            s = rnd.choice(list(ids))
            n = rnd.choice([0, 1, 1, 5, 16, 17, 100])
            try:
                want = m.reserve(ids[s], n)
            except M.NoSpace:
                with pytest.raises(B.AgError) as e:
                    p.reserve(s, n)
                assert e.value.status == B.AG_ERR_NO_SPACE
            else:
                assert p.reserve(s, n) == want
        elif ids:
            s = rnd.choice(list(ids))
            p.seal(s)
            m.seal(ids[s])
        if step % 53 == 0 or step == 2999:
            seen = set()
            for s, ms in ids.items():
                assert p.lengths(s) == m.lengths(ms)
                n = p.lengths(s)["pages"]
                row_pages = [int(x) for x in p.export([s])[0][:n]]
                assert not (seen & set(row_pages)) and len(set(row_pages)) == n
                seen |= set(row_pages)
                x = m.sessions[ms]
                assert [p.page_state(pg) for pg in row_pages] == [m.page_state(q) for q in x.pages]
            st = p.stats()
            assert st["free_pages"] == len(m.free) == P - len(seen) and st["open_sessions"] == len(m.sessions)
    p.destroy()
