"""The KV page manager (paper Sec. III-C, memory management) without a device: the free list, all-or-nothing
reservations, read-only marking, rows, and many threads at once.  Which physical page a session receives is
the manager's choice; the tests check what must hold whichever it chooses (disjoint ownership, conservation,
order of logical pages).  The random walk against the plain model of the bookkeeping (oracle/pager_model.py)
is in tests/test_pager_model_pins.py."""
import random
import threading

import numpy as np
import pytest

from paper_2603_10342_amd import binding as B


def pages_of(p, s):
    n = p.lengths(s)["pages"]
    return [int(x) for x in p.export([s])[0][:n]]


def test_reserve_grows_by_whole_pages_and_reports_the_start():
    p = B.Pager(64, 16, 4, 8)
    s = p.open()
    assert p.lengths(s) == {"reserved": 0, "sealed": 0, "pages": 0}
    assert p.reserve(s, 0) == 0 and p.lengths(s)["pages"] == 0
    assert p.reserve(s, 1) == 0 and p.lengths(s)["pages"] == 1
    assert p.reserve(s, 15) == 1 and p.lengths(s)["pages"] == 1          # fills the page exactly
    assert p.reserve(s, 1) == 16 and p.lengths(s)["pages"] == 2
    assert p.reserve(s, 40) == 17 and p.lengths(s) == {"reserved": 57, "sealed": 0, "pages": 4}
    assert p.stats()["free_pages"] == 60
    rows = p.export([s])
    assert rows.shape == (1, 8) and len(set(rows[0][:4])) == 4 and list(rows[0][4:]) == [rows[0][3]] * 4
    p.destroy()


def test_reservation_is_all_or_nothing():
    p = B.Pager(10, 16, 4, 8)
    a, b = p.open(), p.open()
    p.reserve(a, 16 * 7)
    before = (p.lengths(b), p.stats()["free_pages"], pages_of(p, a))
    with pytest.raises(B.AgError) as e:
        p.reserve(b, 16 * 3 + 1)                       # needs 4 pages, 3 are free
    assert e.value.status == B.AG_ERR_NO_SPACE
    assert (p.lengths(b), p.stats()["free_pages"], pages_of(p, a)) == before
    p.reserve(b, 16 * 3)                               # exactly what is left
    assert p.stats()["free_pages"] == 0
    with pytest.raises(B.AgError) as e:
        p.reserve(a, 16 * 1 + 1)                       # row capacity: 8 pages per session
    assert e.value.status == B.AG_ERR_NO_SPACE and p.lengths(a)["reserved"] == 112
    assert p.stats()["failed_reserves"] == 2
    p.destroy()


def test_sealed_region_is_read_only_until_close():
    p = B.Pager(32, 16, 2, 16)
    s = p.open()
    p.reserve(s, 40)
    pg = pages_of(p, s)
    assert [p.page_state(x) for x in pg] == [B.AG_PAGE_WRITABLE] * 3
    p.seal(s)
    # pages 0 and 1 lie wholly below 40; page 2 still has free slots and stays writable
    assert [p.page_state(x) for x in pg] == [B.AG_PAGE_SEALED, B.AG_PAGE_SEALED, B.AG_PAGE_WRITABLE]
    assert p.lengths(s)["sealed"] == 40
    start = p.reserve(s, 30)
    assert start == 40                                 # new tokens never land below the sealed length
    assert pages_of(p, s)[:3] == pg                    # and the sealed pages keep their place in the row
    p.seal(s)
    assert [p.page_state(x) for x in pages_of(p, s)] == [B.AG_PAGE_SEALED] * 4 + [B.AG_PAGE_WRITABLE]
    held = pages_of(p, s)
    p.close(s)
    assert all(p.page_state(x) == B.AG_PAGE_FREE for x in held) and p.stats()["free_pages"] == 32
    with pytest.raises(B.AgError):
        p.reserve(s, 1)                                # closed
    p.destroy()


def test_sessions_run_out_and_come_back():
    p = B.Pager(8, 16, 2, 4)
    a, b = p.open(), p.open()
    assert a != b
    with pytest.raises(B.AgError) as e:
        p.open()
    assert e.value.status == B.AG_ERR_NO_SPACE
    p.close(a)
    assert p.open() == a
    p.destroy()


def test_bad_arguments():
    for args in ((0, 16, 1, 1), (8, 0, 1, 1), (8, 16, 0, 1), (8, 16, 1, 0), (8, 1 << 20, 1, 1 << 12)):
        with pytest.raises(B.AgError):
            B.Pager(*args)
    p = B.Pager(8, 16, 2, 4)
    s = p.open()
    with pytest.raises(B.AgError):
        p.reserve(s, -1)
    with pytest.raises(B.AgError):
        p.reserve(5, 1)
    with pytest.raises(B.AgError):
        p.page_state(8)
    with pytest.raises(B.AgError):
        p.export([s, 1])                               # session 1 is not open: nothing is written
    l = B.lib()
    assert l.ag_pager_open(None, None) == B.AG_ERR_INVALID_ARG and l.ag_pager_destroy(None) == B.AG_ERR_INVALID_ARG
    assert B.ag_status_string(B.AG_ERR_NO_SPACE) == "AG_ERR_NO_SPACE"
    p.destroy()


def test_threads_share_the_pool_without_losing_or_doubling_pages():
    """A prefill thread and a decode thread (and two more) allocate and release concurrently."""
    P, ps = 512, 16
    p = B.Pager(P, ps, 64, 16)
    errors = []
    seen_lock = threading.Lock()
    live = {}                                          # page -> session, as the threads observed it

    def worker(seed):
        rnd = random.Random(seed)
        try:
            for _ in range(300):
                s = p.open()
                got = []
                for _ in range(rnd.randint(1, 6)):
                    try:
                        p.reserve(s, rnd.randint(1, 40))
                    except B.AgError as e:
                        assert e.status == B.AG_ERR_NO_SPACE
                        break
                mine = pages_of(p, s)
                with seen_lock:
                    for pg in mine:
                        assert pg not in live, f"page {pg} handed to sessions {live[pg]} and {s}"
                        live[pg] = s
                p.seal(s)
                with seen_lock:
                    for pg in mine:
                        del live[pg]
                p.close(s)
        except Exception as e:                          # noqa: BLE001
            errors.append(repr(e))

    ts = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert not errors, errors
    st = p.stats()
    assert st["free_pages"] == P and st["open_sessions"] == 0
    p.destroy()
