// KV page manager (paper Sec. III-C, memory management): free list under a mutex, read-only marking of what
// a committed prefill wrote, one event per session to order the writer's stream against readers' streams,
// and one event per (session, reader stream) so that a closing session's pages are not handed out again
// while a reader's kernels may still be reading them.
// Host code; the only device objects are the events.
#include <mutex>
#include <new>
#include <vector>

#include "ag_internal.h"
#include "ag_pager.h"

using namespace ag;

namespace {

struct Session {
    bool open = false;
    int reserved = 0;                 // tokens handed out
    int sealed = 0;                   // tokens committed: read-only from here on
    std::vector<int32_t> pages;       // logical order
    hipEvent_t ev = nullptr;          // created at the first commit
    hipStream_t ev_stream = nullptr;  // where the last commit was recorded
    bool pending = false;             // the last commit's event may not have completed yet
    struct Reader {                   // one per stream that has released the session (events are kept and reused)
        hipStream_t stream = nullptr;
        hipEvent_t ev = nullptr;
        bool pending = false;         // recorded after the reader's launches and not known to have completed
    };
    std::vector<Reader> readers;
    uint64_t gen = 0;                 // counts commits and releases: close notices one that slipped in while it waited
};

}  // namespace

struct ag_pager {
    int num_pages, ps, max_sessions, max_pages;
    std::mutex mu;
    std::vector<int32_t> free_list;   // a stack: the page freed last is reused first
    std::vector<int32_t> owner;       // page -> session, or -1
    std::vector<int32_t> index;       // page -> logical index within its session
    std::vector<Session> sess;
    ag_pager_stats st{};
};

static Session* find(ag_pager* p, int32_t s)
{
    if (s < 0 || s >= p->max_sessions || !p->sess[s].open) { set_error("session %d is not open", s); return nullptr; }
    return &p->sess[s];
}

ag_status ag_pager_create(int32_t num_pages, int32_t page_size, int32_t max_sessions, int32_t max_pages, ag_pager** out)
{
    if (!out) { set_error("out is NULL"); return AG_ERR_INVALID_ARG; }
    if (num_pages <= 0 || page_size <= 0 || max_sessions <= 0 || max_pages <= 0) {
        set_error("num_pages=%d page_size=%d max_sessions=%d max_pages_per_seq=%d: all must be positive", num_pages,
                  page_size, max_sessions, max_pages);
        return AG_ERR_INVALID_ARG;
    }
    if ((int64_t)max_pages * page_size > 0x7fffffff) { set_error("a row of %d pages of %d tokens overflows 32-bit positions", max_pages, page_size); return AG_ERR_INVALID_ARG; }
    ag_pager* p = new (std::nothrow) ag_pager;
    if (!p) { set_error("out of host memory"); return AG_ERR_INVALID_ARG; }
    p->num_pages = num_pages; p->ps = page_size; p->max_sessions = max_sessions; p->max_pages = max_pages;
    p->free_list.resize((size_t)num_pages);
    for (int i = 0; i < num_pages; ++i) p->free_list[(size_t)i] = num_pages - 1 - i;     // page 0 is handed out first
    p->owner.assign((size_t)num_pages, -1);
    p->index.assign((size_t)num_pages, 0);
    p->sess.resize((size_t)max_sessions);
    p->st.num_pages = num_pages;
    *out = p;
    return AG_OK;
}

ag_status ag_pager_destroy(ag_pager* p)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    for (auto& s : p->sess) {
        if (s.ev) { (void)hipEventSynchronize(s.ev); (void)hipEventDestroy(s.ev); }
        for (auto& r : s.readers)
            if (r.ev) { (void)hipEventSynchronize(r.ev); (void)hipEventDestroy(r.ev); }
    }
    delete p;
    return AG_OK;
}

ag_status ag_pager_open(ag_pager* p, int32_t* out)
{
    if (!p || !out) { set_error("pager or session_out is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    for (int s = 0; s < p->max_sessions; ++s)
        if (!p->sess[(size_t)s].open) {
            Session& x = p->sess[(size_t)s];
            x.open = true; x.reserved = 0; x.sealed = 0; x.pages.clear(); x.pending = false; x.ev_stream = nullptr;
            for (auto& r : x.readers) r.pending = false;
            ++p->st.open_sessions;
            *out = s;
            return AG_OK;
        }
    set_error("all %d sessions are open", p->max_sessions);
    return AG_ERR_NO_SPACE;
}

ag_status ag_pager_close(ag_pager* p, int32_t s)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    // The pages must not be reused while work that touches them may still run: the writer's last commit and
    // every reader that released the session.  The waits happen outside the lock; a commit or release that
    // arrives meanwhile (the generation moved) is waited for in another round.
    for (;;) {
        std::vector<hipEvent_t> wait_for;
        uint64_t gen = 0;
        {
            std::lock_guard<std::mutex> lk(p->mu);
            Session* x = find(p, s);
            if (!x) return AG_ERR_INVALID_ARG;
            if (x->pending) wait_for.push_back(x->ev);
            for (auto& r : x->readers)
                if (r.pending) wait_for.push_back(r.ev);
            gen = x->gen;
        }
        for (hipEvent_t e : wait_for) {
            ag_status st = hip_check(hipEventSynchronize(e), "hipEventSynchronize(close)");
            if (st) return st;
        }
        std::lock_guard<std::mutex> lk(p->mu);
        Session* x = find(p, s);
        if (!x) return AG_ERR_INVALID_ARG;             // closed by another thread meanwhile
        if (x->gen != gen) continue;                   // something was committed or released while we waited
        p->st.close_waits += (int64_t)wait_for.size();
        for (auto it = x->pages.rbegin(); it != x->pages.rend(); ++it) {
            p->owner[(size_t)*it] = -1;
            p->free_list.push_back(*it);
        }
        x->pages.clear();
        x->open = false; x->pending = false; x->reserved = x->sealed = 0;
        for (auto& r : x->readers) r.pending = false;
        --p->st.open_sessions;
        return AG_OK;
    }
}

ag_status ag_pager_reserve(ag_pager* p, int32_t s, int32_t n, int32_t* start_out)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    if (n < 0) { set_error("new_tokens %d is negative", n); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    const int64_t want_tokens = (int64_t)x->reserved + n;
    const int64_t want_pages = (want_tokens + p->ps - 1) / p->ps;
    const int64_t more = want_pages - (int64_t)x->pages.size();
    if (want_pages > p->max_pages) {
        ++p->st.failed_reserves;
        set_error("session %d would need %lld pages, a row holds %d", s, (long long)want_pages, p->max_pages);
        return AG_ERR_NO_SPACE;
    }
    if (more > (int64_t)p->free_list.size()) {
        ++p->st.failed_reserves;
        set_error("session %d needs %lld more pages, %zu are free", s, (long long)more, p->free_list.size());
        return AG_ERR_NO_SPACE;
    }
    for (int64_t i = 0; i < more; ++i) {
        const int32_t pg = p->free_list.back();
        p->free_list.pop_back();
        p->owner[(size_t)pg] = s;
        p->index[(size_t)pg] = (int32_t)x->pages.size();
        x->pages.push_back(pg);
    }
    if (start_out) *start_out = x->reserved;
    x->reserved = (int)want_tokens;
    ++p->st.reserves;
    return AG_OK;
}

ag_status ag_pager_seal(ag_pager* p, int32_t s)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    x->sealed = x->reserved;
    ++p->st.commits;
    return AG_OK;
}

ag_status ag_pager_commit(ag_pager* p, int32_t s, void* stream)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    if (!x->ev) {
        ag_status e = hip_check(hipEventCreateWithFlags(&x->ev, hipEventDisableTiming), "hipEventCreateWithFlags");
        if (e) { x->ev = nullptr; return e; }
    }
    // recorded under the lock: a reader that sees the new sealed length also sees the event that guards it
    ag_status e = hip_check(hipEventRecord(x->ev, (hipStream_t)stream), "hipEventRecord(commit)");
    if (e) return e;
    x->ev_stream = (hipStream_t)stream;
    x->pending = true;
    x->sealed = x->reserved;
    ++x->gen;
    ++p->st.commits;
    return AG_OK;
}

ag_status ag_pager_acquire(ag_pager* p, int32_t s, void* stream, int32_t* sealed_out)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    bool wait = false;
    if (x->pending) {
        if (x->ev_stream == (hipStream_t)stream) {
            // same stream: its own order already puts the reader behind the writer
        } else if (hipEventQuery(x->ev) == hipSuccess) {
            x->pending = false;                        // completed: later readers need not ask again
        } else {
            (void)hipGetLastError();                   // hipErrorNotReady is the expected answer
            ag_status e = hip_check(hipStreamWaitEvent((hipStream_t)stream, x->ev, 0), "hipStreamWaitEvent(acquire)");
            if (e) return e;
            wait = true;
        }
    }
    if (wait) ++p->st.waits_issued; else ++p->st.waits_skipped;
    if (sealed_out) *sealed_out = x->sealed;
    return AG_OK;
}

ag_status ag_pager_release(ag_pager* p, int32_t s, void* stream)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    Session::Reader* r = nullptr;
    for (auto& cand : x->readers)
        if (cand.stream == (hipStream_t)stream) { r = &cand; break; }
    if (!r) {
        Session::Reader fresh;
        fresh.stream = (hipStream_t)stream;
        ag_status e = hip_check(hipEventCreateWithFlags(&fresh.ev, hipEventDisableTiming), "hipEventCreateWithFlags");
        if (e) return e;
        x->readers.push_back(fresh);
        r = &x->readers.back();
    }
    // re-recording moves the event to the stream's newest work: one event per reader stream is enough
    ag_status e = hip_check(hipEventRecord(r->ev, (hipStream_t)stream), "hipEventRecord(release)");
    if (e) return e;
    r->pending = true;
    ++x->gen;
    ++p->st.releases;
    return AG_OK;
}

ag_status ag_pager_lengths(ag_pager* p, int32_t s, int32_t* reserved, int32_t* sealed, int32_t* pages)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    Session* x = find(p, s);
    if (!x) return AG_ERR_INVALID_ARG;
    if (reserved) *reserved = x->reserved;
    if (sealed) *sealed = x->sealed;
    if (pages) *pages = (int32_t)x->pages.size();
    return AG_OK;
}

ag_status ag_pager_export(ag_pager* p, const int32_t* sessions, int32_t n, int32_t* rows)
{
    if (!p || !sessions || !rows || n <= 0) { set_error("pager / sessions / rows_out NULL or n=%d not positive", n); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    for (int i = 0; i < n; ++i)
        if (!find(p, sessions[i])) return AG_ERR_INVALID_ARG;      // before anything is written
    for (int i = 0; i < n; ++i) {
        const Session& x = p->sess[(size_t)sessions[i]];
        int32_t* row = rows + (size_t)i * p->max_pages;
        const int have = (int)x.pages.size();
        for (int j = 0; j < p->max_pages; ++j) row[j] = have ? x.pages[(size_t)(j < have ? j : have - 1)] : 0;
    }
    return AG_OK;
}

int32_t ag_pager_page_state(ag_pager* p, int32_t page)
{
    if (!p) { set_error("pager is NULL"); return AG_ERR_INVALID_ARG; }
    if (page < 0 || page >= p->num_pages) { set_error("page %d outside [0, %d)", page, p->num_pages); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    const int s = p->owner[(size_t)page];
    if (s < 0) return AG_PAGE_FREE;
    const int64_t end = ((int64_t)p->index[(size_t)page] + 1) * p->ps;      // one past the page's last slot
    return end <= p->sess[(size_t)s].sealed ? AG_PAGE_SEALED : AG_PAGE_WRITABLE;
}

ag_status ag_pager_get_stats(ag_pager* p, ag_pager_stats* out)
{
    if (!p || !out) { set_error("pager or out is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(p->mu);
    p->st.free_pages = (int32_t)p->free_list.size();
    *out = p->st;
    return AG_OK;
}
