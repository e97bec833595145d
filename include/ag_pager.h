/*
 * ag_pager.h - C ABI of the KV page manager (paper Sec. III-C, "Memory management"): the prefill thread and
 * the decode thread share one page pool; a manager hands out pages under a mutex, marks what a finished
 * prefill wrote read-only so the decode thread can use it at once without a copy, and orders the two
 * threads' kernels with events so that a decode never reads keys or values that are still being written.
 *
 * The manager is host-side bookkeeping over page NUMBERS of a pool the caller owns (ag_kv_cache in ag.h);
 * it allocates no device memory.  The only device objects it creates are events (timing disabled): one per
 * session for its writer and one per (session, reader stream) for its readers.  Every function is safe to call from several threads at once.
 *
 * Life of a session
 *   ag_pager_open      -> a session id with no pages
 *   ag_pager_reserve   -> room for n more tokens: takes the missing pages from the free list, all or none;
 *                         returns the position the new tokens start at (the prefix length for ag_kv_append)
 *   (caller)           -> ag_pager_export the block-table rows, copy them to the device, enqueue
 *                         ag_kv_append + attention for the reserved tokens on its stream
 *   ag_pager_commit    -> records the session's event on that stream and seals the reserved tokens: they
 *                         are now part of the session's read-only length
 *   ag_pager_acquire   -> a reader about to launch on another stream: makes that stream wait for the
 *                         session's last commit (no wait when it was committed on the same stream, or when
 *                         the event has already completed) and returns the sealed length
 *   (reader)           -> enqueues its attention kernels on that stream
 *   ag_pager_release   -> records, on the reader's stream and after those launches, that the session's pages
 *                         are in use until this point of the stream
 *   ag_pager_close     -> waits for the session's last commit AND for every release recorded for it, then
 *                         returns its pages to the free list: a page is never handed to another session
 *                         while a committed write or a released read of it may still be running.  A reader
 *                         that never calls ag_pager_release is invisible to close (the caller must then order
 *                         close after that reader itself).
 *
 * Errors: ag_status of ag.h; AG_ERR_NO_SPACE means not enough free pages (or sessions, or row capacity) and
 * that nothing was changed.  Messages through ag_last_error().
 */
#ifndef AG_PAGER_H
#define AG_PAGER_H

#include "ag.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { AG_PAGE_FREE = 0, AG_PAGE_WRITABLE = 1, AG_PAGE_SEALED = 2 } ag_page_state;

typedef struct ag_pager ag_pager;

typedef struct ag_pager_stats {
    int32_t num_pages, free_pages, open_sessions;
    int64_t reserves, failed_reserves, commits;
    int64_t waits_issued;      /* ag_pager_acquire calls that made a stream wait for an event */
    int64_t waits_skipped;     /* ... that needed none: same stream, nothing pending, or already complete */
    int64_t releases;          /* ag_pager_release calls */
    int64_t close_waits;       /* events (writer's or readers') that ag_pager_close calls waited for */
} ag_pager_stats;

AG_API ag_status ag_pager_create(int32_t num_pages, int32_t page_size, int32_t max_sessions,
                                 int32_t max_pages_per_seq, ag_pager** out);
/* Waits for every session's event, destroys the events.  Pages are the caller's: nothing else to free. */
AG_API ag_status ag_pager_destroy(ag_pager* pager);

AG_API ag_status ag_pager_open(ag_pager* pager, int32_t* session_out);
AG_API ag_status ag_pager_close(ag_pager* pager, int32_t session);

/*
 * Room for new_tokens >= 0 more tokens after the tokens reserved so far.  *start_out (may be NULL) receives
 * the position of the first new token.  AG_ERR_NO_SPACE, with nothing changed, if the free list or the row
 * (max_pages_per_seq) cannot cover them.  Positions below the session's sealed length are never handed out
 * again: what a committed prefill wrote stays read-only until the session closes.
 */
AG_API ag_status ag_pager_reserve(ag_pager* pager, int32_t session, int32_t new_tokens, int32_t* start_out);

/*
 * Host-only half of a commit: seals everything reserved so far (sealed length = reserved length) without
 * touching any stream.  For callers that order their streams themselves, and for tests without a device.
 */
AG_API ag_status ag_pager_seal(ag_pager* pager, int32_t session);

/* Seals like ag_pager_seal and records the session's event on `stream` (hipStream_t, NULL = default stream),
 * after the work the caller has enqueued there. */
AG_API ag_status ag_pager_commit(ag_pager* pager, int32_t session, void* stream);

/* See the header comment.  *sealed_len_out (may be NULL) receives the session's read-only length. */
AG_API ag_status ag_pager_acquire(ag_pager* pager, int32_t session, void* stream, int32_t* sealed_len_out);

/*
 * A reader is done enqueueing: records an event on `stream` (the stream ag_pager_acquire was given) after the
 * launches the caller has made there.  ag_pager_close waits for it before the session's pages can be reused
 * (paper Sec. III-C: a decode never consumes partially written KV - which a page handed to another session's
 * prefill while the decode still reads it would be).  One event per (session, stream), re-recorded by every call.
 */
AG_API ag_status ag_pager_release(ag_pager* pager, int32_t session, void* stream);

/* Lengths of a session (any pointer may be NULL): tokens reserved, tokens sealed, pages held. */
AG_API ag_status ag_pager_lengths(ag_pager* pager, int32_t session, int32_t* reserved_out, int32_t* sealed_out,
                                  int32_t* pages_out);

/*
 * Block-table rows for a batch: rows_out is a HOST array [n][max_pages_per_seq] (row-major); row i receives
 * the pages of sessions[i] in logical order, the rest of the row is filled with the row's last page (so that
 * clamped reads past the end stay inside the session), or 0 for a session without pages.
 */
AG_API ag_status ag_pager_export(ag_pager* pager, const int32_t* sessions, int32_t n, int32_t* rows_out);

/* State of one physical page, or AG_ERR_INVALID_ARG (< 0).  A page is sealed when every slot of it lies
 * below its session's sealed length. */
AG_API int32_t ag_pager_page_state(ag_pager* pager, int32_t page);

AG_API ag_status ag_pager_get_stats(ag_pager* pager, ag_pager_stats* out);

#ifdef __cplusplus
}
#endif
#endif /* AG_PAGER_H */
