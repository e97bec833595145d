// Host-only exerciser of the library's CPU-side code - argument validation (ag_api), the scheduling layer
// (ag_sched) and the page manager (ag_pager) - built by a plain C++ compiler against the stand-in HIP runtime
// in this folder and run under the sanitizers (see tests/test_host_sanitizers.py).  TEST INFRASTRUCTURE ONLY.
// The kernel launchers are replaced by recorders: no kernel exists in this build.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>
#include <memory>
#include <random>
#include <set>
#include <thread>
#include <vector>

#include "ag_internal.h"
#include "ag_pager.h"
#include "ag_sched.h"

#define CHECK(cond)                                                                       \
    do {                                                                                  \
        if (!(cond)) {                                                                    \
            fprintf(stderr, "%s:%d: CHECK failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, ag_last_error()); \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

// ---- recorders in place of the kernel launchers -------------------------------------------------------
namespace ag {
static std::atomic<int> g_launches[6];
enum { L_APPEND, L_GENERAL, L_PREFILL, L_DECODE, L_MERGED, L_PROBE };
static unsigned char g_fake_scratch[64];
ag_status launch_kv_append(const CacheView&, const void*, const void*, const int32_t*, int, const int32_t*, const int32_t*,
                           const int32_t*, int, int, hipStream_t) { ++g_launches[L_APPEND]; return AG_OK; }
ag_status launch_attn_general(const AttnArgs&, hipStream_t) { ++g_launches[L_GENERAL]; return AG_OK; }
bool prefill_mfma_supported(const AttnArgs& a) { return a.c.dtype == AG_BF16 && a.c.d == 128 && a.c.ps == 16; }
ag_status launch_prefill_mfma(const AttnArgs&, hipStream_t) { ++g_launches[L_PREFILL]; return AG_OK; }
bool decode_mfma_supported(const AttnArgs& a) { return a.c.dtype == AG_BF16 && a.c.d == 128 && a.c.ps == 16; }
size_t decode_workspace_bytes(int batch, int hq, int d, int max_ctx) { return (size_t)batch * hq * (size_t)(d + 2) * 4 * (size_t)(max_ctx / 256 + 2); }
ag_status launch_decode_mfma(const AttnArgs&, void* ws, hipStream_t) { CHECK(ws != nullptr); ++g_launches[L_DECODE]; return AG_OK; }
ag_status decode_static_scratch(void** p) { *p = g_fake_scratch; return AG_OK; }
size_t decode_step_workspace_bytes(int batch, int hq, int d, int max_ctx) { return 256 + decode_workspace_bytes(batch, hq, d, max_ctx); }
ag_status launch_decode_step(const AttnArgs&, const void* k, const void* v, void* ws, hipStream_t) { CHECK(k && v && ws); ++g_launches[L_DECODE]; return AG_OK; }
bool merged_mfma_supported(const AttnArgs& a) { return decode_mfma_supported(a); }
size_t merged_workspace_bytes(int rows, int hq, int max_ctx) { return (size_t)rows * hq * 520 * (size_t)(max_ctx / 256 + 2); }
ag_status launch_merged_mfma(const AttnArgs&, void*, hipStream_t) { ++g_launches[L_MERGED]; return AG_OK; }
ag_status launch_probe(uint32_t*, int, int, hipStream_t) { ++g_launches[L_PROBE]; return AG_OK; }
}  // namespace ag

// ---- 1. validation layer ---------------------------------------------------------------------------------
static void test_validation()
{
    // every buffer is a heap block of the exact size a caller would pass: an overrun is the sanitizer's to find
    std::vector<int32_t> bt(4 * 8), lens(4, 16), cu{0, 16, 32, 48, 64};
    std::vector<uint16_t> q(64 * 8 * 128), out(64 * 8 * 128), kpool(32 * 2 * 16 * 128), vpool(32 * 2 * 16 * 128);
    ag_kv_cache c{kpool.data(), vpool.data(), 32, 16, 2, 128, AG_BF16};
    CHECK(ag_attn_prefill(&c, q.data(), out.data(), bt.data(), 8, lens.data(), cu.data(), 4, 64, 16, 8, 0.1f, nullptr) == AG_OK);
    CHECK(ag::g_launches[ag::L_PREFILL] == 1);
    ag_kv_cache f = c;
    f.dtype = AG_F32;
    CHECK(ag_attn_prefill(&f, q.data(), out.data(), bt.data(), 8, lens.data(), cu.data(), 4, 64, 16, 8, 0.1f, nullptr) == AG_OK);
    CHECK(ag::g_launches[ag::L_GENERAL] == 1);
    CHECK(ag_attn_prefill(nullptr, q.data(), out.data(), bt.data(), 8, lens.data(), cu.data(), 4, 64, 16, 8, 0.1f, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_attn_prefill(&c, q.data(), out.data(), bt.data(), 8, lens.data(), cu.data(), 4, 64, 16, 7, 0.1f, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_attn_prefill(&c, q.data(), out.data(), bt.data(), 8, lens.data(), cu.data(), 4, 64, 16, 8, NAN, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_attn_resume(&c, q.data(), out.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, 16, 129, 8, 0.1f, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_attn_resume(&c, q.data(), out.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, 16, 128, 8, 0.1f, nullptr) == AG_OK);
    for (int bad_d : {0, 100, 264, 512}) {
        ag_kv_cache b = c;
        b.head_dim = bad_d;
        CHECK(ag_kv_append(&b, q.data(), q.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, nullptr) == AG_ERR_UNSUPPORTED);
    }
    CHECK(ag_kv_append(&c, q.data(), q.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, nullptr) == AG_OK);
    CHECK(ag_kv_append(&c, (const char*)q.data() + 2, q.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, nullptr) == AG_ERR_INVALID_ARG);
    // decode: workspace checks, then the static-scratch variant and its size limit
    std::vector<float> ws(ag_attn_decode_workspace_bytes(4, 8, 128, 128) / 4);
    CHECK(ag_attn_decode(&c, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, ws.data(), ws.size() * 4, nullptr) == AG_OK);
    CHECK(ag_attn_decode(&c, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, ws.data(), ws.size() * 4 - 4, nullptr) == AG_ERR_WORKSPACE);
    CHECK(ag_attn_decode(&c, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 129, 8, 0.1f, ws.data(), ws.size() * 4, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_attn_decode_static(&c, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, nullptr) == AG_OK);
    CHECK(ag_attn_decode_static(&c, q.data(), out.data(), bt.data(), 1 << 20, lens.data(), 4096, 1 << 24, 8, 0.1f, nullptr) == AG_ERR_WORKSPACE);
    CHECK(ag::g_launches[ag::L_DECODE] == 2);
    std::vector<float> wss(ag_decode_step_workspace_bytes(4, 8, 128, 128) / 4);
    CHECK(ag_decode_step(&c, q.data(), q.data(), q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, wss.data(), wss.size() * 4, nullptr) == AG_OK);
    CHECK(ag_decode_step(&c, q.data(), nullptr, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, wss.data(), wss.size() * 4, nullptr) == AG_ERR_INVALID_ARG);
    CHECK(ag_decode_step(&c, q.data(), q.data(), q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, wss.data(), wss.size() * 4 - 16, nullptr) == AG_ERR_WORKSPACE);
    CHECK(ag_decode_step(&f, q.data(), q.data(), q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, wss.data(), wss.size() * 4, nullptr) == AG_ERR_UNSUPPORTED);
    CHECK(ag::g_launches[ag::L_DECODE] == 3);
    std::vector<float> wsm(ag_attn_merged_workspace_bytes(64, 8, 128) / 4);
    CHECK(ag_attn_merged(&c, q.data(), out.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, 16, 128, 8, 0.1f,
                         wsm.data(), wsm.size() * 4, nullptr) == AG_OK);
    CHECK(ag_attn_merged(&c, q.data(), out.data(), bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, 64, 16, 128, 8, 0.1f,
                         wsm.data(), 8, nullptr) == AG_ERR_WORKSPACE);
    // ag_debug_validate reads the "device" arrays through the stand-in memcpy: page ids and lengths
    for (size_t i = 0; i < bt.size(); ++i) bt[i] = (int32_t)(i % 32);
    CHECK(ag_debug_validate(&c, bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, nullptr) == AG_OK);
    bt[9] = 32;
    CHECK(ag_debug_validate(&c, bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, nullptr) == AG_ERR_INVALID_ARG);
    bt[9] = 1;
    cu[2] = 31;
    CHECK(ag_debug_validate(&c, bt.data(), 8, lens.data(), lens.data(), cu.data(), 4, nullptr) == AG_ERR_INVALID_ARG);
    // CU masks: exact-size word arrays
    for (int n_xcd : {1, 4, 8})
        for (int per : {8, 32, 38}) {
            const int total = n_xcd * per, n_words = (total + 31) / 32;
            std::unique_ptr<uint32_t[]> w(new uint32_t[(size_t)n_words]);
            CHECK(ag_cumask_build(w.get(), n_words, total, n_xcd, 1, per - 1) == AG_OK);
            int bits = 0;
            for (int i = 0; i < n_words; ++i) bits += __builtin_popcount(w[i]);
            CHECK(bits == n_xcd * (per - 1));
            CHECK(ag_cumask_build(w.get(), n_words - 1 > 0 ? n_words - 1 : 0, total, n_xcd, 0, per) != AG_OK || n_words * 32 - 32 >= total);
            CHECK(ag_cumask_build(w.get(), n_words, total, n_xcd, 1, per) == AG_ERR_INVALID_ARG);
        }
    // the event bracket of the profiling aid
    CHECK(ag_prof_enable(3) == AG_OK);
    for (int i = 0; i < 5; ++i)
        CHECK(ag_attn_decode(&c, q.data(), out.data(), bt.data(), 8, lens.data(), 4, 128, 8, 0.1f, ws.data(), ws.size() * 4, nullptr) == AG_OK);
    int n = 0;
    CHECK(ag_prof_collect(nullptr, nullptr, nullptr, &n) == AG_OK && n == 0);   // the recorders bracket nothing
    CHECK(ag_prof_disable() == AG_OK);
    char name[8];
    int32_t cus = 0, xcd = 0, wave = 0;
    CHECK(ag_device_info(&cus, &xcd, &wave, name, sizeof(name)) == AG_OK && cus == 256 && xcd == 8 && name[7] == 0);
}

// ---- 2. controller and partition table, from several threads -----------------------------------------
static void test_sched()
{
    ag_ctl_params p{32, 4, 8, 256, 4, 64, 64, 512, 200.0, 300.0};
    ag_ctl* ctl = nullptr;
    CHECK(ag_ctl_create(&p, &ctl) == AG_OK);
    ag_ctl_params bad = p;
    bad.r_init = 40;
    ag_ctl* none = nullptr;
    CHECK(ag_ctl_create(&bad, &none) == AG_ERR_INVALID_ARG);
    std::atomic<bool> stop{false};
    std::vector<std::thread> th;
    for (int t = 0; t < 3; ++t)
        th.emplace_back([&, t] {
            std::mt19937 rng(100 + t);
            while (!stop.load()) {
                CHECK(ag_ctl_record_decode(ctl, 100.0 + (double)(rng() % 400)) == AG_OK);
                const int32_t qd = ag_ctl_classify(ctl, AG_REQ_RESUME, (int32_t)(rng() % 600));
                CHECK(qd == AG_QUEUE_DECODE || qd == AG_QUEUE_PREFILL);
            }
        });
    for (int k = 0; k < 2000; ++k) {
        ag_ctl_state st;
        CHECK(ag_ctl_tick(ctl, &st) == AG_OK);
        CHECK(st.r_min >= p.r_base && st.r_min <= p.S && st.b_prefill >= p.b_min && st.b_prefill <= p.b_max);
        CHECK((st.r_min - p.r_init) % p.delta_r == 0 && (st.b_prefill - p.b_init) % p.delta_b == 0);
    }
    stop.store(true);
    for (auto& t : th) t.join();
    CHECK(ag_ctl_destroy(ctl) == AG_OK);

    CHECK(ag_partition_level_for(100, 10, 37) == 40);
    CHECK(ag_partition_level_for(32, 4, 33) == 32 && ag_partition_level_for(32, 4, 0) == 4);
    for (int g : {1, 4, 12, 32}) {
        ag_slots* s = nullptr;
        CHECK(ag_slots_create(g, &s) == AG_OK);
        const int n = ag_slots_count(s);
        CHECK(n == (32 + g - 1) / g && ag_slots_units(s) == 32);
        std::set<void*> seen;
        for (int i = 0; i < n; ++i) {
            int32_t units = 0;
            void *d = nullptr, *pf = nullptr;
            CHECK(ag_slots_get(s, i, &units, &d, &pf) == AG_OK);
            CHECK(units == (i == n - 1 ? 32 : g * (i + 1)) && d && (pf != nullptr) == (units < 32));
            CHECK(seen.insert(d).second && (!pf || seen.insert(pf).second));
            // the two masks are disjoint and together cover the device
            const auto& dm = ((hipStream_t)d)->mask;
            uint32_t all_or = 0, all_and = 0;
            for (size_t w = 0; w < dm.size(); ++w) {
                const uint32_t pm = pf ? ((hipStream_t)pf)->mask[w] : 0u;
                all_and |= dm[w] & pm;
                all_or |= ~(dm[w] | pm);
            }
            CHECK(all_and == 0 && all_or == 0);
        }
        CHECK(ag_slots_get(s, n, nullptr, nullptr, nullptr) == AG_ERR_INVALID_ARG);
        std::vector<std::thread> bt;
        for (int t = 0; t < 3; ++t)
            bt.emplace_back([&, t] {
                for (int k = 0; k < 500; ++k) {
                    int32_t idx = -1;
                    CHECK(ag_slots_bind(s, 1 + (k * 7 + t) % 40, &idx) == AG_OK && idx >= 0 && idx < n);
                    const int cur = ag_slots_current(s);
                    CHECK(cur >= 0 && cur < n);
                }
            });
        for (auto& t : bt) t.join();
        CHECK(ag_slots_destroy(s) == AG_OK);
    }
    CHECK(fakehip::rt().live_streams == 0);
    ag_slots* s = nullptr;
    CHECK(ag_slots_create(0, &s) == AG_ERR_INVALID_ARG && ag_slots_create(33, &s) == AG_ERR_INVALID_ARG);
}

// ---- 3. page manager: ordering of close against writers and readers ------------------------------------
static std::vector<int32_t> pages_of(ag_pager* p, int32_t s, int max_pages)
{
    std::vector<int32_t> row((size_t)max_pages);
    int32_t n = 0;
    CHECK(ag_pager_export(p, &s, 1, row.data()) == AG_OK);
    CHECK(ag_pager_lengths(p, s, nullptr, nullptr, &n) == AG_OK);
    row.resize((size_t)n);
    return row;
}

static void test_pager_ordering()
{
    auto& rt = fakehip::rt();
    ag_pager* p = nullptr;
    CHECK(ag_pager_create(64, 16, 8, 64, &p) == AG_OK);
    hipStream_t writer = nullptr, reader = nullptr, reader2 = nullptr;
    uint32_t m = 1;
    CHECK(hipExtStreamCreateWithCUMask(&writer, 1, &m) == hipSuccess && hipExtStreamCreateWithCUMask(&reader, 1, &m) == hipSuccess &&
          hipExtStreamCreateWithCUMask(&reader2, 1, &m) == hipSuccess);

    // (a) readers still in flight when the session closes: close must wait for the writer's commit AND every
    // reader's release before a single page returns to the free list
    int32_t s = -1, start = -1, sealed = 0;
    CHECK(ag_pager_open(p, &s) == AG_OK && ag_pager_reserve(p, s, 100, &start) == AG_OK && start == 0);
    const std::vector<int32_t> held = pages_of(p, s, 64);
    CHECK(held.size() == 7);
    CHECK(ag_pager_commit(p, s, writer) == AG_OK);
    fakehip::reset_logs();
    CHECK(ag_pager_acquire(p, s, reader, &sealed) == AG_OK && sealed == 100);
    CHECK(rt.stream_waits.size() == 1 && rt.stream_waits[0].stream == reader);     // the reader waits for the commit
    CHECK(ag_pager_release(p, s, reader) == AG_OK);
    CHECK(ag_pager_acquire(p, s, reader2, nullptr) == AG_OK && ag_pager_release(p, s, reader2) == AG_OK);
    fakehip::reset_logs();
    int waits_seen = 0;
    rt.on_event_sync = [&](hipEvent_t) {
        ++waits_seen;
        for (int32_t pg : held) CHECK(ag_pager_page_state(p, pg) != AG_PAGE_FREE);    // not yet reusable
        int32_t other = -1;                                                            // and handed to nobody:
        CHECK(ag_pager_open(p, &other) == AG_OK);                                      // a session that takes every
        CHECK(ag_pager_reserve(p, other, 57 * 16, nullptr) == AG_OK);                  // free page gets none of them
        for (int32_t pg : pages_of(p, other, 64))
            for (int32_t h : held) CHECK(pg != h);
        CHECK(ag_pager_reserve(p, other, 1, nullptr) == AG_ERR_NO_SPACE);
        CHECK(ag_pager_close(p, other) == AG_OK);
    };
    CHECK(ag_pager_close(p, s) == AG_OK);
    CHECK(waits_seen == 3 && rt.host_waits.size() == 3);                               // writer + two reader streams
    for (int32_t pg : held) CHECK(ag_pager_page_state(p, pg) == AG_PAGE_FREE);
    ag_pager_stats st;
    CHECK(ag_pager_get_stats(p, &st) == AG_OK && st.free_pages == 64 && st.close_waits == 3 && st.releases == 2);

    // (b) everything already complete: close waits for nothing that is not pending ... except what it cannot know
    rt.on_event_sync = nullptr;
    CHECK(ag_pager_open(p, &s) == AG_OK && ag_pager_reserve(p, s, 20, nullptr) == AG_OK && ag_pager_commit(p, s, writer) == AG_OK);
    fakehip::finish(writer);
    CHECK(ag_pager_acquire(p, s, reader, nullptr) == AG_OK);                           // finds the commit complete: no wait
    CHECK(ag_pager_get_stats(p, &st) == AG_OK && st.waits_skipped >= 1);
    fakehip::reset_logs();
    CHECK(ag_pager_close(p, s) == AG_OK && rt.host_waits.empty());

    // (c) a commit that slips in while close is waiting outside the lock is waited for too
    CHECK(ag_pager_open(p, &s) == AG_OK && ag_pager_reserve(p, s, 20, nullptr) == AG_OK && ag_pager_commit(p, s, writer) == AG_OK);
    int rounds = 0;
    rt.on_event_sync = [&](hipEvent_t) {
        if (rounds++ == 0) {
            CHECK(ag_pager_reserve(p, s, 5, nullptr) == AG_OK && ag_pager_commit(p, s, reader) == AG_OK);
        }
    };
    fakehip::reset_logs();
    CHECK(ag_pager_close(p, s) == AG_OK);
    CHECK(rounds == 2 && rt.host_waits.size() == 2);
    rt.on_event_sync = nullptr;
    CHECK(ag_pager_get_stats(p, &st) == AG_OK && st.free_pages == 64 && st.open_sessions == 0);

    // (d) same-stream reader: no stream wait is issued, the release still guards the close
    CHECK(ag_pager_open(p, &s) == AG_OK && ag_pager_reserve(p, s, 33, nullptr) == AG_OK && ag_pager_commit(p, s, writer) == AG_OK);
    fakehip::reset_logs();
    CHECK(ag_pager_acquire(p, s, writer, nullptr) == AG_OK && rt.stream_waits.empty());
    CHECK(ag_pager_release(p, s, writer) == AG_OK);
    CHECK(ag_pager_close(p, s) == AG_OK && rt.host_waits.size() == 2);
    CHECK(ag_pager_release(p, s, writer) == AG_ERR_INVALID_ARG);                       // closed
    CHECK(ag_pager_destroy(p) == AG_OK);
    CHECK(rt.live_events == 0);
}

// ---- 4. page manager under four threads -------------------------------------------------------------------
static void test_pager_threads()
{
    ag_pager* p = nullptr;
    const int kPages = 512, kRow = 40;
    CHECK(ag_pager_create(kPages, 16, 64, kRow, &p) == AG_OK);
    std::vector<hipStream_t> streams(4);
    uint32_t m = 1;
    for (auto& s : streams) CHECK(hipExtStreamCreateWithCUMask(&s, 1, &m) == hipSuccess);
    std::atomic<int> failures{0};
    std::vector<std::thread> th;
    for (int t = 0; t < 4; ++t)
        th.emplace_back([&, t] {
            std::mt19937 rng(7 + t);
            std::vector<int32_t> mine;
            std::vector<int32_t> row((size_t)kRow);
            for (int k = 0; k < 3000; ++k) {
                const unsigned op = rng() % 8;
                if ((op == 0 && mine.size() < 12) || mine.empty()) {
                    int32_t s = -1;
                    if (ag_pager_open(p, &s) == AG_OK) mine.push_back(s);
                    if (mine.empty()) continue;
                }
                const size_t i = rng() % mine.size();
                const int32_t s = mine[i];
                switch (op) {
                    case 1: case 2: {
                        const ag_status e = ag_pager_reserve(p, s, (int32_t)(rng() % 90), nullptr);
                        if (e != AG_OK && e != AG_ERR_NO_SPACE) ++failures;
                        break;
                    }
                    case 3: if (ag_pager_commit(p, s, streams[t]) != AG_OK) ++failures; break;
                    case 4: {
                        int32_t sealed = -1, reserved = -1;
                        if (ag_pager_acquire(p, s, streams[(t + 1) % 4], &sealed) != AG_OK) ++failures;
                        if (ag_pager_release(p, s, streams[(t + 1) % 4]) != AG_OK) ++failures;
                        if (ag_pager_lengths(p, s, &reserved, nullptr, nullptr) != AG_OK || sealed > reserved) ++failures;
                        break;
                    }
                    case 5: if (ag_pager_export(p, &s, 1, row.data()) != AG_OK) ++failures; break;
                    case 6:
                        if (ag_pager_close(p, s) != AG_OK) ++failures;
                        mine.erase(mine.begin() + (long)i);
                        break;
                    default: fakehip::finish(streams[rng() % 4]); break;
                }
            }
            for (int32_t s : mine)
                if (ag_pager_close(p, s) != AG_OK) ++failures;
        });
    for (auto& t : th) t.join();
    CHECK(failures.load() == 0);
    ag_pager_stats st;
    CHECK(ag_pager_get_stats(p, &st) == AG_OK && st.free_pages == kPages && st.open_sessions == 0);
    for (int pg = 0; pg < kPages; ++pg) CHECK(ag_pager_page_state(p, pg) == AG_PAGE_FREE);
    CHECK(ag_pager_destroy(p) == AG_OK);
}

int main()
{
    test_validation();
    test_sched();
    test_pager_ordering();
    test_pager_threads();
    printf("host driver ok\n");
    return 0;
}
