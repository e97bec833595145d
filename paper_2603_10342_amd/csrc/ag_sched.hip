// Host-side scheduling layer: the TPOT-driven controller (paper Sec. III-B, Algorithm 1) and the table of
// pre-established CU partitions (paper Sec. III-C).  No kernels here; the only device work is creating and
// destroying the CU-masked streams.
#include <cmath>
#include <mutex>
#include <new>
#include <vector>

#include "ag_internal.h"
#include "ag_sched.h"

using namespace ag;

struct ag_ctl {
    ag_ctl_params p;
    std::mutex mu;
    int32_t r_min, b_prefill;
    double dL = 0.0;        // summed decode-step time of the open interval
    int64_t dK = 0;         // decode steps of the open interval
    double tpot = NAN;
    int64_t intervals = 0, raised = 0, lowered = 0;
};

static void fill_state(const ag_ctl* c, ag_ctl_state* s)
{
    s->r_min = c->r_min;
    s->b_prefill = c->b_prefill;
    s->tpot_us = c->tpot;
    s->intervals = c->intervals;
    s->raised = c->raised;
    s->lowered = c->lowered;
}

ag_status ag_ctl_create(const ag_ctl_params* p, ag_ctl** out)
{
    if (!p || !out) { set_error("params or out is NULL"); return AG_ERR_INVALID_ARG; }
    if (!(p->r_base > 0 && p->r_base <= p->r_init && p->r_init <= p->S)) {
        set_error("need 0 < r_base <= r_init <= S, got r_base=%d r_init=%d S=%d", p->r_base, p->r_init, p->S);
        return AG_ERR_INVALID_ARG;
    }
    if (!(p->b_min >= 0 && p->b_min <= p->b_init && p->b_init <= p->b_max)) {
        set_error("need 0 <= b_min <= b_init <= b_max, got %d %d %d", p->b_min, p->b_init, p->b_max);
        return AG_ERR_INVALID_ARG;
    }
    if (p->delta_r < 0 || p->delta_b < 0) { set_error("negative step"); return AG_ERR_INVALID_ARG; }
    if (!(p->theta_low_us <= p->theta_high_us)) {          // also rejects NaN
        set_error("need theta_low <= theta_high, got %g %g", p->theta_low_us, p->theta_high_us);
        return AG_ERR_INVALID_ARG;
    }
    ag_ctl* c = new (std::nothrow) ag_ctl;
    if (!c) { set_error("out of host memory"); return AG_ERR_INVALID_ARG; }
    c->p = *p;
    c->r_min = p->r_init;
    c->b_prefill = p->b_init;
    *out = c;
    return AG_OK;
}

ag_status ag_ctl_destroy(ag_ctl* c)
{
    if (!c) { set_error("ctl is NULL"); return AG_ERR_INVALID_ARG; }
    delete c;
    return AG_OK;
}

ag_status ag_ctl_record_decode(ag_ctl* c, double step_us)
{
    if (!c) { set_error("ctl is NULL"); return AG_ERR_INVALID_ARG; }
    if (!(step_us >= 0.0)) { set_error("step time %g is not a non-negative number", step_us); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(c->mu);
    c->dL += step_us;
    c->dK += 1;
    return AG_OK;
}

// Which way an interval pushes: +1 when the measured time per decode step is above the band (decode needs
// protection), -1 when it is below (prefill may have more), 0 inside the band or when nothing was measured
// (a NaN compares false both ways).  Both edges are exclusive (Algorithm 1).
static int pressure(double tpot_us, const ag_ctl_params& p)
{
    return (tpot_us > p.theta_high_us) - (tpot_us < p.theta_low_us);
}

// v moved by `by`, held inside [lo, hi]
static int32_t moved_within(int32_t v, int64_t by, int32_t lo, int32_t hi)
{
    const int64_t t = (int64_t)v + by;
    return (int32_t)(t < lo ? lo : t > hi ? hi : t);
}

// The feedback rule of Sec. III-B / Algorithm 1 as one signed step: the decode reservation moves WITH the
// pressure, the resume-prefill budget AGAINST it, each by its own increment and inside its own range.
ag_status ag_ctl_tick(ag_ctl* c, ag_ctl_state* out)
{
    if (!c) { set_error("ctl is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(c->mu);
    const ag_ctl_params& p = c->p;
    c->tpot = c->dK ? c->dL / (double)c->dK : NAN;
    const int dir = pressure(c->tpot, p);
    c->r_min = moved_within(c->r_min, (int64_t)dir * p.delta_r, p.r_base, p.S);
    c->b_prefill = moved_within(c->b_prefill, -(int64_t)dir * p.delta_b, p.b_min, p.b_max);
    c->raised += dir > 0;
    c->lowered += dir < 0;
    c->dL = 0.0;
    c->dK = 0;
    ++c->intervals;
    if (out) fill_state(c, out);
    return AG_OK;
}

ag_status ag_ctl_get(ag_ctl* c, ag_ctl_state* out)
{
    if (!c || !out) { set_error("ctl or state_out is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(c->mu);
    fill_state(c, out);
    return AG_OK;
}

int32_t ag_ctl_classify(ag_ctl* c, int32_t req_type, int32_t len)
{
    if (!c) { set_error("ctl is NULL"); return AG_ERR_INVALID_ARG; }
    if (len < 0) { set_error("negative request length"); return AG_ERR_INVALID_ARG; }
    switch (req_type) {
        case AG_REQ_DECODE: return AG_QUEUE_DECODE;
        case AG_REQ_COLD: return AG_QUEUE_PREFILL;
        case AG_REQ_RESUME: {
            std::lock_guard<std::mutex> lk(c->mu);
            return len <= c->b_prefill ? AG_QUEUE_DECODE : AG_QUEUE_PREFILL;
        }
        default: set_error("unknown request type %d", req_type); return AG_ERR_INVALID_ARG;
    }
}

int32_t ag_partition_level_for(int32_t S, int32_t g, int32_t r_min)
{
    if (g <= 0 || S < g) { set_error("need 0 < g <= S, got g=%d S=%d", g, S); return AG_ERR_INVALID_ARG; }
    if (r_min <= g) return g;
    const int64_t k = ((int64_t)r_min + g - 1) / g;      // multiples of g needed
    return k * g >= S ? S : (int32_t)(k * g);
}

// ---------------------------------------------------------------------------------------------------------

struct ag_slots {
    int S = 0, g = 0;
    struct Entry { int units; hipStream_t decode, prefill; };
    std::vector<Entry> e;
    mutable std::mutex mu;
    int current = 0;
};

static void drop_streams(ag_slots* t)
{
    for (auto& x : t->e) {
        if (x.decode) { (void)hipStreamSynchronize(x.decode); (void)hipStreamDestroy(x.decode); }
        if (x.prefill) { (void)hipStreamSynchronize(x.prefill); (void)hipStreamDestroy(x.prefill); }
    }
    t->e.clear();
}

ag_status ag_slots_create(int32_t g, ag_slots** out)
{
    if (!out) { set_error("out is NULL"); return AG_ERR_INVALID_ARG; }
    int32_t cus = 0, xcd = 0;
    ag_status st = ag_device_info(&cus, &xcd, nullptr, nullptr, 0);
    if (st) return st;
    if (xcd <= 0) xcd = 1;
    if (cus <= 0 || cus % xcd) { set_error("%d CUs do not split evenly over %d XCDs", cus, xcd); return AG_ERR_UNSUPPORTED; }
    const int S = cus / xcd;
    if (g <= 0 || g > S) { set_error("granularity %d outside [1, %d]", g, S); return AG_ERR_INVALID_ARG; }
    ag_slots* t = new (std::nothrow) ag_slots;
    if (!t) { set_error("out of host memory"); return AG_ERR_INVALID_ARG; }
    t->S = S;
    t->g = g;
    const int n_words = (cus + 31) / 32;
    std::vector<uint32_t> words((size_t)n_words);
    for (int units = g;; units = units + g > S ? S : units + g) {
        ag_slots::Entry x{units, nullptr, nullptr};
        void* s = nullptr;
        if ((st = ag_cumask_build(words.data(), n_words, cus, xcd, 0, units)) ||
            (st = ag_stream_create_cumask(&s, words.data(), n_words))) { drop_streams(t); delete t; return st; }
        x.decode = (hipStream_t)s;
        t->e.push_back(x);                               // from here on drop_streams sees the entry
        if (units < S) {
            if ((st = ag_cumask_build(words.data(), n_words, cus, xcd, units, S - units)) ||
                (st = ag_stream_create_cumask(&s, words.data(), n_words))) { drop_streams(t); delete t; return st; }
            t->e.back().prefill = (hipStream_t)s;
        }
        if (units == S) break;
    }
    *out = t;
    return AG_OK;
}

ag_status ag_slots_destroy(ag_slots* t)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    drop_streams(t);
    delete t;
    return AG_OK;
}

int32_t ag_slots_count(const ag_slots* t)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    return (int32_t)t->e.size();
}

int32_t ag_slots_units(const ag_slots* t)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    return t->S;
}

ag_status ag_slots_get(const ag_slots* t, int32_t i, int32_t* units, void** ds, void** ps)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    if (i < 0 || i >= (int32_t)t->e.size()) { set_error("entry %d outside [0, %zu)", i, t->e.size()); return AG_ERR_INVALID_ARG; }
    if (units) *units = t->e[i].units;
    if (ds) *ds = (void*)t->e[i].decode;
    if (ps) *ps = (void*)t->e[i].prefill;
    return AG_OK;
}

ag_status ag_slots_bind(ag_slots* t, int32_t r_min, int32_t* index_out)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    const int32_t units = ag_partition_level_for(t->S, t->g, r_min);
    if (units < 0) return AG_ERR_INVALID_ARG;
    // entries are g, 2g, ..., S in order: the index follows from the size
    const int32_t idx = units >= t->S ? (int32_t)t->e.size() - 1 : units / t->g - 1;
    {
        std::lock_guard<std::mutex> lk(t->mu);
        t->current = idx;
    }
    if (index_out) *index_out = idx;
    return AG_OK;
}

int32_t ag_slots_current(const ag_slots* t)
{
    if (!t) { set_error("slots is NULL"); return AG_ERR_INVALID_ARG; }
    std::lock_guard<std::mutex> lk(t->mu);
    return t->current;
}
