// A stand-in for <hip/hip_runtime.h> that lets the library's HOST-side sources (argument validation, the
// scheduling layer, the page manager) be compiled by a plain C++ compiler and run without a GPU, under the
// address / undefined-behaviour / thread sanitizers.  TEST INFRASTRUCTURE ONLY: nothing here models a kernel.
//
// Streams are counters: recording an event on a stream takes the stream's next ticket, and the event has
// completed once the stream's `done` counter reached that ticket.  Nothing completes by itself: a test moves
// `done` (fakehip::finish), and a host-side wait (hipEventSynchronize / hipStreamSynchronize) first calls the
// test's hook - so the test can look at the library's state at the moment of the wait - and then completes
// what it waited for.  hipStreamWaitEvent is logged.
#pragma once

#include <stdint.h>
#include <string.h>

#include <functional>
#include <mutex>
#include <vector>

#define __host__
#define __device__
#define __global__
#define __forceinline__ inline

typedef enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorNotReady = 600 } hipError_t;
typedef enum { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2 } hipMemcpyKind;
typedef enum { hipDeviceAttributeNumberOfXccs = 1, hipDeviceAttributeMultiprocessorCount = 2 } hipDeviceAttribute_t;
enum { hipEventDisableTiming = 2 };

struct fake_stream { uint64_t enqueued = 0, done = 0; std::vector<uint32_t> mask; bool alive = true; };
struct fake_event { fake_stream* stream = nullptr; uint64_t ticket = 0; bool recorded = false; bool alive = true; };
typedef fake_stream* hipStream_t;
typedef fake_event* hipEvent_t;

struct hipDeviceProp_t { int multiProcessorCount; int warpSize; char gcnArchName[256]; };

namespace fakehip {

struct Runtime {
    std::recursive_mutex mu;
    fake_stream null_stream;
    std::vector<fake_stream*> streams;
    std::vector<fake_event*> events;
    std::function<void(hipEvent_t)> on_event_sync;       // called (without the lock) before a host-side event wait
    struct Wait { hipStream_t stream; hipEvent_t event; uint64_t ticket; };
    std::vector<Wait> stream_waits;                      // every hipStreamWaitEvent, in order
    std::vector<hipEvent_t> host_waits;                  // every hipEventSynchronize, in order
    int live_events = 0, live_streams = 0;
    ~Runtime()                                           // destroyed objects are kept until here, so that a use
    {                                                    // after destroy is an error code, not a dangling pointer
        for (fake_stream* s : streams) delete s;
        for (fake_event* e : events) delete e;
    }
};
inline Runtime& rt() { static Runtime r; return r; }
inline fake_stream* real(hipStream_t s) { return s ? s : &rt().null_stream; }
// the stream's work up to now has finished
inline void finish(hipStream_t s) { std::lock_guard<std::recursive_mutex> lk(rt().mu); real(s)->done = real(s)->enqueued; }
inline void reset_logs() { std::lock_guard<std::recursive_mutex> lk(rt().mu); rt().stream_waits.clear(); rt().host_waits.clear(); }

}  // namespace fakehip

inline const char* hipGetErrorString(hipError_t e) { return e == hipSuccess ? "hipSuccess" : e == hipErrorNotReady ? "hipErrorNotReady" : "hipErrorInvalidValue"; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) { memset(p, 0, sizeof(*p)); p->multiProcessorCount = 256; p->warpSize = 64; strcpy(p->gcnArchName, "gfx950:hostbuild"); return hipSuccess; }
inline hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t a, int) { *v = a == hipDeviceAttributeNumberOfXccs ? 8 : 256; return hipSuccess; }
inline hipError_t hipMemcpy(void* dst, const void* src, size_t n, hipMemcpyKind) { memcpy(dst, src, n); return hipSuccess; }

inline hipError_t hipExtStreamCreateWithCUMask(hipStream_t* s, uint32_t n_words, const uint32_t* words)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    fake_stream* st = new fake_stream;
    st->mask.assign(words, words + n_words);
    fakehip::rt().streams.push_back(st);
    ++fakehip::rt().live_streams;
    *s = st;
    return hipSuccess;
}
inline hipError_t hipStreamSynchronize(hipStream_t s) { fakehip::finish(s); return hipSuccess; }
inline hipError_t hipStreamDestroy(hipStream_t s)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (!s || !s->alive) return hipErrorInvalidValue;
    s->alive = false;                                   // kept allocated: a use after destroy is reported, not a crash
    --fakehip::rt().live_streams;
    return hipSuccess;
}
inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    *e = new fake_event;
    fakehip::rt().events.push_back(*e);
    ++fakehip::rt().live_events;
    return hipSuccess;
}
inline hipError_t hipEventCreate(hipEvent_t* e) { return hipEventCreateWithFlags(e, 0); }
inline hipError_t hipEventDestroy(hipEvent_t e)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (!e || !e->alive) return hipErrorInvalidValue;
    e->alive = false;
    --fakehip::rt().live_events;
    return hipSuccess;
}
inline hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (!e || !e->alive || (s && !s->alive)) return hipErrorInvalidValue;
    e->stream = fakehip::real(s);
    e->ticket = ++e->stream->enqueued;
    e->recorded = true;
    return hipSuccess;
}
inline hipError_t hipEventQuery(hipEvent_t e)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (!e || !e->alive) return hipErrorInvalidValue;
    return !e->recorded || e->stream->done >= e->ticket ? hipSuccess : hipErrorNotReady;
}
inline hipError_t hipEventSynchronize(hipEvent_t e)
{
    std::function<void(hipEvent_t)> hook;
    {
        std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
        if (!e || !e->alive) return hipErrorInvalidValue;
        fakehip::rt().host_waits.push_back(e);
        hook = fakehip::rt().on_event_sync;
    }
    if (hook) hook(e);
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (e->recorded && e->stream->done < e->ticket) e->stream->done = e->ticket;
    return hipSuccess;
}
inline hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    std::lock_guard<std::recursive_mutex> lk(fakehip::rt().mu);
    if (!e || !e->alive || (s && !s->alive)) return hipErrorInvalidValue;
    fakehip::rt().stream_waits.push_back({fakehip::real(s), e, e->ticket});
    return hipSuccess;
}
inline hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b)
{
    if (!a || !b) return hipErrorInvalidValue;
    *ms = 0.001f * (float)(b->ticket - a->ticket);
    return hipSuccess;
}
