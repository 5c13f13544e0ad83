// A stand-in for the few HIP runtime calls the staging ring makes, for a ThreadSanitizer build of
// the host code without a GPU.  "Device" memory is host memory.  Every stream is a worker thread
// that runs its queue in order, so copies and event waits are as asynchronous as on the real
// runtime and a missing wait shows up as a data race between a reader thread, a copy and a
// "kernel".  A kernel launch is replaced by a queue entry that reads the first source byte and
// writes the first output byte of every piece of the launch: enough for the race detector to see
// which buffers a launch touches.  Nothing here moves tensor data the way the kernels do.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <thread>

#include "fst_internal.h"

namespace {

// Completion counters are atomics: a thread learns that an event completed only by waiting on it
// (acquire), exactly the ordering the real runtime gives.
struct FakeEvent {
    std::atomic<uint64_t> recorded{0}, completed{0};
    void wait_for(uint64_t ticket) const
    {
        while (completed.load(std::memory_order_acquire) < ticket) std::this_thread::sleep_for(std::chrono::microseconds(20));
    }
};

// A stream: one producer (the thread that owns the stager) appends nodes to a linked list, the
// worker follows the list.  The only ordering this creates is submission -> execution; a worker's
// progress is never visible to the producer through the queue (no shared mutex), so the race
// detector is not blinded by orderings the real runtime does not give.
struct FakeStream {
    struct Node {
        std::function<void()> f;
        std::atomic<Node *> next{nullptr};
    };
    Node *tail;                         // producer side
    std::atomic<bool> stop{false};
    std::thread worker;
    FakeStream()
    {
        Node *first = new Node;         // sentinel
        tail = first;
        worker = std::thread([this, first] { run(first); });
    }
    ~FakeStream()
    {
        stop.store(true, std::memory_order_release);
        worker.join();
    }
    void run(Node *at)
    {
        for (;;) {
            Node *n = at->next.load(std::memory_order_acquire);
            if (!n) {
                if (stop.load(std::memory_order_acquire) && !at->next.load(std::memory_order_acquire)) { delete at; return; }
                std::this_thread::sleep_for(std::chrono::microseconds(20));
                continue;
            }
            delete at;
            at = n;
            at->f();
        }
    }
    void push(std::function<void()> f)
    {
        Node *n = new Node;
        n->f = std::move(f);
        tail->next.store(n, std::memory_order_release);
        tail = n;
    }
};

FakeStream *as_stream(hipStream_t s) { return reinterpret_cast<FakeStream *>(s); }
FakeEvent *as_event(hipEvent_t e) { return reinterpret_cast<FakeEvent *>(e); }

}  // namespace

extern "C" {

hipError_t hipHostMalloc(void **p, size_t n, unsigned) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = reinterpret_cast<hipStream_t>(new FakeStream); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { delete as_stream(s); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = reinterpret_cast<hipEvent_t>(new FakeEvent); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete as_event(e); return hipSuccess; }

hipError_t hipEventRecord(hipEvent_t e, hipStream_t s)
{
    FakeEvent *ev = as_event(e);
    const uint64_t ticket = ev->recorded.fetch_add(1, std::memory_order_relaxed) + 1;
    as_stream(s)->push([ev, ticket] {
        uint64_t seen = ev->completed.load(std::memory_order_relaxed);
        while (seen < ticket && !ev->completed.compare_exchange_weak(seen, ticket, std::memory_order_release)) {}
    });
    return hipSuccess;
}

hipError_t hipEventSynchronize(hipEvent_t e)
{
    FakeEvent *ev = as_event(e);
    ev->wait_for(ev->recorded.load(std::memory_order_relaxed));
    return hipSuccess;
}

hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned)
{
    FakeEvent *ev = as_event(e);
    const uint64_t ticket = ev->recorded.load(std::memory_order_relaxed);
    as_stream(s)->push([ev, ticket] { ev->wait_for(ticket); });
    return hipSuccess;
}

hipError_t hipMemcpyAsync(void *dst, const void *src, size_t n, hipMemcpyKind, hipStream_t s)
{
    if (!s) { std::memcpy(dst, src, n); return hipSuccess; }
    as_stream(s)->push([dst, src, n] { std::memcpy(dst, src, n); });
    return hipSuccess;
}

hipError_t hipMemcpy(void *dst, const void *src, size_t n, hipMemcpyKind) { std::memcpy(dst, src, n); return hipSuccess; }

hipError_t hipStreamSynchronize(hipStream_t s)
{
    if (!s) return hipSuccess;
    auto done = std::make_shared<std::atomic<bool>>(false);
    as_stream(s)->push([done] { done->store(true, std::memory_order_release); });
    while (!done->load(std::memory_order_acquire)) std::this_thread::sleep_for(std::chrono::microseconds(20));
    return hipSuccess;
}

const char *hipGetErrorString(hipError_t) { return "fake HIP runtime"; }

}  // extern "C"

namespace fst {

// The launch as the race detector sees it: on the launch's stream, one read per piece from the
// source buffer and one write per piece to its output.
int launch_class_kernels(uint32_t, const DevDesc *descs_dev, const uint32_t *, uint32_t n_tiles, uint32_t, const void *raw_dev,
                         void *stream)
{
    if (n_tiles == 0) return FST_OK;
    const uint8_t *raw = static_cast<const uint8_t *>(raw_dev);
    auto touch = [descs_dev, n_tiles, raw] {
        uint32_t tiles = 0;
        for (const DevDesc *d = descs_dev; tiles < n_tiles; ++d) {
            *reinterpret_cast<volatile uint8_t *>(d->dst) = *reinterpret_cast<const volatile uint8_t *>(raw + d->src_off);
            tiles += d->n_tiles;
        }
    };
    if (stream) as_stream(static_cast<hipStream_t>(stream))->push(touch); else touch();
    return FST_OK;
}

}  // namespace fst
