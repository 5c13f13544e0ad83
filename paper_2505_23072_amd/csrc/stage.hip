// Pinned-host staging ring (paper Section III-A: the path without GPUDirect Storage reads file
// blocks into a small DMA-able bounce buffer in host memory and copies them to the GPU from
// there; Section IV: up to 16 I/O threads, 160 MB of bounce buffer each).
//
// Reader threads fill ring slots, several threads per slot (a block is read in parts, so a slot
// is full after a fraction of the time one thread would need, while the copy out of it stays one
// large transfer); the calling thread is the only one that enqueues GPU work (reader threads only
// wait, with hipEventSynchronize, for the copy out of the ring slot they are about to refill): it
// issues one hipMemcpyAsync per filled slot on the copy stream, in block order, and as soon as
// the last block of a group is queued it makes the compute stream wait for that copy and queues
// the group's kernels.  Kernels of group g therefore run while the bytes of group g+1 are still
// crossing PCIe.  For checkpoints larger than device memory the raw buffer is itself a ring of
// device slots; a slot is overwritten only after the kernels of its previous group are done.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cerrno>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <unistd.h>

#include "fst_internal.h"

struct fst_stager {
    uint32_t n_slots = 0, n_threads = 0;
    uint64_t slot_bytes = 0;
    uint8_t *pinned = nullptr;
    hipStream_t copy = nullptr, compute = nullptr;
    std::vector<hipEvent_t> slot_done;      // copy out of ring slot s has finished
    std::vector<hipEvent_t> events;         // pool for group events
};

namespace fst {
namespace {

#define HIP_TRY(call)                                                                   \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess) return fail(FST_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

struct Block {
    uint32_t group, file;
    uint64_t off, len;       // plain: file range [off, off+len).  Compacted: bytes [skip, skip+len) of the image of
    uint64_t row_bytes;      //   the rows of row_bytes bytes that start at file offsets off, off+stride, ...
    uint64_t stride, skip;   //   (stride 0 = plain)
    uint8_t *dst;            // device address
    bool first, last;        // of its group
};

// A block is read in parts of part_bytes by whichever reader thread comes next.
struct Part {
    uint32_t block;
    uint64_t off, len;       // inside the block
};

struct Shared {
    std::mutex mu;
    std::condition_variable cv;
    std::vector<uint8_t> filled, issued;
    std::vector<uint32_t> parts_left;        // per block, guarded by mu
    bool abort = false;
    int status = FST_OK;
    std::atomic<size_t> next{0};
    std::atomic<uint64_t> read_ns{0};
};

double now_s()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

int ensure_events(fst_stager *s, size_t n)
{
    while (s->events.size() < n) {
        hipEvent_t ev;
        HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        s->events.push_back(ev);
    }
    return FST_OK;
}

void reader(fst_stager *s, const std::vector<Block> *blocks, const std::vector<Part> *parts, Shared *sh,
            fst_read_fn read, void *ctx, bool skip_read)
{
    const size_t n = parts->size();
    for (;;) {
        const size_t k = sh->next.fetch_add(1);
        if (k >= n) return;
        const Part &pt = (*parts)[k];
        const size_t i = pt.block;
        const uint32_t slot = uint32_t(i % s->n_slots);
        if (i >= s->n_slots) {
            // the slot's previous block must have been copied out
            {
                std::unique_lock<std::mutex> lk(sh->mu);
                sh->cv.wait(lk, [&] { return sh->abort || sh->issued[i - s->n_slots]; });
                if (sh->abort) return;
            }
            if (hipEventSynchronize(s->slot_done[slot]) != hipSuccess) {
                std::lock_guard<std::mutex> lk(sh->mu);
                sh->abort = true;
                sh->status = fail(FST_E_HIP, "hipEventSynchronize failed in a reader");
                sh->cv.notify_all();
                return;
            }
        }
        const Block &b = (*blocks)[i];
        int rc = 0;
        if (!skip_read) {
            const auto t0 = std::chrono::steady_clock::now();
            uint8_t *to = s->pinned + uint64_t(slot) * s->slot_bytes + pt.off;
            if (b.stride == 0) {
                rc = read(ctx, int32_t(b.file), b.off + pt.off, to, pt.len);
            } else {
                // compacted rows: one read per row segment, back to back into the ring slot
                uint64_t pos = b.skip + pt.off, left = pt.len;
                while (left && !rc) {
                    const uint64_t r = pos / b.row_bytes, col = pos - r * b.row_bytes;
                    const uint64_t n = std::min(b.row_bytes - col, left);
                    rc = read(ctx, int32_t(b.file), b.off + r * b.stride + col, to, n);
                    to += n;
                    pos += n;
                    left -= n;
                }
            }
            sh->read_ns += uint64_t(std::chrono::duration_cast<std::chrono::nanoseconds>(
                                        std::chrono::steady_clock::now() - t0).count());
        }
        std::lock_guard<std::mutex> lk(sh->mu);
        if (rc) {
            sh->abort = true;
            sh->status = fail(FST_E_IO, "read of file %u at %llu (+%llu) failed", b.file,
                              (unsigned long long)(b.off + pt.off), (unsigned long long)pt.len);
        }
        if (--sh->parts_left[i] == 0 || rc) {
            sh->filled[i] = 1;
            sh->cv.notify_all();
        }
        if (rc) return;
    }
}

int stage_impl(fst_stager *s, const fst_plan *p, fst_read_fn read, void *ctx, int layout, void *raw_dev, size_t raw_len,
               void *const *slot_dev, size_t n_dev_slots, size_t dev_slot_bytes, void *const *out_ptrs, void *ws,
               size_t ws_len, uint32_t flags, fst_stage_stats *stats)
{
    const bool streamed = layout == FST_LAYOUT_SLOT;
    const bool packed = layout == FST_LAYOUT_PACKED;
    const bool kernels = !(flags & FST_STAGE_NO_KERNELS);
    const bool skip_read = (flags & FST_STAGE_NO_READ) != 0;
    if (!s || !p) return fail(FST_E_ARG, "fst_stage: NULL argument");
    if (!read && !skip_read) return fail(FST_E_ARG, "fst_stage: no read callback");
    if (kernels && !out_ptrs && !p->outputs.empty()) return fail(FST_E_ARG, "fst_stage: out_ptrs is NULL");
    if (layout == FST_LAYOUT_RESIDENT && p->has_compact)
        return fail(FST_E_ARG, "the plan's groups stage compacted rows: use the streamed or the packed load");
    if (packed && raw_len < p->packed_bytes)
        return fail(FST_E_RANGE, "the packed buffer has %zu bytes, the plan needs %llu", raw_len,
                    (unsigned long long)p->packed_bytes);
    const size_t ng = p->groups.size();
    const double t_start = now_s();

    // device tables of every group, uploaded once before any copy is queued
    std::vector<TableImage> images(kernels ? ng : 0);
    std::vector<size_t> table_at(ng, 0);
    std::vector<uint8_t> all;
    for (size_t g = 0; g < ng; ++g) {
        const Group &gr = p->groups[g];
        if (streamed) {
            const uint64_t need = gr.slot_bytes;
            if (need > dev_slot_bytes)
                return fail(FST_E_RANGE, "group %zu needs %llu bytes, device slots have %zu", g,
                            (unsigned long long)need, dev_slot_bytes);
            if (!slot_dev[g % n_dev_slots] || reinterpret_cast<uintptr_t>(slot_dev[g % n_dev_slots]) % FST_RAW_ALIGN)
                return fail(FST_E_ALIGN, "device slot %zu is NULL or not %d-byte aligned", g % n_dev_slots, FST_RAW_ALIGN);
        } else if (!packed && p->raw_base[gr.file] + gr.hi > raw_len) {
            return fail(FST_E_RANGE, "group %zu ends at byte %llu of a raw buffer of %zu", g,
                        (unsigned long long)(p->raw_base[gr.file] + gr.hi), raw_len);
        }
        if (kernels) {
            if (int rc = build_image(p, g, g + 1, out_ptrs, streamed ? dev_slot_bytes : raw_len, layout, images[g]))
                return rc;
            table_at[g] = all.size();                       // blobs are whole multiples of 256 bytes
            all.insert(all.end(), images[g].blob.begin(), images[g].blob.end());
        }
    }
    if (!streamed) {
        if (!raw_dev || reinterpret_cast<uintptr_t>(raw_dev) % FST_RAW_ALIGN)
            return fail(FST_E_ALIGN, "%s buffer is NULL or not %d-byte aligned", packed ? "packed" : "raw", FST_RAW_ALIGN);
    }
    if (kernels && !all.empty()) {
        if (!ws || reinterpret_cast<uintptr_t>(ws) % 256) return fail(FST_E_ALIGN, "workspace is NULL or not 256-byte aligned");
        if (ws_len < all.size())
            return fail(FST_E_RANGE, "workspace has %zu bytes, %zu needed", ws_len, all.size());
        HIP_TRY(hipMemcpy(ws, all.data(), all.size(), hipMemcpyHostToDevice));
    }

    // cut the groups' staged extents into blocks of at most one ring slot
    std::vector<Block> blocks;
    for (size_t g = 0; g < ng; ++g) {
        const Group &gr = p->groups[g];
        const size_t first_block = blocks.size();
        for (const Extent &ex : gr.extents) {
            uint8_t *base = streamed ? static_cast<uint8_t *>(slot_dev[g % n_dev_slots]) + ex.slot_off
                            : packed ? static_cast<uint8_t *>(raw_dev) + gr.packed_off + ex.slot_off
                                     : static_cast<uint8_t *>(raw_dev) + p->raw_base[gr.file] + ex.lo;
            const uint64_t image = ex.image_bytes();
            for (uint64_t o = 0; o < image; o += s->slot_bytes) {
                const uint64_t len = std::min<uint64_t>(s->slot_bytes, image - o);
                if (ex.compact())
                    blocks.push_back(Block{uint32_t(g), gr.file, ex.lo, len, ex.row_bytes, ex.stride, o, base + o, false, false});
                else
                    blocks.push_back(Block{uint32_t(g), gr.file, ex.lo + o, len, 0, 0, 0, base + o, false, false});
            }
        }
        if (blocks.size() > first_block) {
            blocks[first_block].first = true;
            blocks.back().last = true;
        }
    }
    const size_t nb = blocks.size();
    if (int rc = ensure_events(s, streamed ? n_dev_slots + 1 : 1)) return rc;

    // parts of a sixteenth of a slot (4 KiB .. 8 MiB): the threads fill one slot together
    const uint64_t part_bytes = std::min<uint64_t>(std::max<uint64_t>((s->slot_bytes / 16 + 4095) / 4096 * 4096, 4096), 8ull << 20);
    std::vector<Part> parts;
    Shared sh;
    sh.filled.assign(nb, 0);
    sh.issued.assign(nb, 0);
    sh.parts_left.assign(nb, 0);
    for (size_t i = 0; i < nb; ++i)
        for (uint64_t o = 0; o < blocks[i].len; o += part_bytes) {
            parts.push_back(Part{uint32_t(i), o, std::min<uint64_t>(part_bytes, blocks[i].len - o)});
            ++sh.parts_left[i];
        }
    std::vector<std::thread> threads;
    const uint32_t nt = uint32_t(std::min<size_t>(s->n_threads, std::max<size_t>(parts.size(), 1)));
    int status = FST_OK;
    try {
        threads.reserve(nt);
        for (uint32_t t = 0; t < nt; ++t) threads.emplace_back(reader, s, &blocks, &parts, &sh, read, ctx, skip_read);
    } catch (...) {
        // a thread could not be started: stop the ones that run, report, copy nothing
        status = fail(FST_E_NOMEM, "could not start %u reader threads", nt);
    }

    uint64_t staged = 0;
    hipEvent_t ready = s->events[0];
    for (size_t i = 0; i < nb && status == FST_OK; ++i) {
        {
            std::unique_lock<std::mutex> lk(sh.mu);
            sh.cv.wait(lk, [&] { return sh.abort || sh.filled[i]; });
            if (sh.abort) { status = sh.status ? sh.status : FST_E_IO; break; }
        }
        const Block &b = blocks[i];
        const uint32_t slot = uint32_t(i % s->n_slots);
        hipError_t e = hipSuccess;
        if (streamed && b.first && b.group >= n_dev_slots && kernels)
            e = hipStreamWaitEvent(s->copy, s->events[1 + b.group % n_dev_slots], 0);   // slot's old group done
        if (e == hipSuccess)
            e = hipMemcpyAsync(b.dst, s->pinned + uint64_t(slot) * s->slot_bytes, b.len, hipMemcpyHostToDevice, s->copy);
        if (e == hipSuccess) e = hipEventRecord(s->slot_done[slot], s->copy);
        if (e != hipSuccess) { status = fail(FST_E_HIP, "staging copy failed: %s", hipGetErrorString(e)); break; }
        staged += b.len;
        {
            std::lock_guard<std::mutex> lk(sh.mu);
            sh.issued[i] = 1;
        }
        sh.cv.notify_all();
        if (b.last && kernels) {
            e = hipEventRecord(ready, s->copy);
            if (e == hipSuccess) e = hipStreamWaitEvent(s->compute, ready, 0);
            if (e != hipSuccess) { status = fail(FST_E_HIP, "stream hand-over failed: %s", hipGetErrorString(e)); break; }
            const void *src = streamed ? slot_dev[b.group % n_dev_slots] : raw_dev;
            status = launch_ranges(images[b.group], static_cast<const uint8_t *>(ws) + table_at[b.group], src,
                                   s->compute);
            if (status == FST_OK && streamed) {
                e = hipEventRecord(s->events[1 + b.group % n_dev_slots], s->compute);
                if (e != hipSuccess) status = fail(FST_E_HIP, "hipEventRecord failed: %s", hipGetErrorString(e));
            }
        }
    }
    if (status != FST_OK) {
        std::lock_guard<std::mutex> lk(sh.mu);
        sh.abort = true;
        sh.cv.notify_all();
    }
    for (auto &t : threads) t.join();
    // everything queued must drain before buffers may be reused or freed
    hipError_t e1 = hipStreamSynchronize(s->copy), e2 = hipStreamSynchronize(s->compute);
    if (status == FST_OK && (e1 != hipSuccess || e2 != hipSuccess))
        status = fail(FST_E_HIP, "stream synchronisation failed: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2));
    if (stats) {
        stats->staged_bytes = staged;
        stats->n_copies = nb;
        stats->seconds_total = now_s() - t_start;
        stats->seconds_read = double(sh.read_ns.load()) * 1e-9;
    }
    return status;
}

}  // namespace
}  // namespace fst

using namespace fst;

extern "C" {

static int stager_create_impl(const fst_stager_config *cfg, fst_stager **out)
{
    if (!out) return fail(FST_E_ARG, "fst_stager_create: out is NULL");
    *out = nullptr;
    fst_stager *s = new (std::nothrow) fst_stager;
    if (!s) return fail(FST_E_NOMEM, "out of memory");
    s->n_slots = cfg && cfg->n_slots ? cfg->n_slots : 8;
    s->n_threads = cfg && cfg->n_threads ? cfg->n_threads : 8;
    s->slot_bytes = cfg && cfg->slot_bytes ? cfg->slot_bytes : (64ull << 20);
    if (s->n_slots > 1024 || s->n_threads > 256 || s->slot_bytes % 256 || s->slot_bytes > (4ull << 30)) {
        delete s;
        return fail(FST_E_ARG, "stager config out of range (slots <= 1024, threads <= 256, slot_bytes %% 256 == 0)");
    }
    auto cleanup = [&](const char *what, hipError_t e) {
        fst_stager_destroy(s);
        return fail(FST_E_HIP, "%s: %s", what, hipGetErrorString(e));
    };
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&s->pinned), size_t(s->n_slots) * s->slot_bytes, hipHostMallocDefault);
    if (e != hipSuccess) { s->pinned = nullptr; return cleanup("hipHostMalloc", e); }
    if ((e = hipStreamCreateWithFlags(&s->copy, hipStreamNonBlocking)) != hipSuccess) return cleanup("hipStreamCreate", e);
    if ((e = hipStreamCreateWithFlags(&s->compute, hipStreamNonBlocking)) != hipSuccess) return cleanup("hipStreamCreate", e);
    try {
        s->slot_done.reserve(s->n_slots);
    } catch (...) {
        fst_stager_destroy(s);
        throw;
    }
    for (uint32_t i = 0; i < s->n_slots; ++i) {
        hipEvent_t ev;
        if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return cleanup("hipEventCreate", e);
        s->slot_done.push_back(ev);         // reserved above: cannot throw
    }
    *out = s;
    return FST_OK;
}

int fst_stager_create(const fst_stager_config *cfg, fst_stager **out)
{
    try {
        return stager_create_impl(cfg, out);
    } catch (const std::bad_alloc &) {
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

void fst_stager_destroy(fst_stager *s)
{
    if (!s) return;
    for (hipEvent_t ev : s->slot_done) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : s->events) (void)hipEventDestroy(ev);
    if (s->copy) (void)hipStreamDestroy(s->copy);
    if (s->compute) (void)hipStreamDestroy(s->compute);
    if (s->pinned) (void)hipHostFree(s->pinned);
    delete s;
}

int fst_read_fds(void *ctx, int32_t file, uint64_t off, void *dst, uint64_t len)
{
    const int fd = static_cast<const int *>(ctx)[file];
    uint8_t *d = static_cast<uint8_t *>(dst);
    uint64_t done = 0;
    while (done < len) {
        const ssize_t r = pread(fd, d + done, len - done, off_t(off + done));
        if (r < 0) { if (errno == EINTR) continue; return -1; }
        if (r == 0) return -1;      // file shorter than its header says
        done += uint64_t(r);
    }
    return 0;
}

int fst_stage_resident(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx, void *raw_dev,
                       size_t raw_len, void *const *out_ptrs, void *dev_workspace, size_t workspace_len,
                       uint32_t flags, fst_stage_stats *stats)
{
    try {
        return stage_impl(s, p, read, read_ctx, FST_LAYOUT_RESIDENT, raw_dev, raw_len, nullptr, 0, 0, out_ptrs,
                          dev_workspace, workspace_len, flags, stats);
    } catch (const std::bad_alloc &) {
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

int fst_stage_packed(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx, void *packed_dev,
                     size_t packed_len, void *const *out_ptrs, void *dev_workspace, size_t workspace_len,
                     uint32_t flags, fst_stage_stats *stats)
{
    try {
        return stage_impl(s, p, read, read_ctx, FST_LAYOUT_PACKED, packed_dev, packed_len, nullptr, 0, 0, out_ptrs,
                          dev_workspace, workspace_len, flags, stats);
    } catch (const std::bad_alloc &) {
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

int fst_stage_streamed(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx, void *const *slot_dev,
                       size_t n_dev_slots, size_t dev_slot_bytes, void *const *out_ptrs, void *dev_workspace,
                       size_t workspace_len, uint32_t flags, fst_stage_stats *stats)
{
    if (!slot_dev || n_dev_slots == 0) return fail(FST_E_ARG, "fst_stage_streamed: no device slots");
    try {
        return stage_impl(s, p, read, read_ctx, FST_LAYOUT_SLOT, nullptr, 0, slot_dev, n_dev_slots, dev_slot_bytes,
                          out_ptrs, dev_workspace, workspace_len, flags, stats);
    } catch (const std::bad_alloc &) {
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

}  // extern "C"
