// fst_materialize_static: fst_materialize for callers that cannot allocate device memory.  The
// piece and hint tables, which fst_materialize puts into a workspace the caller allocates, go into
// a device array that is part of the library's code object, so no allocation happens anywhere on
// the way: the call builds the table on the host, copies it into the array and launches the same
// kernels with the array's address.
#include <hip/hip_runtime.h>

#include <mutex>

#include "fst_internal.h"

namespace {

// One copy per GPU that loads the library, held until the process ends.
static __device__ __align__(256) unsigned char scratch[FST_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};      // the array's device address, per device ordinal

// The address of `scratch` on the current device.  In host code the array's name is only a
// handle for this lookup, never an address to hand to a kernel or a copy.
int scratch_address(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fst::fail(FST_E_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fst::fail(FST_E_RANGE, "device ordinal %d is beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fst::fail(FST_E_HIP, "hipGetSymbolAddress(built-in workspace): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FST_OK;
}

}  // namespace

extern "C" int fst_materialize_static(const void *raw_dev, size_t raw_len, const fst_plan *p, size_t group,
                                      void *const *out_ptrs, void *stream)
{
    try {
        if (!p) return fst::fail(FST_E_ARG, "fst_materialize_static: plan is NULL");
        // the size the tables of this call take is known from the plan alone: refuse before anything is enqueued
        size_t need = 0, g0 = group, g1 = group + 1;
        if (group == FST_ALL_GROUPS) { g0 = 0; g1 = p->groups.size(); }
        else if (group >= p->groups.size()) return fst::fail(FST_E_RANGE, "group %zu out of range", group);
        size_t n_pieces = 0, n_hints = 0;
        for (size_t g = g0; g < g1; ++g) {
            n_pieces += p->groups[g].pieces.size();
            n_hints += p->groups[g].hint_bound;
        }
        need = fst::table_bytes(n_pieces, n_hints);
        if (n_pieces && need > FST_STATIC_WORKSPACE_BYTES)
            return fst::fail(FST_E_RANGE, "the tables of this call may take %zu bytes, the built-in workspace holds %u: "
                                          "pass fewer groups per call or use fst_materialize with a workspace of your own",
                             need, unsigned(FST_STATIC_WORKSPACE_BYTES));
        void *ws = nullptr;
        if (int rc = scratch_address(&ws)) return rc;
        return fst::materialize_into(raw_dev, raw_len, p, group, out_ptrs, ws, FST_STATIC_WORKSPACE_BYTES, stream,
                                     FST_LAYOUT_RESIDENT, true);
    } catch (const std::bad_alloc &) {
        return fst::fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fst::fail(FST_E_ARG, "unexpected internal error");
    }
}
