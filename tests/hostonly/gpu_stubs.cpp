// Stand-ins for the entry points that need a GPU, so that the host parts of the library (header
// parser, load planner) link alone for a sanitizer build.  Every one reports FST_E_HIP.
#include "fst_internal.h"

extern "C" {
int fst_prepare(const fst_plan *, size_t, int32_t, size_t, void *const *, void *, size_t, void *) { return FST_E_HIP; }
int fst_launch(const fst_plan *, size_t, const void *, size_t, void *) { return FST_E_HIP; }
int fst_materialize(const void *, size_t, const fst_plan *, size_t, void *const *, void *, size_t, void *) { return FST_E_HIP; }
int fst_materialize_static(const void *, size_t, const fst_plan *, size_t, void *const *, void *) { return FST_E_HIP; }
int fst_materialize_slot(const void *, size_t, const fst_plan *, size_t, void *const *, void *, size_t, void *) { return FST_E_HIP; }
int fst_stager_create(const fst_stager_config *, fst_stager **) { return FST_E_HIP; }
void fst_stager_destroy(fst_stager *) {}
int fst_read_fds(void *, int32_t, uint64_t, void *, uint64_t) { return -1; }
int fst_stage_resident(fst_stager *, const fst_plan *, fst_read_fn, void *, void *, size_t, void *const *, void *, size_t,
                       uint32_t, fst_stage_stats *) { return FST_E_HIP; }
int fst_stage_packed(fst_stager *, const fst_plan *, fst_read_fn, void *, void *, size_t, void *const *, void *, size_t,
                     uint32_t, fst_stage_stats *) { return FST_E_HIP; }
int fst_stage_streamed(fst_stager *, const fst_plan *, fst_read_fn, void *, void *const *, size_t, size_t, void *const *,
                       void *, size_t, uint32_t, fst_stage_stats *) { return FST_E_HIP; }
}
