// The entry point with the built-in device workspace needs device code: absent from CPU builds.
#include "fst_internal.h"
extern "C" int fst_materialize_static(const void *, size_t, const fst_plan *, size_t, void *const *, void *) { return FST_E_HIP; }
