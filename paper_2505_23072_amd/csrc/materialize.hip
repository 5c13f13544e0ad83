// Host side of fst_materialize: checks the operands against what the kernels assume, builds the
// device table of pieces for one group (or all), copies it into the caller's workspace and
// launches one kernel per launch class (paper Section III-B: preprocessing offloaded to the GPU).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>

#include "fst_internal.h"

namespace fst {

namespace {

uint32_t tiles_of(const Piece &pc)
{
    const uint64_t per = tile_units(pc.path);
    return uint32_t((pc.n_units + per - 1) / per);
}

// Multiplier m and shift s with floor(n / d) == umulhi(2n, m) >> s for every n < 2^31, d in
// [1, 2^31]: s = ceil(log2 d), m = ceil(2^(31+s) / d).  m*d exceeds 2^(31+s) by e < d <= 2^s, so
// n*m / 2^(31+s) exceeds n/d by n*e / (d * 2^(31+s)) < 1/d, too little to reach the next integer.
void division_magic(uint32_t d, uint32_t &m, uint32_t &s)
{
    s = 0;
    while ((uint64_t(1) << s) < d) ++s;
    m = uint32_t(((uint64_t(1) << (31 + s)) + d - 1) / d);
}

}  // namespace

// Builds the device image for groups [g0, g1) as ONE launch set (pieces of all those groups
// merged per class).  In the slot layout (group g0 alone) and in the packed layout a piece's bytes
// are found through the extent that holds them.
int build_image(const fst_plan *p, size_t g0, size_t g1, void *const *out_ptrs, size_t src_len, int layout,
                TableImage &image)
{
    std::vector<DevDesc> &descs = image.descs;
    std::vector<LaunchRange> &ranges = image.ranges;
    struct Ref { const Piece *pc; const Group *gr; };
    std::vector<Ref> order;
    for (size_t g = g0; g < g1; ++g)
        for (const Piece &pc : p->groups[g].pieces) order.push_back({&pc, &p->groups[g]});
    std::stable_sort(order.begin(), order.end(),
                     [](const Ref &a, const Ref &b) { return launch_class(*a.pc) < launch_class(*b.pc); });
    descs.clear();
    ranges.clear();
    image.hints.clear();
    descs.reserve(order.size());
    for (const Ref &ref : order) {
        const Piece *pc = ref.pc;
        const Output &o = p->outputs[pc->output];
        const uintptr_t out = reinterpret_cast<uintptr_t>(out_ptrs[pc->output]);
        if (out == 0) return fail(FST_E_ARG, "out_ptrs[%u] is NULL but the output has %llu bytes", pc->output,
                                  (unsigned long long)o.info.nbytes);
        if (out % FST_OUTPUT_ALIGN)
            return fail(FST_E_ALIGN, "out_ptrs[%u] is not %d-byte aligned", pc->output, FST_OUTPUT_ALIGN);
        uint64_t src_off;
        if (layout == FST_LAYOUT_RESIDENT) {
            if (pc->compact)
                return fail(FST_E_ARG, "the plan's groups stage compacted rows: use the slot or the packed layout");
            src_off = p->raw_base[o.info.file] + pc->src_file_off;
        } else {
            if (pc->extent >= ref.gr->extents.size()) return fail(FST_E_ARG, "output %u: no staged extent", pc->output);
            const Extent &ex = ref.gr->extents[pc->extent];
            // a piece over a compacted extent is laid out over the extent's image; others sit at their file offset
            const uint64_t inside = pc->compact ? pc->src_file_off : pc->src_file_off - ex.lo;
            if ((!pc->compact && (pc->src_file_off < ex.lo || pc->src_file_off + pc->src_span > ex.hi)) ||
                (pc->compact && inside + pc->src_span > ex.image_bytes()))
                return fail(FST_E_RANGE, "output %u: source bytes are not inside their staged extent", pc->output);
            src_off = (layout == FST_LAYOUT_PACKED ? ref.gr->packed_off : 0) + ex.slot_off + inside;
        }
        // the kernels read whole dwords around unaligned bytes: round the end up to 4
        const uint64_t end = (src_off + pc->src_span + 3) & ~uint64_t(3);
        if (end > ((uint64_t(src_len) + 3) & ~uint64_t(3)))
            return fail(FST_E_RANGE, "output %u reads bytes [%llu, %llu) but the buffer has %zu", pc->output,
                        (unsigned long long)src_off, (unsigned long long)(src_off + pc->src_span), src_len);
        const uint32_t cls = launch_class(*pc);
        if (ranges.empty() || ranges.back().cls != cls) ranges.push_back({cls, uint32_t(descs.size()), 0, 0, 0, 0});
        LaunchRange &r = ranges.back();
        DevDesc d{};
        d.src_off = src_off;
        d.src_stride = pc->src_stride;
        d.dst = uint64_t(out) + pc->dst_off;
        d.n_units = pc->n_units;
        d.units_per_row = pc->units_per_row;
        d.unit0 = pc->unit0;
        d.grain = pc->grain;
        d.staged = pc->staged ? 1u : 0u;
        d.tile0 = r.tiles;
        d.n_tiles = tiles_of(*pc);
        if (pc->path != PATH_ELEM && pc->units_per_row) division_magic(pc->units_per_row, d.div_m, d.div_s);
        if (uint64_t(r.tiles) + d.n_tiles > 0x7FFFFFFFull) return fail(FST_E_RANGE, "too many tiles in one launch");
        r.tiles += d.n_tiles;
        r.count += 1;
        descs.push_back(d);
    }
    // hints: for every span of 2^hint_shift tiles of a launch, the piece (counted from the launch's
    // first) that holds the span's first tile, and one more entry naming the launch's last piece.  The
    // table runs on over the tile indices that the launch's last workgroup has beyond the last tile:
    // they lead to the last piece, where a wavefront sees that its tile lies past the piece's end.
    // (A table of pairs -- the owners of a span's first and last tile, which would spare small
    // tensors that fill their spans exactly the one search step -- measured 6 to 11 % slower on large
    // tensors.)
    for (LaunchRange &r : ranges) {
        r.hint_first = uint32_t(image.hints.size());
        r.hint_shift = hint_shift_for(r.tiles, r.count);
        const uint32_t padded = workgroups_of(class_path(r.cls), r.tiles) * (class_path(r.cls) == PATH_ELEM ? 1 : WG_TILES);
        const uint32_t span = 1u << r.hint_shift;
        uint32_t at = 0;                            // the last piece that starts at or before the span's first tile
        for (uint32_t t = 0; t < padded; t += span) {
            while (at + 1 < r.count && descs[r.first + at + 1].tile0 <= t) ++at;
            image.hints.push_back(at);
        }
        image.hints.push_back(r.count - 1);
    }
    // one blob for the upload: pieces, then hints on a 256-byte boundary
    image.blob.assign(table_bytes(descs.size(), image.hints.size()), 0);
    if (!descs.empty()) std::memcpy(image.blob.data(), descs.data(), descs.size() * sizeof(DevDesc));
    if (!image.hints.empty())
        std::memcpy(image.blob.data() + table_hint_offset(descs.size()), image.hints.data(),
                    image.hints.size() * sizeof(uint32_t));
    return FST_OK;
}

int launch_ranges(const TableImage &image, const void *table_dev, const void *src_dev, void *stream)
{
    const DevDesc *descs = static_cast<const DevDesc *>(table_dev);
    const uint32_t *hints = reinterpret_cast<const uint32_t *>(static_cast<const uint8_t *>(table_dev) +
                                                               table_hint_offset(image.descs.size()));
    for (const LaunchRange &r : image.ranges)
        if (int rc = launch_class_kernels(r.cls, descs + r.first, hints + r.hint_first, r.tiles, r.hint_shift, src_dev, stream))
            return rc;
    return FST_OK;
}

namespace {

int group_range(const fst_plan *p, size_t group, int layout, size_t &g0, size_t &g1)
{
    if (group == FST_ALL_GROUPS) {
        if (layout == FST_LAYOUT_SLOT) return fail(FST_E_ARG, "the slot layout takes one group at a time");
        g0 = 0;
        g1 = p->groups.size();
    } else {
        if (group >= p->groups.size()) return fail(FST_E_RANGE, "group %zu out of range", group);
        g0 = group;
        g1 = group + 1;
    }
    return FST_OK;
}

// Builds the group's table and enqueues its upload into the workspace.  Caller holds image_mu.
int prepare_locked(const fst_plan *p, size_t group, int layout, size_t src_len, void *const *out_ptrs, void *ws,
                   size_t ws_len, void *stream, bool builtin = false)
{
    size_t g0, g1;
    if (int rc = group_range(p, group, layout, g0, g1)) return rc;
    TableImage &image = (builtin ? p->builtin_images : p->images)[group];
    image.dev = nullptr;
    size_t n_pieces = 0;
    for (size_t g = g0; g < g1; ++g) n_pieces += p->groups[g].pieces.size();
    if (n_pieces == 0) {                       // nothing to launch: prepared, with an empty table
        image = TableImage{};
        image.prepared = true;
        return FST_OK;
    }
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256) return fail(FST_E_ALIGN, "workspace is NULL or not 256-byte aligned");
    if (int rc = build_image(p, g0, g1, out_ptrs, src_len, layout, image)) return rc;
    if (ws_len < image.blob.size())
        return fail(FST_E_RANGE, "workspace has %zu bytes, %zu needed", ws_len, image.blob.size());
    hipError_t e = hipMemcpyAsync(ws, image.blob.data(), image.blob.size(), hipMemcpyHostToDevice,
                                  static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FST_E_HIP, "table upload failed: %s", hipGetErrorString(e));
    image.dev = ws;
    image.src_len = src_len;
    image.prepared = true;
    return FST_OK;
}

// Enqueues the kernels of a prepared group.  Caller holds image_mu.
int launch_locked(const fst_plan *p, size_t group, const void *src_dev, size_t src_len, void *stream,
                  bool builtin = false)
{
    const std::map<size_t, TableImage> &images = builtin ? p->builtin_images : p->images;
    auto it = images.find(group);
    if (it == images.end() || !it->second.prepared)
        return fail(FST_E_ARG, "group %zu has no uploaded table: call fst_prepare first", group);
    const TableImage &image = it->second;
    if (image.ranges.empty()) return FST_OK;
    if (!src_dev) return fail(FST_E_ARG, "source buffer is NULL");
    if (reinterpret_cast<uintptr_t>(src_dev) % FST_RAW_ALIGN)
        return fail(FST_E_ALIGN, "source buffer is not %d-byte aligned", FST_RAW_ALIGN);
    if (src_len < image.src_len)
        return fail(FST_E_RANGE, "source buffer has %zu bytes, the table was prepared for %zu", src_len, image.src_len);
    return launch_ranges(image, image.dev, src_dev, stream);
}

}  // namespace

int materialize_into(const void *src_dev, size_t src_len, const fst_plan *p, size_t group, void *const *out_ptrs,
                     void *ws, size_t ws_len, void *stream, int layout, bool builtin)
{
    if (!p || (!out_ptrs && !p->outputs.empty())) return fail(FST_E_ARG, "fst_materialize: NULL argument");
    std::lock_guard<std::mutex> lock(p->image_mu);
    if (int rc = prepare_locked(p, group, layout, src_len, out_ptrs, ws, ws_len, stream, builtin)) return rc;
    return launch_locked(p, group, src_dev, src_len, stream, builtin);
}

}  // namespace fst

using namespace fst;

#define FST_GUARD(expr)                                              \
    try { return (expr); }                                           \
    catch (const std::bad_alloc &) { return fail(FST_E_NOMEM, "out of memory"); } \
    catch (...) { return fail(FST_E_ARG, "unexpected internal error"); }

namespace {

int prepare_impl(const fst_plan *p, size_t group, int32_t layout, size_t src_len, void *const *out_ptrs, void *ws,
                 size_t ws_len, void *stream)
{
    if (!p || (!out_ptrs && !p->outputs.empty())) return fail(FST_E_ARG, "fst_prepare: NULL argument");
    if (layout != FST_LAYOUT_RESIDENT && layout != FST_LAYOUT_SLOT && layout != FST_LAYOUT_PACKED)
        return fail(FST_E_ARG, "fst_prepare: unknown layout %d", layout);
    std::lock_guard<std::mutex> lock(p->image_mu);
    return prepare_locked(p, group, layout, src_len, out_ptrs, ws, ws_len, stream);
}

int launch_impl(const fst_plan *p, size_t group, const void *src_dev, size_t src_len, void *stream)
{
    if (!p) return fail(FST_E_ARG, "fst_launch: plan is NULL");
    std::lock_guard<std::mutex> lock(p->image_mu);
    return launch_locked(p, group, src_dev, src_len, stream);
}

int materialize_impl(const void *src_dev, size_t src_len, const fst_plan *p, size_t group, void *const *out_ptrs,
                     void *ws, size_t ws_len, void *stream, int layout)
{
    return materialize_into(src_dev, src_len, p, group, out_ptrs, ws, ws_len, stream, layout, false);
}

}  // namespace

extern "C" {

int fst_prepare(const fst_plan *p, size_t group, int32_t layout, size_t src_len, void *const *out_ptrs,
                void *dev_workspace, size_t workspace_len, void *stream)
{
    FST_GUARD(prepare_impl(p, group, layout, src_len, out_ptrs, dev_workspace, workspace_len, stream));
}

int fst_launch(const fst_plan *p, size_t group, const void *src_dev, size_t src_len, void *stream)
{
    FST_GUARD(launch_impl(p, group, src_dev, src_len, stream));
}

int fst_materialize(const void *raw_dev, size_t raw_len, const fst_plan *p, size_t group, void *const *out_ptrs,
                    void *dev_workspace, size_t workspace_len, void *stream)
{
    FST_GUARD(materialize_impl(raw_dev, raw_len, p, group, out_ptrs, dev_workspace, workspace_len, stream, FST_LAYOUT_RESIDENT));
}

int fst_materialize_slot(const void *slot_dev, size_t slot_len, const fst_plan *p, size_t group,
                         void *const *out_ptrs, void *dev_workspace, size_t workspace_len, void *stream)
{
    FST_GUARD(materialize_impl(slot_dev, slot_len, p, group, out_ptrs, dev_workspace, workspace_len, stream, FST_LAYOUT_SLOT));
}

}  // extern "C"
