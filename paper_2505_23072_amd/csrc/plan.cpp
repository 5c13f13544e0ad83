// Load planner (host): resolves requested names over the parsed headers, works out each rank's
// share (paper Section III-B: same-shaped partitions along one dimension; Section II-A: input
// projections split column-wise, output projections row-wise) under the row-major layout rule of
// Section III-A, and emits flat copy descriptors grouped by the file byte ranges that get staged.
#include <algorithm>
#include <cstring>
#include <memory>
#include <new>

#include "fst_internal.h"

namespace fst {

uint32_t conv_kind(int s, int d)
{
    if (d == FST_KEEP || d == s) return CONV_COPY;
    if (s == FST_F16 && d == FST_BF16) return CONV_H2B;
    if (s == FST_BF16 && d == FST_F16) return CONV_B2H;
    if (s == FST_F16 && d == FST_F32) return CONV_H2F;
    if (s == FST_BF16 && d == FST_F32) return CONV_B2F;
    if (s == FST_F32 && d == FST_F16) return CONV_F2H;
    if (s == FST_F32 && d == FST_BF16) return CONV_F2B;
    if (s == FST_F64 && d == FST_F32) return CONV_D2F;
    if (s == FST_F32 && d == FST_F64) return CONV_F2D;
    if (s == FST_F64 && d == FST_F16) return CONV_D2H;
    if (s == FST_F64 && d == FST_BF16) return CONV_D2B;
    if (s == FST_F16 && d == FST_F64) return CONV_H2D;
    if (s == FST_BF16 && d == FST_F64) return CONV_B2D;
    if (s == FST_F8_E5M2) return d == FST_F16 ? CONV_E5H : d == FST_BF16 ? CONV_E5B : d == FST_F32 ? CONV_E5F : CONV_COUNT;
    if (s == FST_F8_E4M3) return d == FST_F16 ? CONV_E4H : d == FST_BF16 ? CONV_E4B : d == FST_F32 ? CONV_E4F : CONV_COUNT;
    return CONV_COUNT;
}

namespace {

constexpr uint64_t kMinGroupBytes = 4096;
constexpr uint64_t kCutElems = 256;     // rows are cut inside at multiples of this many elements
// Ragged rows at least this long (in units) go through the element path: the spliced and gather
// paths count units of a piece in 32 bits, from the start of the piece's first row.
constexpr uint64_t kRaggedRowMaxUnits = 1ull << 30;

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Append the public descriptor and the device pieces for rows [r0, r1) of output `oi`, or, when
// e1 > e0, for elements [e0, e1) of the single row r0.  extent: index of the group's compacted
// extent staged for exactly these rows (SIZE_MAX: the bytes lie in the group's plain ranges);
// compact: that extent holds several rows back to back, so the device sees one contiguous row.
int add_work(fst_plan *p, Group &g, uint32_t oi, uint64_t r0, uint64_t r1, uint64_t e0, uint64_t e1,
             size_t extent = SIZE_MAX, bool compact = false)
{
    const Output &o = p->outputs[oi];
    const uint32_t conv = conv_kind(o.src_dtype, o.info.dtype);
    const uint64_t es_s = fst_dtype_size(o.src_dtype), es_d = fst_dtype_size(o.info.dtype);
    const bool partial = e1 > e0;
    const uint64_t file_rows = partial ? 1 : r1 - r0;
    const uint64_t file_relems = partial ? e1 - e0 : o.row_elems;
    const uint64_t file_src0 = o.src_file_off + r0 * o.src_stride + (partial ? e0 * es_s : 0);
    const uint64_t dst0 = (r0 * o.row_elems + (partial ? e0 : 0)) * es_d;
    if (file_rows == 0 || file_relems == 0) return FST_OK;

    fst_descriptor d{};
    d.output = oi;
    d.file = o.info.file;
    d.group = uint32_t(&g - p->groups.data());
    d.src_dtype = o.src_dtype;
    d.dst_dtype = o.info.dtype;
    d.src_file_off = file_src0;
    d.src_stride = file_rows > 1 ? o.src_stride : 0;
    d.dst_off = dst0;
    d.row_elems = file_relems;
    d.n_rows = file_rows;
    p->descs.push_back(d);

    // what the device sees: the file geometry, or one row over the compacted image (offset 0 = its start)
    const uint64_t rows = compact ? 1 : file_rows;
    const uint64_t relems = compact ? file_rows * file_relems : file_relems;
    const uint64_t src0 = compact ? 0 : file_src0;
    const uint64_t stride = rows > 1 ? o.src_stride : 0;
    // source address modulo 256 of offset `off`: file byte x sits at x + phase (mod 256) in every layout
    const uint64_t phase0 = g.phase + (compact ? g.extents[extent].lo : 0);   // (while a group is built, extents = the compacted ones)

    // the kernels count in units: bytes when nothing is converted, elements otherwise
    const uint64_t unit_s = conv_src_bytes(conv), unit_d = conv_dst_bytes(conv);
    const uint64_t row_units = conv == CONV_COPY ? relems * es_s : relems;
    const uint64_t chunk = conv_chunk_elems(conv);
    const uint64_t align = conv_store_align(conv);

    auto push = [&](uint32_t path, uint64_t soff, uint64_t doff, uint64_t n_units, uint64_t upr, uint64_t nrows,
                    uint64_t unit0) -> int {
        if (upr > (nrows > 1 ? (1ull << 31) : uint64_t(UINT32_MAX)))
            return fail(FST_E_RANGE, "a row of output %u is too long for one descriptor", oi);
        Piece pc;
        pc.output = oi;
        pc.path = path;
        pc.conv = conv;
        pc.own_extent = extent != SIZE_MAX;
        pc.extent = pc.own_extent ? uint32_t(extent) : 0;
        pc.compact = compact;
        pc.src_file_off = soff;
        pc.src_stride = nrows > 1 ? stride : 0;
        pc.dst_off = doff;
        pc.n_units = n_units;
        pc.units_per_row = uint32_t(upr);
        pc.unit0 = uint32_t(unit0);
        const uint64_t per_unit_s = path == PATH_VEC ? chunk * unit_s : unit_s;
        pc.src_span = (nrows - 1) * pc.src_stride + upr * per_unit_s;
        const uint64_t addr = phase0 + soff;
        pc.dword_aligned = (addr % 4 == 0) && (nrows == 1 || stride % 4 == 0);
        if (path == PATH_GATHER) {
            // the largest power of two (at most 8 bytes) that divides the first address, the stride and the row
            // length: loads of that size never straddle a row end
            uint32_t grain = 8;
            while (grain > 1 && (addr % grain || stride % grain || (upr * unit_s) % grain)) grain /= 2;
            pc.grain = grain;
            pc.staged = grain <= 4 && gather_span_fits(tile_units(path) * chunk, upr, unit_s, stride);
        }
        const bool chunks = path != PATH_ELEM;
        const uint64_t elems = chunks ? n_units * chunk : n_units;
        pc.read_bytes = elems * unit_s;
        pc.write_bytes = elems * unit_d;
        const uint64_t tiles = ceil_div(n_units, tile_units(path));
        if (tiles > (1u << 30)) return fail(FST_E_RANGE, "output %u needs too many tiles", oi);
        g.pieces.push_back(pc);
        g.read_bytes += pc.read_bytes;
        g.write_bytes += pc.write_bytes;
        return FST_OK;
    };
    // units between dst byte `at` and the next store boundary of the output
    auto head_units = [&](uint64_t at, uint64_t limit) { return std::min<uint64_t>(limit, (align - at % align) % align / unit_d); };

    if (rows == 1) {
        // one long row.  When it does not start on a store boundary of the output (a cut inside an
        // output with ragged rows), the units up to the next boundary go through the element path.
        const uint64_t head = head_units(dst0, row_units);
        if (head)
            if (int rc = push(PATH_ELEM, src0, dst0, head, head, 1, 0)) return rc;
        const uint64_t s1 = src0 + head * unit_s, d1 = dst0 + head * unit_d;
        const uint64_t full = (row_units - head) / chunk, tail = (row_units - head) % chunk;
        // the body, in pieces whose chunk indices fit 32 bits
        for (uint64_t c = 0; c < full; c += VEC_PIECE_MAX_UNITS) {
            const uint64_t n = std::min(full - c, VEC_PIECE_MAX_UNITS);
            if (int rc = push(PATH_VEC, s1 + c * chunk * unit_s, d1 + c * chunk * unit_d, n, 1, 1, 0)) return rc;
            Piece &pc = g.pieces.back();
            pc.units_per_row = 0;       // 0 = a single row of any length
            pc.src_span = n * chunk * unit_s;
        }
        if (tail)
            if (int rc = push(PATH_ELEM, s1 + full * chunk * unit_s, d1 + full * chunk * unit_d, tail, tail, 1, 0))
                return rc;
    } else if (row_units % chunk == 0) {
        // rows of whole chunks: every row starts on a store boundary of the output
        const uint64_t upr = row_units / chunk;
        if (upr > VEC_PIECE_MAX_UNITS) return fail(FST_E_RANGE, "a row of output %u is too long for one descriptor", oi);
        const uint64_t rows_per = VEC_PIECE_MAX_UNITS / upr;
        for (uint64_t r = 0; r < rows; r += rows_per) {
            const uint64_t nr = std::min(rows - r, rows_per);
            if (int rc = push(PATH_VEC, src0 + r * stride, dst0 + r * upr * chunk * unit_d, nr * upr, upr, nr, 0))
                return rc;
        }
    } else if (row_units >= kRaggedRowMaxUnits) {
        if (int rc = push(PATH_ELEM, src0, dst0, rows * row_units, row_units, rows, 0)) return rc;
    } else {
        // ragged rows: chunks are cut from the output stream, which keeps the stores aligned.  Rows of
        // at least one chunk are spliced (a chunk that straddles a row end comes from two rows), shorter
        // ones gathered unit by unit.  The units before the first store boundary and after the last whole
        // chunk go through the element path.  Unit indices inside a piece, counted from the start of the
        // piece's first row, stay below 2^31.
        const uint32_t path = row_units >= chunk ? PATH_SPLICE : PATH_GATHER;
        const uint64_t total = rows * row_units;
        const uint64_t head = head_units(dst0, total);
        const uint64_t full = (total - head) / chunk, tail = (total - head) % chunk;
        const uint64_t per_piece = (SPLICE_PIECE_MAX_UNITS - kRaggedRowMaxUnits) / chunk * chunk;
        auto rows_from = [&](uint64_t first, uint64_t n) { return (first + n - 1) / row_units - first / row_units + 1; };
        if (head)
            if (int rc = push(PATH_ELEM, src0, dst0, head, row_units, rows_from(0, head), 0)) return rc;
        for (uint64_t cu = 0; cu < full * chunk; cu += per_piece) {
            const uint64_t n = std::min(per_piece, full * chunk - cu), first = head + cu;
            if (int rc = push(path, src0 + first / row_units * stride, dst0 + first * unit_d, n / chunk, row_units,
                              rows_from(first, n), first % row_units))
                return rc;
        }
        if (tail) {
            const uint64_t first = head + full * chunk;
            if (int rc = push(PATH_ELEM, src0 + first / row_units * stride, dst0 + first * unit_d, tail, row_units,
                              rows_from(first, tail), first % row_units))
                return rc;
        }
    }
    return FST_OK;
}

uint64_t round_up_256(uint64_t v) { return (v + FST_RAW_ALIGN - 1) / FST_RAW_ALIGN * FST_RAW_ALIGN; }

// Slot space of `bytes` staged bytes whose first one is file byte lo: the image starts at the
// phase the file's bytes have in every layout ((lo + phase) % 256), so a source has the same
// alignment wherever it is staged, and the next image starts on the following 256-byte boundary.
uint64_t extent_space(const Group &g, uint64_t lo, uint64_t bytes) { return round_up_256((lo + g.phase) % FST_RAW_ALIGN + bytes); }

uint64_t sat_add(uint64_t a, uint64_t b) { return a > UINT64_MAX - b ? UINT64_MAX : a + b; }

// The plain ranges of a group under construction form a set of intervals that lie further apart
// than min_gap; a new range absorbs every interval it overlaps or comes within min_gap of.
// Returns the bounds of the interval the range would end up in and the slot space of the
// intervals it would absorb.
struct Merge { uint64_t lo, hi, absorbed_space; std::map<uint64_t, uint64_t>::const_iterator first, last; };
Merge merge_of(const Group &g, uint64_t s_lo, uint64_t s_hi, uint64_t min_gap)
{
    Merge m{s_lo, s_hi, 0, g.plain.end(), g.plain.end()};
    auto it = g.plain.upper_bound(s_lo);
    // step back over intervals that end within min_gap before s_lo (they are further apart than min_gap
    // from each other, so at most one can)
    if (it != g.plain.begin()) {
        auto prev = std::prev(it);
        if (sat_add(prev->second, min_gap) >= s_lo) it = prev;
    }
    m.first = it;
    while (it != g.plain.end() && it->first <= sat_add(m.hi, min_gap)) {
        m.lo = std::min(m.lo, it->first);
        m.hi = std::max(m.hi, it->second);
        m.absorbed_space += extent_space(g, it->first, it->second - it->first);
        ++it;
    }
    m.last = it;
    return m;
}

// Slot space of the group if the plain byte range [s_lo, s_hi) were added.
uint64_t space_with(const Group &g, uint64_t s_lo, uint64_t s_hi, uint64_t min_gap)
{
    const Merge m = merge_of(g, s_lo, s_hi, min_gap);
    return g.slot_bytes - m.absorbed_space + extent_space(g, m.lo, m.hi - m.lo);
}

void add_range(Group &g, uint64_t s_lo, uint64_t s_hi, uint64_t min_gap)
{
    const Merge m = merge_of(g, s_lo, s_hi, min_gap);
    g.slot_bytes = g.slot_bytes - m.absorbed_space + extent_space(g, m.lo, m.hi - m.lo);
    g.plain.erase(m.first, m.last);
    g.plain[m.lo] = m.hi;
    g.lo = g.hi == 0 ? s_lo : std::min(g.lo, s_lo);        // hi == 0: the group's first range
    g.hi = std::max(g.hi, s_hi);
}

// Adds a compacted extent: n_rows segments of row_bytes, `stride` apart in the file, back to back in
// the image.  Returns its index among the group's compacted extents.
size_t add_compact(Group &g, uint64_t lo, uint64_t row_bytes, uint64_t n_rows, uint64_t stride)
{
    Extent e;
    e.lo = lo;
    e.hi = lo + (n_rows - 1) * stride + row_bytes;
    e.row_bytes = row_bytes;
    e.n_rows = n_rows;
    e.stride = n_rows > 1 ? stride : 0;
    g.slot_bytes += extent_space(g, lo, n_rows * row_bytes);
    g.lo = g.hi == 0 ? lo : std::min(g.lo, lo);
    g.hi = std::max(g.hi, e.hi);
    g.extents.push_back(e);
    return g.extents.size() - 1;
}

// Fixes the group's extents: the plain intervals in file order, then the compacted extents; gives
// every extent its place in the slot image and every piece the index of the extent that holds it.
int close_group(fst_plan *p, Group &g, size_t desc_begin)
{
    g.desc_begin = desc_begin;
    g.desc_end = p->descs.size();
    std::vector<Extent> all;
    all.reserve(g.plain.size() + g.extents.size());
    for (const auto &iv : g.plain) {
        Extent e;
        e.lo = iv.first;
        e.hi = iv.second;
        e.row_bytes = e.hi - e.lo;
        all.push_back(e);
    }
    const size_t n_plain = all.size();
    all.insert(all.end(), g.extents.begin(), g.extents.end());
    g.extents.swap(all);
    g.plain.clear();
    uint64_t at = 0;
    for (Extent &e : g.extents) {
        e.slot_off = at + (e.lo + g.phase) % FST_RAW_ALIGN;
        at += extent_space(g, e.lo, e.image_bytes());
    }
    g.slot_bytes = at;
    for (Piece &pc : g.pieces) {
        if (pc.own_extent) { pc.extent += uint32_t(n_plain); continue; }
        // the plain extent with the largest lo <= the piece's first byte
        auto it = std::upper_bound(g.extents.begin(), g.extents.begin() + n_plain, pc.src_file_off,
                                   [](uint64_t v, const Extent &e) { return v < e.lo; });
        if (it == g.extents.begin() || pc.src_file_off + pc.src_span > (it - 1)->hi)
            return fail(FST_E_RANGE, "output %u: source bytes are not inside one staged extent", pc.output);
        pc.extent = uint32_t(it - 1 - g.extents.begin());
    }
    std::stable_sort(g.pieces.begin(), g.pieces.end(),
                     [](const Piece &a, const Piece &b) { return launch_class(a) < launch_class(b); });
    return FST_OK;
}

}  // namespace

int build_groups(fst_plan *p, uint64_t max_bytes, uint64_t min_gap, uint64_t min_seg)
{
    if (max_bytes != 0 && max_bytes < kMinGroupBytes)
        return fail(FST_E_ARG, "max_group_bytes must be 0 or at least %llu", (unsigned long long)kMinGroupBytes);
    // in a slot an extent starts at its phase (up to 255 bytes) and is padded to 256
    const uint64_t budget = max_bytes ? max_bytes - 2 * (FST_RAW_ALIGN - 1) : UINT64_MAX;
    {
        std::lock_guard<std::mutex> lock(p->image_mu);
        p->images.clear();
        p->builtin_images.clear();
    }
    p->descs.clear();
    p->groups.clear();
    p->read_bytes = p->write_bytes = 0;
    p->min_gap = min_gap;
    p->has_compact = false;

    // outputs per file, in file order
    std::vector<std::vector<uint32_t>> per_file(p->n_files);
    size_t n_work = 0;
    for (uint32_t i = 0; i < p->outputs.size(); ++i)
        if (p->outputs[i].info.nbytes) { per_file[p->outputs[i].info.file].push_back(i); ++n_work; }
    p->groups.reserve(n_work + p->n_files);
    std::vector<Group> &G = p->groups;

    for (uint32_t f = 0; f < p->n_files; ++f) {
        auto &list = per_file[f];
        std::sort(list.begin(), list.end(), [&](uint32_t a, uint32_t b) {
            return p->outputs[a].src_file_off < p->outputs[b].src_file_off;
        });
        bool open = false;
        size_t desc_begin = 0;
        auto start = [&]() {
            G.emplace_back();
            G.back().file = f;
            G.back().phase = p->raw_base[f] % FST_RAW_ALIGN;
            desc_begin = p->descs.size();
            open = true;
        };
        int close_rc = FST_OK;
        auto finish = [&]() {
            if (open)
                if (int rc = close_group(p, G.back(), desc_begin)) close_rc = rc;
            open = false;
        };
        for (uint32_t oi : list) {
            const Output &o = p->outputs[oi];
            const uint64_t es_s = fst_dtype_size(o.src_dtype);
            const uint64_t row_bytes = o.row_elems * es_s;
            const uint64_t s_lo = o.src_file_off;
            const uint64_t s_hi = s_lo + (o.n_rows - 1) * o.src_stride + row_bytes;
            // compacted staging: the rows of a strided share (a partition along an inner dimension, the
            // blocks of a fused matrix) are read one by one and staged back to back, so that nothing of
            // the other ranks' shares crosses the bus; only for rows long enough to be worth a read each
            if (min_seg != UINT64_MAX && o.n_rows > 1 && o.src_stride > row_bytes && row_bytes >= min_seg &&
                row_bytes <= budget) {
                const uint64_t rows_per = std::max<uint64_t>(1, std::min(o.n_rows, budget / row_bytes));
                for (uint64_t r = 0; r < o.n_rows; r += rows_per) {
                    const uint64_t nr = std::min(o.n_rows - r, rows_per);
                    const uint64_t c_lo = s_lo + r * o.src_stride;
                    if (nr == 1) {          // a single segment is a plain range
                        if (open && max_bytes && space_with(G.back(), c_lo, c_lo + row_bytes, min_gap) > max_bytes) finish();
                        if (!open) start();
                        add_range(G.back(), c_lo, c_lo + row_bytes, min_gap);
                        if (int rc = add_work(p, G.back(), oi, r, r + 1, 0, 0)) return rc;
                        continue;
                    }
                    if (open && max_bytes && G.back().slot_bytes + extent_space(G.back(), c_lo, nr * row_bytes) > max_bytes) finish();
                    if (!open) start();
                    const size_t ex = add_compact(G.back(), c_lo, row_bytes, nr, o.src_stride);
                    if (int rc = add_work(p, G.back(), oi, r, r + nr, 0, 0, ex, true)) return rc;
                }
                p->has_compact = true;
                continue;
            }
            // sparse staging: rows that lie further apart than min_gap (the blocks of a fused matrix) are
            // staged, and worked on, one by one, so the bytes between them stay out
            if (min_gap != UINT64_MAX && o.n_rows > 1 && o.src_stride - row_bytes > min_gap && row_bytes <= budget) {
                for (uint64_t r = 0; r < o.n_rows; ++r) {
                    const uint64_t c_lo = s_lo + r * o.src_stride, c_hi = c_lo + row_bytes;
                    if (open && max_bytes && space_with(G.back(), c_lo, c_hi, min_gap) > max_bytes) finish();
                    if (!open) start();
                    add_range(G.back(), c_lo, c_hi, min_gap);
                    if (int rc = add_work(p, G.back(), oi, r, r + 1, 0, 0)) return rc;
                }
                continue;
            }
            if (s_hi - s_lo <= budget) {
                if (open && max_bytes && space_with(G.back(), s_lo, s_hi, min_gap) > max_bytes) finish();
                if (!open) start();
                Group &g = G.back();
                add_range(g, s_lo, s_hi, min_gap);
                if (int rc = add_work(p, g, oi, 0, o.n_rows, 0, 0)) return rc;
                continue;
            }
            // the tensor alone exceeds a group: cut between rows, and inside rows that are too long
            finish();
            if (row_bytes <= budget) {
                const uint64_t rows_per = 1 + (budget - row_bytes) / o.src_stride;
                for (uint64_t r = 0; r < o.n_rows; r += rows_per) {
                    const uint64_t r1 = std::min(o.n_rows, r + rows_per);
                    start();
                    const uint64_t c_lo = s_lo + r * o.src_stride;
                    add_range(G.back(), c_lo, c_lo + (r1 - r - 1) * o.src_stride + row_bytes, min_gap);
                    if (int rc = add_work(p, G.back(), oi, r, r1, 0, 0)) return rc;
                    finish();
                }
            } else {
                const uint64_t cut = (budget / es_s) / kCutElems * kCutElems;
                if (cut == 0) return fail(FST_E_RANGE, "max_group_bytes too small to cut a row");
                for (uint64_t r = 0; r < o.n_rows; ++r)
                    for (uint64_t e = 0; e < o.row_elems; e += cut) {
                        const uint64_t e1 = std::min(o.row_elems, e + cut);
                        start();
                        const uint64_t c_lo = s_lo + r * o.src_stride + e * es_s;
                        add_range(G.back(), c_lo, c_lo + (e1 - e) * es_s, min_gap);
                        if (int rc = add_work(p, G.back(), oi, r, r, e, e1)) return rc;
                        finish();
                    }
            }
        }
        finish();
        if (close_rc) return close_rc;
    }
    p->max_group_pieces = 0;
    p->total_pieces = 0;
    uint64_t packed = 0;
    for (Group &g : G) {
        p->max_group_pieces = std::max(p->max_group_pieces, g.pieces.size());
        p->total_pieces += g.pieces.size();
        // a launch of k pieces and T tiles has at most T / 1024 + 2k + 2 spans (hint_shift_for: below the
        // largest shift a span is longer than half the mean piece), the last workgroup's spare tiles included,
        // and two table entries per span
        g.hint_bound = 4 * N_CLASSES;
        for (const Piece &pc : g.pieces)
            g.hint_bound += 2 * (ceil_div(pc.n_units, tile_units(pc.path)) >> MAX_HINT_SHIFT) + 8;
        p->read_bytes += g.read_bytes;
        p->write_bytes += g.write_bytes;
        g.packed_off = packed;
        packed += g.slot_bytes;                 // a multiple of 256
    }
    p->packed_bytes = packed;
    return FST_OK;
}

namespace {

int plan_impl(const fst_header *const *hdrs, const uint64_t *raw_base, size_t n_files,
              const char *const *names, const fst_request *reqs, size_t n_names, int32_t rank,
              int32_t world, fst_plan **out)
{
    if (!out) return fail(FST_E_ARG, "fst_plan_create: out is NULL");
    *out = nullptr;
    if (!hdrs || !raw_base || (!names && n_names) || (!reqs && n_names))
        return fail(FST_E_ARG, "fst_plan_create: NULL argument");
    if (n_files == 0 || n_files > UINT32_MAX) return fail(FST_E_ARG, "fst_plan_create: bad file count");
    if (world < 1 || rank < 0 || rank >= world)
        return fail(FST_E_SHARD, "rank %d is not inside world %d", rank, world);

    std::unique_ptr<fst_plan> p(new fst_plan);
    p->n_files = n_files;
    for (size_t f = 0; f < n_files; ++f) {
        if (!hdrs[f]) return fail(FST_E_ARG, "header %zu is NULL", f);
        p->raw_base.push_back(raw_base[f]);
        p->file_size.push_back(hdrs[f]->file_size);
    }
    // one index over the whole file set (a tensor name must be unique over it): name -> (file, tensor)
    size_t n_tensors = 0;
    for (size_t f = 0; f < n_files; ++f) n_tensors += hdrs[f]->tensors.size();
    std::unordered_map<std::string, std::pair<uint32_t, uint32_t>> where;
    where.reserve(n_tensors * 2);
    for (size_t f = 0; f < n_files; ++f)
        for (size_t k = 0; k < hdrs[f]->tensors.size(); ++k) {
            const Tensor &t = hdrs[f]->tensors[k];
            auto ins = where.emplace(t.name, std::make_pair(uint32_t(f), uint32_t(k)));
            if (!ins.second)
                return fail(FST_E_DUP_NAME, "tensor %s is in file %u and in file %zu", t.name.c_str(), ins.first->second.first, f);
        }

    p->outputs.resize(n_names);
    for (size_t i = 0; i < n_names; ++i) {
        if (!names[i]) return fail(FST_E_ARG, "names[%zu] is NULL", i);
        auto hit = where.find(names[i]);
        if (hit == where.end()) return fail(FST_E_NOT_FOUND, "tensor %s is in none of the %zu files", names[i], n_files);
        const size_t file = hit->second.first;
        const Tensor *t = &hdrs[file]->tensors[hit->second.second];
        const fst_request &rq = reqs[i];
        const int32_t dd = rq.dst_dtype == FST_KEEP ? t->dtype : rq.dst_dtype;
        if (dd < 0 || dd >= FST_DTYPE_COUNT) return fail(FST_E_DTYPE, "%s: unknown target dtype %d", names[i], rq.dst_dtype);
        if (conv_kind(t->dtype, dd) == CONV_COUNT)
            return fail(FST_E_CAST, "%s: no conversion from %s to %s", names[i], fst_dtype_name(t->dtype), fst_dtype_name(dd));
        const int32_t d = rq.shard_dim;
        if (rq.blocks < 1 || (d < 0 && rq.blocks != 1) || (rq.blocks > 1 && d != 0))
            return fail(FST_E_SHARD, "%s: blocks=%d needs shard_dim 0", names[i], rq.blocks);
        if (d >= t->ndim) return fail(FST_E_SHARD, "%s: shard_dim %d but the tensor has %d dims", names[i], d, t->ndim);
        const int32_t req_rank = rq.rank < 0 ? rank : rq.rank;
        if (req_rank >= world) return fail(FST_E_SHARD, "%s: rank %d is not inside world %d", names[i], req_rank, world);

        Output &o = p->outputs[i];
        o.info = fst_output_info{};
        o.info.dtype = dd;
        o.info.ndim = t->ndim;
        o.info.align = FST_OUTPUT_ALIGN;
        o.info.file = uint32_t(file);
        o.src_dtype = t->dtype;
        const uint64_t es = fst_dtype_size(t->dtype);
        const uint64_t body = 8 + hdrs[file]->n_json;
        o.tensor_begin = body + t->begin;
        uint64_t numel = 1;
        for (int k = 0; k < t->ndim; ++k) { o.info.shape[k] = t->shape[k]; numel *= t->shape[k]; }
        if (d < 0) {
            o.n_rows = 1;
            o.row_elems = numel;
            o.src_stride = 0;
            o.src_file_off = o.tensor_begin;
        } else {
            const uint64_t parts = uint64_t(rq.blocks) * uint64_t(world);
            if (t->shape[d] % parts)
                return fail(FST_E_SHARD, "%s: dim %d of size %llu is not divisible by %llu", names[i], d,
                            (unsigned long long)t->shape[d], (unsigned long long)parts);
            uint64_t outer = 1, inner = 1;
            for (int k = 0; k < d; ++k) outer *= t->shape[k];
            for (int k = d + 1; k < t->ndim; ++k) inner *= t->shape[k];
            const uint64_t per = t->shape[d] / parts;
            o.info.shape[d] = t->shape[d] / uint64_t(world);
            o.n_rows = outer * uint64_t(rq.blocks);
            o.row_elems = per * inner;
            o.src_stride = (t->shape[d] / uint64_t(rq.blocks)) * inner * es;
            o.src_file_off = o.tensor_begin + uint64_t(req_rank) * per * inner * es;
            numel = o.n_rows * o.row_elems;
            if (o.n_rows > 1 && o.src_stride == o.row_elems * es) {   // rows are back to back
                o.row_elems *= o.n_rows;
                o.n_rows = 1;
            }
            if (o.n_rows <= 1) o.src_stride = 0;
        }
        if (numel == 0) { o.n_rows = 0; o.row_elems = 0; }
        o.info.nbytes = numel * fst_dtype_size(dd);
    }
    if (int rc = build_groups(p.get(), 0, UINT64_MAX, UINT64_MAX)) return rc;
    *out = p.release();
    return FST_OK;
}

}  // namespace
}  // namespace fst

using namespace fst;

#define FST_GUARD(expr)                                              \
    try { return (expr); }                                           \
    catch (const std::bad_alloc &) { return fail(FST_E_NOMEM, "out of memory"); } \
    catch (...) { return fail(FST_E_ARG, "unexpected internal error"); }

extern "C" {

int fst_plan_create(const fst_header *const *hdrs, const uint64_t *raw_base, size_t n_files,
                    const char *const *names, const fst_request *reqs, size_t n_names, int32_t rank,
                    int32_t world, fst_plan **out)
{
    FST_GUARD(plan_impl(hdrs, raw_base, n_files, names, reqs, n_names, rank, world, out));
}

int fst_plan_uniform(const fst_header *const *hdrs, const uint64_t *raw_base, size_t n_files,
                     const char *const *names, size_t n_names, int32_t dst_dtype, int32_t shard_dim,
                     int32_t rank, int32_t world, fst_plan **out)
{
    try {
        std::vector<fst_request> reqs(n_names, fst_request{dst_dtype, shard_dim, 1, -1});
        return plan_impl(hdrs, raw_base, n_files, names, reqs.data(), n_names, rank, world, out);
    } catch (const std::bad_alloc &) {
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

size_t fst_plan_output_count(const fst_plan *p) { return p ? p->outputs.size() : 0; }

int fst_plan_output(const fst_plan *p, size_t i, fst_output_info *out)
{
    if (!p || !out) return fail(FST_E_ARG, "fst_plan_output: NULL argument");
    if (i >= p->outputs.size()) return fail(FST_E_RANGE, "output index %zu out of range", i);
    *out = p->outputs[i].info;
    return FST_OK;
}

int fst_plan_set_groups_compact(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes,
                                uint64_t min_segment_bytes, size_t *n_groups)
{
    if (!p) return fail(FST_E_ARG, "fst_plan_set_groups: plan is NULL");
    int rc;
    try { rc = build_groups(p, max_group_bytes, min_gap_bytes, min_segment_bytes); }
    catch (const std::bad_alloc &) { rc = fail(FST_E_NOMEM, "out of memory"); }
    catch (...) { rc = fail(FST_E_ARG, "unexpected internal error"); }
    if (rc) {                       // leave the plan usable: back to one group per file
        try { build_groups(p, 0, UINT64_MAX, UINT64_MAX); } catch (...) {}
        return rc;
    }
    if (n_groups) *n_groups = p->groups.size();
    return FST_OK;
}

int fst_plan_set_groups_sparse(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes, size_t *n_groups)
{
    return fst_plan_set_groups_compact(p, max_group_bytes, min_gap_bytes, UINT64_MAX, n_groups);
}

int fst_plan_set_groups(fst_plan *p, uint64_t max_group_bytes, size_t *n_groups)
{
    return fst_plan_set_groups_sparse(p, max_group_bytes, UINT64_MAX, n_groups);
}

size_t fst_plan_group_count(const fst_plan *p) { return p ? p->groups.size() : 0; }

int fst_plan_group(const fst_plan *p, size_t g, fst_group_info *out)
{
    if (!p || !out) return fail(FST_E_ARG, "fst_plan_group: NULL argument");
    if (g >= p->groups.size()) return fail(FST_E_RANGE, "group index %zu out of range", g);
    const Group &gr = p->groups[g];
    out->file = gr.file;
    out->n_descriptors = uint32_t(gr.desc_end - gr.desc_begin);
    out->n_extents = uint32_t(gr.extents.size());
    out->lo = gr.lo;
    out->hi = gr.hi;
    out->slot_bytes = gr.slot_bytes;
    out->staged_bytes = 0;
    for (const Extent &e : gr.extents) out->staged_bytes += e.image_bytes();
    out->packed_offset = gr.packed_off;
    out->read_bytes = gr.read_bytes;
    out->write_bytes = gr.write_bytes;
    return FST_OK;
}

int fst_plan_group_extent(const fst_plan *p, size_t g, size_t i, fst_extent *out)
{
    if (!p || !out) return fail(FST_E_ARG, "fst_plan_group_extent: NULL argument");
    if (g >= p->groups.size()) return fail(FST_E_RANGE, "group index %zu out of range", g);
    if (i >= p->groups[g].extents.size()) return fail(FST_E_RANGE, "extent index %zu out of range", i);
    const Extent &e = p->groups[g].extents[i];
    out->lo = e.lo;
    out->hi = e.hi;
    out->slot_offset = e.slot_off;
    out->row_bytes = e.row_bytes;
    out->n_rows = e.n_rows;
    out->stride = e.stride;
    return FST_OK;
}

size_t fst_plan_descriptor_count(const fst_plan *p) { return p ? p->descs.size() : 0; }

int fst_plan_descriptor(const fst_plan *p, size_t i, fst_descriptor *out)
{
    if (!p || !out) return fail(FST_E_ARG, "fst_plan_descriptor: NULL argument");
    if (i >= p->descs.size()) return fail(FST_E_RANGE, "descriptor index %zu out of range", i);
    *out = p->descs[i];
    return FST_OK;
}

uint64_t fst_plan_read_bytes(const fst_plan *p) { return p ? p->read_bytes : 0; }
uint64_t fst_plan_write_bytes(const fst_plan *p) { return p ? p->write_bytes : 0; }
uint64_t fst_plan_packed_bytes(const fst_plan *p) { return p ? p->packed_bytes : 0; }

size_t fst_plan_workspace_bytes(const fst_plan *p)
{
    if (!p) return 0;
    // room for the tables of all groups side by side (the stager uploads them together); a table
    // of several groups merged is never larger
    size_t n = 0;
    for (const Group &g : p->groups) n += table_bytes(g.pieces.size(), g.hint_bound);
    return std::max<size_t>(n, 256);
}

void fst_plan_free(fst_plan *p) { delete p; }

}  // extern "C"
