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
    return CONV_COUNT;
}

uint32_t conv_src_bytes(uint32_t c)
{
    return c == CONV_COPY ? 1 : c == CONV_D2F ? 8 : (c == CONV_F2H || c == CONV_F2B || c == CONV_F2D) ? 4 : 2;
}
uint32_t conv_dst_bytes(uint32_t c)
{
    return c == CONV_COPY ? 1 : c == CONV_F2D ? 8 : (c == CONV_H2F || c == CONV_B2F || c == CONV_D2F) ? 4 : 2;
}
uint32_t conv_chunk_elems(uint32_t c) { return c == CONV_COPY ? 16 : (c == CONV_D2F || c == CONV_F2D) ? 4 : 8; }

namespace {

constexpr uint64_t kMinGroupBytes = 4096;
constexpr uint64_t kCutElems = 256;     // rows are cut inside at multiples of this many elements

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Append the public descriptor and the device pieces for rows [r0, r1) of output `oi`, or, when
// e1 > e0, for elements [e0, e1) of the single row r0.
int add_work(fst_plan *p, Group &g, uint32_t oi, uint64_t r0, uint64_t r1, uint64_t e0, uint64_t e1)
{
    const Output &o = p->outputs[oi];
    const uint32_t conv = conv_kind(o.src_dtype, o.info.dtype);
    const uint64_t es_s = fst_dtype_size(o.src_dtype), es_d = fst_dtype_size(o.info.dtype);
    const bool partial = e1 > e0;
    const uint64_t rows = partial ? 1 : r1 - r0;
    const uint64_t relems = partial ? e1 - e0 : o.row_elems;
    const uint64_t src0 = o.src_file_off + r0 * o.src_stride + (partial ? e0 * es_s : 0);
    const uint64_t dst0 = (r0 * o.row_elems + (partial ? e0 : 0)) * es_d;
    if (rows == 0 || relems == 0) return FST_OK;

    fst_descriptor d{};
    d.output = oi;
    d.file = o.info.file;
    d.group = uint32_t(&g - p->groups.data());
    d.src_dtype = o.src_dtype;
    d.dst_dtype = o.info.dtype;
    d.src_file_off = src0;
    d.src_stride = rows > 1 ? o.src_stride : 0;
    d.dst_off = dst0;
    d.row_elems = relems;
    d.n_rows = rows;
    p->descs.push_back(d);

    // the kernels count in units: bytes when nothing is converted, elements otherwise
    const uint64_t unit_s = conv_src_bytes(conv), unit_d = conv_dst_bytes(conv);
    const uint64_t row_units = conv == CONV_COPY ? relems * es_s : relems;
    const uint64_t chunk = conv_chunk_elems(conv);
    const uint64_t base_abs = p->raw_base[o.info.file] + src0;   // raw_base is 256-aligned

    auto push = [&](uint32_t path, uint64_t soff, uint64_t doff, uint64_t n_units, uint64_t upr,
                    uint64_t nrows) -> int {
        if (upr > (nrows > 1 ? (1ull << 31) : uint64_t(UINT32_MAX)))
            return fail(FST_E_RANGE, "a row of output %u is too long for one descriptor", oi);
        Piece pc;
        pc.output = oi;
        pc.path = path;
        pc.conv = conv;
        pc.src_file_off = soff;
        pc.src_stride = nrows > 1 ? o.src_stride : 0;
        pc.dst_off = doff;
        pc.n_units = n_units;
        pc.units_per_row = uint32_t(upr);
        const uint64_t per_unit_s = path == PATH_VEC ? chunk * unit_s : unit_s;
        pc.src_span = (nrows - 1) * pc.src_stride + upr * per_unit_s;
        pc.dword_aligned = ((p->raw_base[o.info.file] + soff) % 4 == 0) && (nrows == 1 || o.src_stride % 4 == 0);
        const uint64_t elems = path == PATH_ELEM ? n_units : n_units * chunk;
        pc.read_bytes = elems * unit_s;
        pc.write_bytes = elems * unit_d;
        const uint64_t tiles = ceil_div(n_units, tile_units(path));
        if (tiles > (1u << 30)) return fail(FST_E_RANGE, "output %u needs too many tiles", oi);
        g.pieces.push_back(pc);
        g.read_bytes += pc.read_bytes;
        g.write_bytes += pc.write_bytes;
        return FST_OK;
    };
    (void)base_abs;

    if (rows == 1) {
        // one long row.  When it does not start on a 16-byte boundary of the output (a cut inside an
        // output with ragged rows), the units up to the next boundary go through the element path.
        const uint64_t head = std::min<uint64_t>(row_units, (16 - dst0 % 16) % 16 / unit_d);
        if (head)
            if (int rc = push(PATH_ELEM, src0, dst0, head, head, 1)) return rc;
        const uint64_t s1 = src0 + head * unit_s, d1 = dst0 + head * unit_d;
        const uint64_t full = (row_units - head) / chunk, tail = (row_units - head) % chunk;
        // the body, in pieces whose chunk indices fit 32 bits
        for (uint64_t c = 0; c < full; c += VEC_PIECE_MAX_UNITS) {
            const uint64_t n = std::min(full - c, VEC_PIECE_MAX_UNITS);
            if (int rc = push(PATH_VEC, s1 + c * chunk * unit_s, d1 + c * chunk * unit_d, n, 1, 1)) return rc;
            Piece &pc = g.pieces.back();
            pc.units_per_row = 0;       // 0 = a single row of any length
            pc.src_span = n * chunk * unit_s;
        }
        if (tail)
            if (int rc = push(PATH_ELEM, s1 + full * chunk * unit_s, d1 + full * chunk * unit_d, tail, tail, 1))
                return rc;
    } else if (row_units % chunk == 0) {
        const uint64_t upr = row_units / chunk;
        if (upr > VEC_PIECE_MAX_UNITS) return fail(FST_E_RANGE, "a row of output %u is too long for one descriptor", oi);
        const uint64_t rows_per = VEC_PIECE_MAX_UNITS / upr;
        for (uint64_t r = 0; r < rows; r += rows_per) {
            const uint64_t nr = std::min(rows - r, rows_per);
            if (int rc = push(PATH_VEC, src0 + r * o.src_stride, dst0 + r * upr * chunk * unit_d, nr * upr, upr, nr))
                return rc;
        }
    } else if (dst0 % 16 == 0 && row_units >= chunk && row_units < SPLICE_PIECE_MAX_UNITS) {
        // ragged rows of at least one chunk: chunks are cut from the output stream, which keeps the
        // stores 16-byte aligned; a chunk that straddles a row end is spliced from two rows.  Unit
        // indices inside a piece stay below 2^31; pieces are cut after a multiple of 16 rows, which
        // keeps every piece's first output byte 16-byte aligned.
        uint64_t rows_per = SPLICE_PIECE_MAX_UNITS / row_units;       // rows whose units fit the index range
        if (rows > rows_per) rows_per = rows_per / 16 * 16;
        if (rows_per == 0) {
            if (int rc = push(PATH_ELEM, src0, dst0, rows * row_units, row_units, rows)) return rc;
            return FST_OK;
        }
        for (uint64_t r = 0; r < rows; r += rows_per) {
            const uint64_t nr = std::min(rows - r, rows_per);
            const uint64_t units = nr * row_units, full = units / chunk, tail = units % chunk;
            const uint64_t s0 = src0 + r * o.src_stride, d0 = dst0 + r * row_units * unit_d;
            if (int rc = push(PATH_SPLICE, s0, d0, full, row_units, nr)) return rc;
            if (tail)       // the last units of the last row
                if (int rc = push(PATH_ELEM, s0 + (nr - 1) * o.src_stride + (row_units - tail) * unit_s,
                                  d0 + full * chunk * unit_d, tail, tail, 1))
                    return rc;
        }
    } else {
        if (int rc = push(PATH_ELEM, src0, dst0, rows * row_units, row_units, rows)) return rc;
    }
    return FST_OK;
}

uint64_t round_up_256(uint64_t v) { return (v + FST_RAW_ALIGN - 1) / FST_RAW_ALIGN * FST_RAW_ALIGN; }

// Slot space of an extent: it starts at its file phase (lo % 256) so sources keep their alignment,
// and the next extent starts on the following 256-byte boundary.
uint64_t extent_space(uint64_t lo, uint64_t hi) { return round_up_256(lo % FST_RAW_ALIGN + (hi - lo)); }

// Slot space of the group if the byte range [s_lo, s_hi) were added (ranges arrive in file order).
uint64_t space_with(const Group &g, uint64_t s_lo, uint64_t s_hi, uint64_t min_gap)
{
    if (g.extents.empty()) return extent_space(s_lo, s_hi);
    const Extent &last = g.extents.back();
    if (s_lo <= last.hi || s_lo - last.hi <= min_gap)
        return g.slot_bytes - extent_space(last.lo, last.hi) + extent_space(last.lo, std::max(last.hi, s_hi));
    return g.slot_bytes + extent_space(s_lo, s_hi);
}

void add_range(Group &g, uint64_t s_lo, uint64_t s_hi, uint64_t min_gap)
{
    g.slot_bytes = space_with(g, s_lo, s_hi, min_gap);
    if (!g.extents.empty() && (s_lo <= g.extents.back().hi || s_lo - g.extents.back().hi <= min_gap)) {
        g.extents.back().hi = std::max(g.extents.back().hi, s_hi);
    } else {
        Extent e;
        e.lo = s_lo;
        e.hi = s_hi;
        g.extents.push_back(e);
    }
    g.lo = g.extents.front().lo;
    g.hi = std::max(g.hi, s_hi);
}

void close_group(fst_plan *p, Group &g, size_t desc_begin)
{
    g.desc_begin = desc_begin;
    g.desc_end = p->descs.size();
    uint64_t at = 0;
    for (Extent &e : g.extents) {
        e.slot_off = at + e.lo % FST_RAW_ALIGN;
        at += extent_space(e.lo, e.hi);
    }
    g.slot_bytes = at;
    std::stable_sort(g.pieces.begin(), g.pieces.end(),
                     [](const Piece &a, const Piece &b) { return launch_class(a) < launch_class(b); });
}

}  // namespace

int build_groups(fst_plan *p, uint64_t max_bytes, uint64_t min_gap)
{
    if (max_bytes != 0 && max_bytes < kMinGroupBytes)
        return fail(FST_E_ARG, "max_group_bytes must be 0 or at least %llu", (unsigned long long)kMinGroupBytes);
    // in a slot an extent starts at its file phase (up to 255 bytes) and is padded to 256
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
            desc_begin = p->descs.size();
            open = true;
        };
        auto finish = [&]() {
            if (open) close_group(p, G.back(), desc_begin);
            open = false;
        };
        for (uint32_t oi : list) {
            const Output &o = p->outputs[oi];
            const uint64_t es_s = fst_dtype_size(o.src_dtype);
            const uint64_t row_bytes = o.row_elems * es_s;
            const uint64_t s_lo = o.src_file_off;
            const uint64_t s_hi = s_lo + (o.n_rows - 1) * o.src_stride + row_bytes;
            // sparse staging: rows that lie further apart than min_gap (the blocks of a fused
            // matrix) are staged, and worked on, one by one, so the bytes between them stay out
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
    }
    p->max_group_pieces = 0;
    p->total_pieces = 0;
    for (Group &g : G) {
        p->max_group_pieces = std::max(p->max_group_pieces, g.pieces.size());
        p->total_pieces += g.pieces.size();
        // a launch of k pieces with t_i tiles has ceil(sum t_i / HINT_SPAN) <= sum (t_i / HINT_SPAN + 1) hints,
        // plus its closing entry
        g.hint_bound = N_CLASSES;               // the closing entry of every launch
        for (const Piece &pc : g.pieces)
            g.hint_bound += ceil_div(pc.n_units, tile_units(pc.path)) / HINT_SPAN + 1;
        p->read_bytes += g.read_bytes;
        p->write_bytes += g.write_bytes;
    }
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
        if (raw_base[f] % FST_RAW_ALIGN)
            return fail(FST_E_ALIGN, "raw_base[%zu] is not a multiple of %d", f, FST_RAW_ALIGN);
        p->raw_base.push_back(raw_base[f]);
        p->file_size.push_back(hdrs[f]->file_size);
    }
    // a tensor name must be unique over the whole file set
    for (size_t f = 0; f < n_files; ++f)
        for (const Tensor &t : hdrs[f]->tensors)
            for (size_t g = 0; g < f; ++g)
                if (hdrs[g]->index.count(t.name))
                    return fail(FST_E_DUP_NAME, "tensor %s is in file %zu and in file %zu", t.name.c_str(), g, f);

    p->outputs.resize(n_names);
    for (size_t i = 0; i < n_names; ++i) {
        if (!names[i]) return fail(FST_E_ARG, "names[%zu] is NULL", i);
        const Tensor *t = nullptr;
        size_t file = 0;
        for (size_t f = 0; f < n_files && !t; ++f) {
            auto it = hdrs[f]->index.find(names[i]);
            if (it != hdrs[f]->index.end()) { t = &hdrs[f]->tensors[it->second]; file = f; }
        }
        if (!t) return fail(FST_E_NOT_FOUND, "tensor %s is in none of the %zu files", names[i], n_files);
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
    if (int rc = build_groups(p.get(), 0, UINT64_MAX)) return rc;
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

int fst_plan_set_groups_sparse(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes, size_t *n_groups)
{
    if (!p) return fail(FST_E_ARG, "fst_plan_set_groups: plan is NULL");
    int rc;
    try { rc = build_groups(p, max_group_bytes, min_gap_bytes); }
    catch (const std::bad_alloc &) { rc = fail(FST_E_NOMEM, "out of memory"); }
    catch (...) { rc = fail(FST_E_ARG, "unexpected internal error"); }
    if (rc) {                       // leave the plan usable: back to one group per file
        try { build_groups(p, 0, UINT64_MAX); } catch (...) {}
        return rc;
    }
    if (n_groups) *n_groups = p->groups.size();
    return FST_OK;
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
    for (const Extent &e : gr.extents) out->staged_bytes += e.hi - e.lo;
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
