// A CPU interpreter of the device tables (pieces + hints), for tests without a GPU.  It stands in
// for the kernel launcher: every launch walks its workgroups, wavefront tiles and lanes in the
// order and with the 32-bit index arithmetic the kernels use, finds each tile's piece through the
// hint table, and moves the bytes one chunk at a time.  Every address a kernel would touch is
// checked against the source and output ranges the test registered -- including the whole dwords
// the kernels read around unaligned bytes and the second read of a spliced chunk -- and a
// violation makes the launch fail.  Element conversion is the oracle's (this file is test code):
// what is checked here is the planner's geometry and the table format, not the conversion
// arithmetic of the kernels.  "Device" memory is host memory; see fake_hip_sync.cpp.
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "fst_internal.h"
#include "fst_oracle.h"

namespace {

struct Range { uintptr_t lo, hi; };
std::mutex g_mu;
Range g_source{0, 0};
std::vector<Range> g_outputs;
uint64_t g_chunks = 0, g_violations = 0, g_direct = 0;   // g_direct: tiles whose piece took one search step at most
uint64_t g_staged = 0;                                   // gathered tiles that went through the LDS area
char g_first_violation[256] = "";

void violation(const char *what, uint64_t a, uint64_t b)
{
    if (g_violations++ == 0) std::snprintf(g_first_violation, sizeof g_first_violation, "%s (%llu, %llu)", what,
                                           (unsigned long long)a, (unsigned long long)b);
}

bool readable(const uint8_t *p, uint64_t n) { return uintptr_t(p) >= g_source.lo && uintptr_t(p) + n <= g_source.hi; }
bool writable(const uint8_t *p, uint64_t n)
{
    for (const Range &r : g_outputs)
        if (uintptr_t(p) >= r.lo && uintptr_t(p) + n <= r.hi) return true;
    return false;
}

// A read of n bytes at p the way the byte-aligned loads do it: the enclosing aligned dwords.
void check_dword_read(const uint8_t *p, uint64_t n, const char *what)
{
    const uintptr_t a = uintptr_t(p) & ~uintptr_t(3), b = (uintptr_t(p) + n + 3) & ~uintptr_t(3);
    if (!readable(reinterpret_cast<const uint8_t *>(a), b - a)) violation(what, uintptr_t(p) - g_source.lo, n);
}
void check_read(const uint8_t *p, uint64_t n, uint64_t align, const char *what)
{
    if (!readable(p, n) || uintptr_t(p) % align) violation(what, uintptr_t(p) - g_source.lo, n);
}
void check_write(const uint8_t *p, uint64_t n, uint64_t align, const char *what)
{
    if (!writable(p, n) || uintptr_t(p) % align) violation(what, uintptr_t(p), n);
}

struct ConvInfo { uint32_t cs, cd, ch; int sd, dd; };      // chunk bytes in / out, units per chunk, oracle dtypes
ConvInfo conv_info(uint32_t conv)
{
    using namespace fst;
    switch (conv) {
    case CONV_COPY: return {16, 16, 16, ORC_U8, ORC_U8};
    case CONV_H2B: return {16, 16, 8, ORC_F16, ORC_BF16};
    case CONV_B2H: return {16, 16, 8, ORC_BF16, ORC_F16};
    case CONV_H2F: return {8, 16, 4, ORC_F16, ORC_F32};
    case CONV_B2F: return {8, 16, 4, ORC_BF16, ORC_F32};
    case CONV_F2H: return {32, 16, 8, ORC_F32, ORC_F16};
    case CONV_F2B: return {32, 16, 8, ORC_F32, ORC_BF16};
    case CONV_D2F: return {32, 16, 4, ORC_F64, ORC_F32};
    case CONV_F2D: return {8, 16, 2, ORC_F32, ORC_F64};
    case CONV_D2H: return {32, 8, 4, ORC_F64, ORC_F16};
    case CONV_D2B: return {32, 8, 4, ORC_F64, ORC_BF16};
    case CONV_H2D: return {4, 16, 2, ORC_F16, ORC_F64};
    case CONV_E5H: return {8, 16, 8, ORC_F8_E5M2, ORC_F16};
    case CONV_E5B: return {8, 16, 8, ORC_F8_E5M2, ORC_BF16};
    case CONV_E5F: return {4, 16, 4, ORC_F8_E5M2, ORC_F32};
    case CONV_E4H: return {8, 16, 8, ORC_F8_E4M3, ORC_F16};
    case CONV_E4B: return {8, 16, 8, ORC_F8_E4M3, ORC_BF16};
    case CONV_E4F: return {4, 16, 4, ORC_F8_E4M3, ORC_F32};
    default: return {4, 16, 2, ORC_BF16, ORC_F64};
    }
}

uint32_t fast_div(uint32_t n, uint32_t m, uint32_t s) { return uint32_t((uint64_t(uint32_t(n << 1)) * m) >> 32) >> s; }

void convert_and_store(const ConvInfo &ci, const uint8_t *units, uint32_t n_units, uint8_t *dst)
{
    if (ci.sd == ci.dd) std::memcpy(dst, units, n_units * (ci.cs / ci.ch));
    else if (orc_cast_array(units, n_units, ci.sd, ci.dd, dst) != ORC_OK) violation("conversion refused", 0, 0);
}

// One piece's chunk c, as the vector, spliced and gather kernels move it.
void run_chunk(uint32_t path, bool byte_variant, const ConvInfo &ci, const fst::DevDesc &d, const uint8_t *raw, uint32_t c)
{
    using namespace fst;
    const uint32_t US = ci.cs / ci.ch;
    uint8_t buf[32];
    const uint8_t *src = raw + d.src_off;
    if (path == PATH_VEC) {
        const uint8_t *s;
        if (d.units_per_row == 0) {
            s = src + uint64_t(c) * ci.cs;
        } else {
            const uint32_t r = fast_div(c, d.div_m, d.div_s);
            if (r != c / d.units_per_row) violation("fast_div differs from the division", c, d.units_per_row);
            s = src + uint64_t(r) * d.src_stride + uint64_t(c - r * d.units_per_row) * ci.cs;
        }
        if (byte_variant) check_dword_read(s, ci.cs, "vector chunk (byte-aligned source) reads outside the source");
        else check_read(s, ci.cs, 4, "vector chunk (dword-aligned source) reads outside the source or off a dword");
        std::memcpy(buf, s, ci.cs);
    } else {
        const uint32_t u0 = d.unit0 + c * ci.ch;
        if (uint64_t(d.unit0) + uint64_t(c) * ci.ch >= (1ull << 31)) violation("unit index beyond 2^31", d.unit0, c);
        const uint32_t upr = d.units_per_row;
        if (path == PATH_SPLICE) {
            const uint32_t r = fast_div(u0, d.div_m, d.div_s);
            if (r != u0 / upr) violation("fast_div differs from the division", u0, upr);
            const uint32_t col = u0 - r * upr;
            const uint8_t *row = src + uint64_t(r) * d.src_stride;
            check_dword_read(row + uint64_t(col) * US, ci.cs, "spliced chunk: first read outside the source");
            const uint32_t k = upr - col;
            if (k < ci.ch) {
                check_dword_read(row + d.src_stride - k * US, ci.cs, "spliced chunk: second read outside the source");
                if (d.src_stride < uint64_t(k) * US) violation("spliced chunk: row shorter than the overlap", k, d.src_stride);
            }
            for (uint32_t j = 0; j < ci.ch; ++j) {
                const uint8_t *p = j < k ? row + uint64_t(col + j) * US : row + d.src_stride + uint64_t(j - k) * US;
                std::memcpy(buf + j * US, p, US);
            }
        } else {   // PATH_GATHER
            const uint32_t step = ci.sd == ci.dd ? d.grain : 1;                            // units fetched per load
            const uint32_t load_bytes = step * US;
            const bool aligned = ci.sd == ci.dd ? true : d.grain >= US;
            for (uint32_t j = 0; j < ci.ch; j += step) {
                const uint32_t u = u0 + j;
                const uint32_t r = fast_div(u, d.div_m, d.div_s);
                if (r != u / upr) violation("fast_div differs from the division", u, upr);
                const uint32_t col = u - r * upr;
                if (col + step > upr) violation("gather load straddles a row end", col, upr);
                const uint8_t *p = src + uint64_t(r) * d.src_stride + uint64_t(col) * US;
                check_read(p, load_bytes, aligned ? load_bytes : 1, "gather load outside the source or misaligned");
                std::memcpy(buf + j * US, p, load_bytes);
            }
        }
    }
    uint8_t *t = reinterpret_cast<uint8_t *>(d.dst) + uint64_t(c) * ci.cd;
    check_write(t, ci.cd, ci.cd == 8 ? 8 : 16, "chunk store outside its output or misaligned");
    if (g_violations) return;
    convert_and_store(ci, buf, ci.ch, t);
    ++g_chunks;
}

// A tile of a gathered piece that goes through LDS: the wavefront reads everything from the dword of
// the tile's first wanted byte to the dword of its last one into an area of GATHER_LDS_BYTES, and
// every chunk is put together from bytes of that area.
void run_staged_gather_tile(const ConvInfo &ci, const fst::DevDesc &d, const uint8_t *raw, uint32_t c0, uint32_t n)
{
    using namespace fst;
    const uint32_t US = ci.cs / ci.ch, upr = d.units_per_row;
    if (d.src_stride >= GATHER_LDS_BYTES) { violation("staged gather: stride too long", d.src_stride, 0); return; }
    const uint32_t stride = uint32_t(d.src_stride);
    if (uint64_t(d.unit0) + (uint64_t(c0) + n) * ci.ch > (1ull << 31)) violation("unit index beyond 2^31", d.unit0, c0);
    const uint32_t t0 = d.unit0 + c0 * ci.ch, t1 = t0 + n * ci.ch - 1;
    const uint32_t r0 = fast_div(t0, d.div_m, d.div_s), r1 = fast_div(t1, d.div_m, d.div_s);
    if (r0 != t0 / upr || r1 != t1 / upr) violation("fast_div differs from the division", t0, upr);
    const uint32_t col0 = t0 - r0 * upr, col1 = t1 - r1 * upr;
    const uint8_t *base = raw + d.src_off;
    const uintptr_t first = uintptr_t(base) + uint64_t(r0) * stride + col0 * US;
    const uint8_t *from = reinterpret_cast<const uint8_t *>(first & ~uintptr_t(3));
    const uint32_t lead = uint32_t(first) & 3u;
    const uint32_t span = (lead + (r1 - r0) * stride + (col1 + 1 - col0) * US + 3u) & ~3u;
    if (span > GATHER_LDS_BYTES) { violation("staged gather: the tile's span exceeds the LDS area", span, c0); return; }
    check_read(from, span, 4, "staged gather: span outside the source");
    if (g_violations) return;
    std::vector<uint8_t> area(from, from + span);
    ++g_staged;
    for (uint32_t lane = 0; lane < n && !g_violations; ++lane) {
        const uint32_t c = c0 + lane, u0 = d.unit0 + c * ci.ch;
        uint8_t buf[32];
        for (uint32_t j = 0; j < ci.ch; ++j) {
            const uint32_t u = u0 + j, r = fast_div(u, d.div_m, d.div_s);
            if (r != u / upr) violation("fast_div differs from the division", u, upr);
            const uint32_t at = lead + (r - r0) * stride + (u - r * upr) * US - col0 * US;
            if (at + US > span) { violation("staged gather: unit outside the area", at, span); return; }
            std::memcpy(buf + j * US, area.data() + at, US);
        }
        uint8_t *t = reinterpret_cast<uint8_t *>(d.dst) + uint64_t(c) * ci.cd;
        check_write(t, ci.cd, ci.cd == 8 ? 8 : 16, "chunk store outside its output or misaligned");
        if (g_violations) return;
        convert_and_store(ci, buf, ci.ch, t);
        ++g_chunks;
    }
}

void run_elem_tile(const ConvInfo &ci, const fst::DevDesc &d, const uint8_t *raw, uint32_t t)
{
    using namespace fst;
    const uint32_t ES = ci.cs / ci.ch, ED = ci.cd / ci.ch;
    const uint64_t e0 = uint64_t(t) * ELEM_TILE_UNITS;
    const uint32_t n = (t + 1 == d.n_tiles) ? uint32_t(d.n_units - e0) : ELEM_TILE_UNITS;
    if (n == 0 || n > ELEM_TILE_UNITS) violation("element tile length", n, t);
    for (uint32_t i = 0; i < n && !g_violations; ++i) {
        const uint64_t g = uint64_t(d.unit0) + e0 + i;
        const uint64_t r = g / d.units_per_row;
        const uint8_t *s = raw + d.src_off + r * d.src_stride + (g - r * d.units_per_row) * ES;
        check_read(s, ES, 1, "element read outside the source");
        uint8_t *o = reinterpret_cast<uint8_t *>(d.dst) + (e0 + i) * ED;
        check_write(o, ED, ED, "element store outside its output or misaligned");
        if (g_violations) return;
        convert_and_store(ci, s, 1, o);
    }
}

}  // namespace

extern "C" {
// Test hooks: the byte ranges launches may read and write; counters.
void fst_test_set_source(const void *p, uint64_t len)
{
    std::lock_guard<std::mutex> lock(g_mu);
    // a source buffer must be readable up to the next multiple of 4 bytes (the contract of fst_materialize)
    g_source = {uintptr_t(p), (uintptr_t(p) + len + 3) & ~uintptr_t(3)};
}
void fst_test_clear_outputs(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_outputs.clear();
    g_chunks = g_violations = g_direct = g_staged = 0;
    g_first_violation[0] = 0;
}
void fst_test_add_output(const void *p, uint64_t len)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_outputs.push_back({uintptr_t(p), uintptr_t(p) + len});
}
uint64_t fst_test_violations(void) { return g_violations; }
uint64_t fst_test_direct_tiles(void) { return g_direct; }
uint64_t fst_test_staged_tiles(void) { return g_staged; }
const char *fst_test_first_violation(void) { return g_first_violation; }
}

namespace fst {

int launch_class_kernels(uint32_t cls, const DevDesc *descs, const uint32_t *hints, uint32_t n_tiles, uint32_t hint_shift,
                         const void *raw_dev, void *)
{
    if (n_tiles == 0) return FST_OK;
    std::lock_guard<std::mutex> lock(g_mu);
    const uint32_t path = class_path(cls), conv = class_conv(cls);
    const bool byte_variant = path == PATH_VEC && cls % 2 == 1;
    const ConvInfo ci = conv_info(conv);
    const uint8_t *raw = static_cast<const uint8_t *>(raw_dev);
    std::vector<uint8_t> seen(n_tiles, 0);
    for (const LaunchPart &part : split_launch(workgroups_of(path, n_tiles)))
        for (uint32_t blk = 0; blk < part.n_wg; ++blk) {
            const uint32_t pos = part.wg_base + (path == PATH_ELEM ? blk : tile_of_workgroup(blk, part.n_wg));
            for (uint32_t wave = 0; wave < (path == PATH_ELEM ? 1u : WG_TILES); ++wave) {
                const uint32_t b = path == PATH_ELEM ? pos : pos * WG_TILES + wave;
                if (b < n_tiles && seen[b]++) violation("tile visited twice", b, 0);
                // find_piece
                uint32_t lo = hints[b >> hint_shift], hi = hints[(b >> hint_shift) + 1];
                if (b < n_tiles && hi - lo <= 1) ++g_direct;
                while (lo < hi) {
                    const uint32_t mid = (lo + hi + 1) >> 1;
                    if (descs[mid].tile0 <= b) lo = mid; else hi = mid - 1;
                }
                const DevDesc &d = descs[lo];
                if (b >= n_tiles) {         // a spare tile of the last workgroup: must show as past the end of its piece
                    if (b < d.tile0 || b - d.tile0 < d.n_tiles) violation("spare tile lands inside a piece", b, lo);
                    continue;
                }
                if (b < d.tile0 || b - d.tile0 >= d.n_tiles) { violation("hint table names the wrong piece", b, lo); continue; }
                const uint32_t t = b - d.tile0;
                if (path == PATH_ELEM) { run_elem_tile(ci, d, raw, t); continue; }
                const uint32_t c0 = t * VEC_TILE_UNITS;
                const uint32_t n = (t + 1 == d.n_tiles) ? uint32_t(d.n_units) - c0 : VEC_TILE_UNITS;
                if (n == 0 || n > VEC_TILE_UNITS) violation("tile length", n, t);
                if (path == PATH_GATHER && d.staged) { run_staged_gather_tile(ci, d, raw, c0, n); continue; }
                for (uint32_t lane = 0; lane < n && !g_violations; ++lane) run_chunk(path, byte_variant, ci, d, raw, c0 + lane);
            }
        }
    for (uint32_t b = 0; b < n_tiles; ++b)
        if (!seen[b]) violation("tile never visited", b, 0);
    if (g_violations) return fail(FST_E_RANGE, "table interpreter: %s", g_first_violation);
    return FST_OK;
}

}  // namespace fst
