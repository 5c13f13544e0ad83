// Internal structures shared by the host parts (parser, planner, stager) and the kernel launcher.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <map>
#include <mutex>
#include <string>
#include <unordered_map>
#include <utility>
#include <vector>

#include "fst.h"

namespace fst {

int fail(int status, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

struct Tensor {
    std::string name;
    int32_t dtype = 0;
    int32_t ndim = 0;
    uint64_t shape[FST_MAX_DIMS] = {};
    uint64_t begin = 0, end = 0;
};

}  // namespace fst

struct fst_header {
    uint64_t n_json = 0;
    uint64_t file_size = 0;
    std::vector<fst::Tensor> tensors;                      // ordered by offset
    std::unordered_map<std::string, size_t> index;          // name -> position in `tensors`
    std::vector<std::pair<std::string, std::string>> metadata;
};

namespace fst {

// How a descriptor's rows are moved.  The vector path moves whole chunks (16 bytes when nothing
// is converted, 2 to 8 elements otherwise: conv_chunk_elems) of rows that are a whole number
// of chunks.  The spliced path serves rows that are not, but are at least one chunk long: its
// chunks are cut from the output stream, so a chunk may take its first units from the end of one
// row and the rest from the start of the next.  The gather path serves rows shorter than a chunk:
// a chunk of the output stream is put together from several rows, unit by unit.  The element path
// moves single elements: the few units before the first 16-byte boundary of the output and after
// the last whole chunk of a piece.
enum Path : uint32_t { PATH_VEC = 0, PATH_ELEM = 1, PATH_SPLICE = 2, PATH_GATHER = 3, PATH_COUNT = 4 };

// Conversion kinds (Section III-B).  COPY moves bytes and ignores the element type.  H = binary16,
// B = bfloat16, F = binary32, D = binary64; E5 and E4 = the 8-bit floats E5M2 and E4M3 (widened only).
enum Conv : uint32_t {
    CONV_COPY = 0, CONV_H2B, CONV_B2H, CONV_H2F, CONV_B2F, CONV_F2H, CONV_F2B, CONV_D2F, CONV_F2D,
    CONV_D2H, CONV_D2B, CONV_H2D, CONV_B2D, CONV_E5H, CONV_E5B, CONV_E5F, CONV_E4H, CONV_E4B, CONV_E4F, CONV_COUNT
};

// One unit of kernel work, as uploaded to the device (64 bytes).
struct DevDesc {
    uint64_t src_off;        // byte offset of row 0 from the source pointer of the launch
    uint64_t src_stride;     // bytes between rows
    uint64_t dst;            // device address of the first output byte of this piece
    uint64_t n_units;        // VEC: chunks in total (rows * units_per_row); SPLICE, GATHER: chunks; ELEM: elements
    uint32_t units_per_row;  // VEC: chunks per row (0 = one row of any length); SPLICE, GATHER, ELEM: elements per
                             //   row (bytes per row when nothing is converted)
    uint32_t tile0;          // index of this piece's first tile inside its launch
    uint32_t n_tiles;
    uint32_t div_m;          // division by units_per_row as a multiplication: see fast_div
    uint32_t div_s;          //   (0 = divisor is 1)
    uint32_t unit0;          // SPLICE, GATHER: the piece's first unit is unit `unit0` of the row at src_off
    uint32_t grain;          // GATHER: every unit's source address is a multiple of this many bytes (1, 2, 4 or 8)
    uint32_t staged;         // GATHER: 1 = the source span of every tile fits the wavefront's LDS area (see GATHER_LDS_BYTES)
};
static_assert(sizeof(DevDesc) == 64, "DevDesc is 64 bytes");

// Host-side piece: a DevDesc minus the output address, plus bookkeeping.
struct Piece {
    uint32_t output = 0;
    uint32_t path = PATH_VEC;
    uint32_t conv = CONV_COPY;
    bool dword_aligned = true;   // every chunk source address is a multiple of 4
    uint64_t src_file_off = 0;   // file offset of row 0
    uint64_t src_stride = 0;
    uint64_t dst_off = 0;        // byte offset inside the output
    uint64_t n_units = 0;
    uint32_t units_per_row = 0;
    uint32_t unit0 = 0;          // SPLICE, GATHER: first unit, counted from the start of the row at src_file_off
    uint32_t grain = 1;          // GATHER: alignment every unit's source address has, by the geometry alone
    bool staged = false;         // GATHER: tiles are read through LDS
    uint64_t src_span = 0;       // bytes from row 0 start to the end of the last row
    uint64_t read_bytes = 0, write_bytes = 0;
    // where the source bytes are staged: index of the extent inside the piece's group (for bytes
    // in the group's plain ranges it is looked up when the group is closed; own_extent: an extent
    // staged for this piece's rows alone).  compact: the extent holds several rows back to back
    // and the piece is laid out over that image: src_file_off is then the offset of row 0 inside
    // the image, not in the file.
    uint32_t extent = 0;
    bool own_extent = false;
    bool compact = false;
};

// A byte range [lo, hi) of a file that is staged; in the slot layout its first byte sits at
// slot_off.  A compacted extent (n_rows > 1) stages only n_rows segments of row_bytes each, the
// r-th starting at file offset lo + r*stride, and its image holds them back to back.
struct Extent {
    uint64_t lo = 0, hi = 0, slot_off = 0;
    uint64_t row_bytes = 0, n_rows = 1, stride = 0;      // row_bytes = hi - lo for a plain extent
    bool compact() const { return n_rows > 1; }
    uint64_t image_bytes() const { return n_rows * row_bytes; }
};

struct Group {
    uint32_t file = 0;
    uint64_t phase = 0;                     // raw_base[file] % 256: file byte x sits at an address = x + phase (mod 256) in every layout
    uint64_t lo = 0, hi = 0;                // first and last+1 staged file byte
    std::vector<Extent> extents;            // plain extents, ascending and disjoint, then the compacted ones
    std::map<uint64_t, uint64_t> plain;     // while the group is built: plain ranges lo -> hi (extents: compacted only)
    uint64_t slot_bytes = 0;                // slot space the extents take
    uint64_t packed_off = 0;                // packed layout: where the group's slot image starts
    size_t desc_begin = 0, desc_end = 0;    // public descriptors [begin, end)
    std::vector<Piece> pieces;              // sorted by launch class
    size_t hint_bound = 0;                  // upper bound of this group's hint entries
    uint64_t read_bytes = 0, write_bytes = 0;
};

struct Output {
    fst_output_info info;
    // geometry of the request, kept so that groups can be re-cut
    int32_t src_dtype = 0;
    uint64_t src_file_off = 0;   // file offset of row 0 of the rank's share
    uint64_t src_stride = 0;
    uint64_t row_elems = 0;
    uint64_t n_rows = 0;
    uint64_t tensor_begin = 0;   // file offset of the stored tensor (for ordering)
};

// Launch classes: (conv, byte-aligned?) for the vector path, then one class per conversion for each
// of the element, spliced and gather paths.
constexpr uint32_t N_CLASSES = CONV_COUNT * (PATH_COUNT + 1);
inline uint32_t launch_class(const Piece &p)
{
    if (p.path == PATH_VEC) return p.conv * 2 + (p.dword_aligned ? 0 : 1);
    return CONV_COUNT * (p.path + 1) + p.conv;
}

// Geometry of the kernels, fixed at compile time and needed by the planner to count tiles.
// The vector, spliced and gather kernels run 1024-thread workgroups (16 wavefronts) in which every
// lane moves one chunk.  One chunk per lane measured fastest: many short-lived wavefronts keep more
// requests in flight than fewer wavefronts with several loads each.  A tile is what one wavefront
// moves, 64 chunks (1 KiB of 16-byte chunks), and a workgroup takes WG_TILES consecutive tiles of
// the launch, each wavefront looking up the piece of its own tile: a tensor of a few KiB then
// wastes at most 63 lanes, not most of a workgroup, and a workgroup can span several small tensors.
constexpr uint32_t VEC_BLOCK_THREADS = 1024;
constexpr uint32_t WAVE = 64;
constexpr uint32_t VEC_TILE_UNITS = WAVE;                                     // chunks per tile
constexpr uint32_t WG_TILES = VEC_BLOCK_THREADS / WAVE;                       // tiles per workgroup
constexpr uint32_t ELEM_BLOCK_THREADS = 256;
constexpr uint32_t ELEM_TILE_UNITS = ELEM_BLOCK_THREADS * 16;                 // elements per tile (one workgroup)
inline uint32_t tile_units(uint32_t path) { return path == PATH_ELEM ? ELEM_TILE_UNITS : VEC_TILE_UNITS; }
// Workgroups a launch of n_tiles tiles of `path` needs.
inline uint32_t workgroups_of(uint32_t path, uint32_t n_tiles)
{
    return path == PATH_ELEM ? n_tiles : (n_tiles + WG_TILES - 1) / WG_TILES;
}
// Workgroups are dealt to the 8 XCDs round-robin.  The tile index is permuted so that each XCD
// works on runs of XCD_RUN consecutive tiles (512 KiB of output), which measured faster than both
// tile-by-tile interleaving and giving each XCD one contiguous eighth.
constexpr uint32_t XCD_COUNT = 8;
constexpr uint32_t XCD_RUN = 32;
// A wavefront finds its piece through a hint table with one entry per span of 2^hint_shift tiles
// (the piece that holds the span's first tile) plus a closing entry per launch (its last piece): the
// owner of a tile lies between its span's entry and the next one; when they coincide (a span inside
// one tensor) nothing is searched.  The span is chosen per launch, about the launch's mean piece
// length but at most 1024 tiles (1 MiB of 16-byte chunks): on large tensors spans of 256 KiB
// measured 3 % slower than 1 MiB with a byte-aligned source (more distinct table lines for the
// scalar cache) and spans of 2 to 16 MiB the same, while a launch of thousands of 8 KiB tensors gets
// spans of 8 tiles and one search step at most.
constexpr uint32_t MAX_HINT_SHIFT = 10;
inline uint32_t hint_shift_for(uint32_t n_tiles, uint32_t n_pieces)
{
    uint32_t shift = 0;
    while (shift < MAX_HINT_SHIFT && (uint64_t(2) << shift) * n_pieces <= n_tiles) ++shift;
    return shift;
}
// The work-item count of one dispatch (workgroups x workgroup size) must fit 32 bits, so a launch
// class with more workgroups than MAX_LAUNCH_WORKGROUPS goes out as several launches, each with
// the index of its first workgroup as an argument.  The limit is a whole number of permutation
// spans, so that every launch but the last of a class permutes whole spans (tile_of_workgroup).
constexpr uint32_t MAX_LAUNCH_WORKGROUPS =
    uint32_t(((uint64_t(1) << 32) / VEC_BLOCK_THREADS - 1) / (XCD_COUNT * XCD_RUN) * (XCD_COUNT * XCD_RUN));
struct LaunchPart { uint32_t wg_base, n_wg; };
inline std::vector<LaunchPart> split_launch(uint32_t n_wg, uint32_t max_wg = MAX_LAUNCH_WORKGROUPS)
{
    std::vector<LaunchPart> parts;
    for (uint32_t at = 0; at < n_wg;) {
        const uint32_t n = n_wg - at < max_wg ? n_wg - at : max_wg;
        parts.push_back({at, n});
        at += n;
    }
    return parts;
}
// Workgroup index -> position inside one launch of n_wg workgroups.  Workgroup i runs on XCD
// i % 8; within every span of 8*XCD_RUN workgroups, XCD x gets the positions x*XCD_RUN ..
// x*XCD_RUN+XCD_RUN-1 of the span, in order.  A bijection of [0, n_wg).
#ifdef __HIPCC__
#define FST_HOST_DEVICE __host__ __device__
#else
#define FST_HOST_DEVICE
#endif
FST_HOST_DEVICE inline uint32_t tile_of_workgroup(uint32_t wg, uint32_t n_wg)
{
    constexpr uint32_t SPAN = XCD_COUNT * XCD_RUN;
    if (wg >= n_wg / SPAN * SPAN) return wg;             // the ragged last span keeps its order
    const uint32_t r = wg % SPAN;
    return wg - r + (r % XCD_COUNT) * XCD_RUN + r / XCD_COUNT;
}
// Gathered pieces whose loads would be 4 bytes or less read a tile's whole source span -- the bytes
// from the tile's first to its last wanted byte, the other ranks' columns in between included -- with
// coalesced 16-byte loads into an LDS area of the wavefront, and put the chunks together from there.
// It applies when that span, rounded out to dwords, fits the area for every tile of the piece.
constexpr uint32_t GATHER_LDS_BYTES = 4096;              // per wavefront: 64 KiB per workgroup
inline bool gather_span_fits(uint64_t units_per_tile, uint64_t units_per_row, uint64_t unit_bytes, uint64_t stride)
{
    // a run of units_per_tile units that starts anywhere in a row touches at most this many rows
    const uint64_t rows = (units_per_tile - 1) / units_per_row + 2;
    return stride < GATHER_LDS_BYTES && 3 + (rows - 1) * stride + units_per_row * unit_bytes + 3 <= GATHER_LDS_BYTES;
}
// Vector pieces are cut so that chunk indices inside a piece fit 32 bits.
constexpr uint64_t VEC_PIECE_MAX_UNITS = 1ull << 31;
// Spliced pieces are cut so that element indices inside a piece stay below 2^31.
constexpr uint64_t SPLICE_PIECE_MAX_UNITS = (1ull << 31) - 64;

uint32_t conv_kind(int src_dtype, int dst_dtype);            // CONV_*; CONV_COUNT if unsupported
// Geometry of a conversion, shared by the planner and the kernels: bytes per source and per result
// element (COPY moves bytes: 1 and 1), and the elements of a chunk, which is what a lane moves with
// one 16-byte store when the conversion widens, and 8 elements (4 from binary64) when it narrows or
// keeps the width; COPY: 16 bytes.
constexpr uint32_t conv_src_bytes(uint32_t c)
{
    return (c == CONV_COPY || (c >= CONV_E5H && c <= CONV_E4F)) ? 1
         : (c == CONV_D2F || c == CONV_D2H || c == CONV_D2B) ? 8
         : (c == CONV_F2H || c == CONV_F2B || c == CONV_F2D) ? 4 : 2;
}
constexpr uint32_t conv_dst_bytes(uint32_t c)
{
    return c == CONV_COPY ? 1
         : (c == CONV_F2D || c == CONV_H2D || c == CONV_B2D) ? 8
         : (c == CONV_H2F || c == CONV_B2F || c == CONV_D2F || c == CONV_E5F || c == CONV_E4F) ? 4 : 2;
}
constexpr uint32_t conv_chunk_elems(uint32_t c)
{
    return c == CONV_COPY ? 16
         : conv_dst_bytes(c) > conv_src_bytes(c) ? 16 / conv_dst_bytes(c)
         : conv_src_bytes(c) == 8 ? 4 : 8;
}
static_assert(CONV_E5H + 5 == CONV_E4F, "the 8-bit float conversions are numbered in a row");
// Bytes of output a lane stores at once: 16, or 8 for binary64 -> 16-bit (4 elements of 2 bytes).
// A piece's first output byte must be a multiple of it (16-byte aligned where the chunk is longer).
inline uint32_t conv_store_align(uint32_t conv) { return conv == CONV_D2H || conv == CONV_D2B ? 8 : 16; }

// One kernel launch: pieces [first, first+count) of a device table, all of one launch class, with
// their hint entries [hint_first, ...).
struct LaunchRange { uint32_t cls, first, count, tiles, hint_first, hint_shift; };
inline uint32_t class_path(uint32_t cls) { return cls < CONV_COUNT * 2 ? uint32_t(PATH_VEC) : cls / CONV_COUNT - 1; }
inline uint32_t class_conv(uint32_t cls) { return cls < CONV_COUNT * 2 ? cls / 2 : cls % CONV_COUNT; }
// Host copy of a device table: pieces, hints, and the launches over them.
struct TableImage {
    std::vector<DevDesc> descs;
    std::vector<uint32_t> hints;      // per launch: for every span of tiles the piece (counted from the launch's first)
                                      //   holding the span's first tile, then the launch's last piece
    std::vector<LaunchRange> ranges;
    std::vector<uint8_t> blob;        // what is copied to the device: descs, then hints at table_hint_offset
    // set by fst_prepare: where the blob was uploaded and the source length it was checked against
    const void *dev = nullptr;
    size_t src_len = 0;
    bool prepared = false;
};
// Bytes a table occupies in the workspace: pieces first, hints after them on a 256-byte boundary.
inline size_t table_hint_offset(size_t n_descs) { return (n_descs * sizeof(DevDesc) + 255) / 256 * 256; }
inline size_t table_bytes(size_t n_descs, size_t n_hints)
{
    return (table_hint_offset(n_descs) + n_hints * sizeof(uint32_t) + 255) / 256 * 256;
}

}  // namespace fst

struct fst_plan {
    size_t n_files = 0;
    std::vector<uint64_t> raw_base;
    std::vector<uint64_t> file_size;
    std::vector<fst::Output> outputs;
    std::vector<fst_descriptor> descs;        // public view, grouped
    std::vector<fst::Group> groups;
    uint64_t read_bytes = 0, write_bytes = 0;
    uint64_t min_gap = UINT64_MAX;            // unread file ranges longer than this are not staged
    uint64_t packed_bytes = 0;                // packed layout: length of all slot images side by side
    bool has_compact = false;                 // some extent is compacted: no resident layout
    size_t max_group_pieces = 0;
    size_t total_pieces = 0;
    // Host copies of the device tables that fst_materialize uploads, one per group index (and one
    // for "all groups").  They belong to the plan so that an enqueued upload never outlives its
    // source; re-cutting the groups drops them.
    mutable std::mutex image_mu;
    mutable std::map<size_t, fst::TableImage> images;
    // the same for calls that upload into the library's built-in workspace (fst_materialize_static)
    mutable std::map<size_t, fst::TableImage> builtin_images;
};

namespace fst {
int build_groups(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes, uint64_t min_segment_bytes);

// Device table for groups [g0, g1) merged into one launch set.  layout: FST_LAYOUT_RESIDENT,
// FST_LAYOUT_SLOT (sources addressed inside the slot image of group g0; g1 == g0+1) or
// FST_LAYOUT_PACKED (the slot images of all groups side by side).
int build_image(const fst_plan *p, size_t g0, size_t g1, void *const *out_ptrs, size_t src_len, int layout,
                TableImage &image);
// table_dev: where image.blob was copied.
int launch_ranges(const TableImage &image, const void *table_dev, const void *src_dev, void *stream);
// fst_materialize with the table kept in `images` (the plan's map for caller workspaces or the one
// for the built-in workspace).
int materialize_into(const void *src_dev, size_t src_len, const fst_plan *p, size_t group, void *const *out_ptrs,
                     void *ws, size_t ws_len, void *stream, int layout, bool builtin);
// Launch the kernels of one class.  descs_dev / hints_dev: the class's arrays on the device.
int launch_class_kernels(uint32_t cls, const DevDesc *descs_dev, const uint32_t *hints_dev, uint32_t n_tiles,
                         uint32_t hint_shift, const void *raw_dev, void *stream);
}  // namespace fst
