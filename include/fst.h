/*
 * fst -- device-side deserialization of safetensors files on one AMD MI355X (gfx950).
 *
 * Method: "Speeding up Model Loading with fastsafetensors" (arXiv 2505.23072).  Whole files, or
 * large groups of their on-disk bytes, are copied verbatim into one raw device buffer (Section
 * III-A, aggregated tensor deserialization); GPU kernels then turn the raw bytes into typed,
 * aligned tensors: they fix the alignment the format does not define, convert the element type
 * in the same pass, and keep one rank's partition of a tensor (Section III-B, GPU offloading).
 *
 * C ABI.  Every function returns FST_OK (0) or a negative fst_status; none aborts or throws.
 * fst_last_error() gives a human-readable message for the calling thread's last failure.
 * "host" / "device" in a comment says which memory a pointer refers to.
 *
 * Ownership: the library owns fst_header, fst_plan and fst_stager objects (host memory; the
 * stager also owns pinned host memory).  The caller owns ALL device memory -- raw buffer,
 * outputs, workspace -- and the streams; the library never allocates or frees device memory and
 * never synchronises a stream unless the function says so.  Buffers passed to an enqueueing call
 * must stay alive until the stream has passed that point (the paper's rule that users keep the
 * buffers until close(), Section III-C).
 */
#ifndef FST_H
#define FST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FST_MAX_DIMS 8
#define FST_MAX_HEADER_BYTES 100000000ull   /* largest accepted JSON length N */
#define FST_OUTPUT_ALIGN 256                /* required alignment of every output pointer */
#define FST_RAW_ALIGN 256                   /* required alignment of raw buffers and file bases */
#define FST_ALL_GROUPS ((size_t)-1)

typedef enum fst_status {
    FST_OK = 0,
    FST_E_TRUNCATED = -1,      /* fewer bytes given than the header needs */
    FST_E_HEADER_SIZE = -2,    /* N < 2, N > FST_MAX_HEADER_BYTES, or 8+N beyond the file */
    FST_E_JSON = -3,           /* header text is not well-formed JSON / UTF-8 */
    FST_E_SCHEMA = -4,         /* JSON that is not a layout definition */
    FST_E_DTYPE = -5,          /* unknown dtype string */
    FST_E_SIZE_MISMATCH = -6,  /* end - begin != prod(shape) * sizeof(dtype) */
    FST_E_OFFSETS = -7,        /* tensors do not tile the body exactly */
    FST_E_DUP_NAME = -8,       /* a key twice in one file, or one name in two files */
    FST_E_NOT_FOUND = -9,      /* requested name is in no file */
    FST_E_SHARD = -10,         /* bad shard dim / rank / world / blocks, or dim not divisible */
    FST_E_CAST = -11,          /* conversion other than among {F64, F32, F16, BF16} */
    FST_E_ALIGN = -12,         /* a pointer or base offset misses its required alignment */
    FST_E_RANGE = -13,         /* too many dims, buffer too small, index out of range */
    FST_E_HIP = -14,           /* a HIP runtime call failed */
    FST_E_NOMEM = -15,
    FST_E_IO = -16,            /* a read callback / pread failed */
    FST_E_ARG = -17            /* NULL or inconsistent argument */
} fst_status;

/* Element types of the container (Section II-A: "data types").  FST_KEEP = no conversion. */
typedef enum fst_dtype {
    FST_KEEP = -1,
    FST_F64 = 0, FST_F32, FST_F16, FST_BF16, FST_F8_E5M2, FST_F8_E4M3,
    FST_I64, FST_I32, FST_I16, FST_I8,
    FST_U64, FST_U32, FST_U16, FST_U8,
    FST_BOOL,
    FST_DTYPE_COUNT
} fst_dtype;

typedef struct fst_header fst_header;   /* parsed layout definition of one file */
typedef struct fst_plan fst_plan;       /* load plan: outputs, copy descriptors, groups */
typedef struct fst_stager fst_stager;   /* pinned-host staging ring */

const char *fst_last_error(void);
const char *fst_status_name(int status);
const char *fst_dtype_name(int dtype);          /* "BF16", ...; NULL if unknown */
int fst_dtype_from_name(const char *s, size_t len);   /* dtype or FST_E_DTYPE */
size_t fst_dtype_size(int dtype);               /* bytes per element; 0 if unknown */

/* ---------------------------------------------------------------- header (Section II-A, Fig. 1)
 *
 * A file is: 8 bytes holding the size N of the header text (read as little-endian u64), N bytes
 * of JSON mapping each tensor key to {dtype, shape, data_offsets:[begin,end]} (offsets relative
 * to the first body byte, i.e. file offset 8+N), then the tensor bytes.
 */

/* first8 (host): at least 8 bytes.  Writes N.  FST_E_TRUNCATED if nbytes < 8. */
int fst_header_len(const void *first8, size_t nbytes, uint64_t *n_out);

/*
 * bytes (host): the first 8+N bytes of a file (more is fine); file_size: size of the whole file.
 * Validates: N in [2, FST_MAX_HEADER_BYTES] and 8+N <= file_size; text starts with '{', is
 * well-formed JSON in UTF-8 (only white space may follow the closing brace), at most three
 * levels deep, no key twice; every entry except "__metadata__" (string -> string map, kept) has
 * exactly dtype/shape/data_offsets; at most FST_MAX_DIMS dims; end-begin = prod(shape)*size; and
 * the byte ranges, ordered by begin, tile the body [0, file_size-8-N) with no hole or overlap.
 * On success *out is a new header (free with fst_header_free); on failure *out = NULL.
 */
int fst_parse_header(const void *bytes, size_t nbytes, uint64_t file_size, fst_header **out);

typedef struct fst_tensor_info {
    const char *name;                /* borrowed from the header; UTF-8, NUL-terminated */
    size_t name_len;
    int32_t dtype;                   /* fst_dtype */
    int32_t ndim;
    uint64_t shape[FST_MAX_DIMS];
    uint64_t begin, end;             /* relative to the body */
} fst_tensor_info;

size_t fst_header_count(const fst_header *h);
/* Tensors are indexed in order of their offsets.  FST_E_RANGE if i >= count. */
int fst_header_tensor(const fst_header *h, size_t i, fst_tensor_info *out);
/* Index of the tensor called `name`, or FST_E_NOT_FOUND. */
int64_t fst_header_find(const fst_header *h, const char *name);
uint64_t fst_header_body_offset(const fst_header *h);   /* 8 + N */
/* The raw_base phase (below FST_RAW_ALIGN) that puts the first byte after the header, and with it
 * every tensor whose offset in the body is a multiple of 4 or 16, on such a boundary in device
 * memory: -(8 + N) modulo FST_RAW_ALIGN.  See fst_plan_create. */
uint64_t fst_aligned_phase(const fst_header *h);
uint64_t fst_header_file_size(const fst_header *h);
size_t fst_header_metadata_count(const fst_header *h);
int fst_header_metadata(const fst_header *h, size_t i, const char **key, const char **value);
void fst_header_free(fst_header *h);

/* ---------------------------------------------------------------- plan
 *
 * A request asks for one named tensor as one rank sees it:
 *   dst_dtype  FST_KEEP, or a floating-point type other than the stored one: any pair among
 *              F64, F32, F16 and BF16 (conversion in the same pass as the copy, Section III-B;
 *              one rounding, to nearest even, also from F64 to a 16-bit type); or F16, BF16 or F32
 *              for a tensor stored as F8_E5M2 or F8_E4M3 (the 8-bit floats of Section VI; exact).
 *              Any other pair with differing types: FST_E_CAST.
 *   shard_dim  -1 = whole tensor; d >= 0 = the rank's equal share of dimension d (Section III-B).
 *              Column-wise split of an input projection = dim 0 of the stored [out, in] matrix,
 *              row-wise split of an output projection = dim 1 (Section II-A).
 *   blocks     1, or b > 1 with shard_dim 0: dimension 0 is b stacked sub-tensors (fused QKV);
 *              each is split by rank and the rank's parts are concatenated in block order.
 *   rank       -1 = the rank given to fst_plan_create; r >= 0 = this request is rank r's share.
 *              Asking for one name once per rank yields every rank's share from one pass over
 *              the raw bytes: the single-GPU half of the paper's scatter (Section III-B, Fig. 6).
 * shape[shard_dim] must be divisible by blocks*world (FST_E_SHARD otherwise; no padding).
 */
typedef struct fst_request {
    int32_t dst_dtype;
    int32_t shard_dim;
    int32_t blocks;
    int32_t rank;
} fst_request;

/*
 * hdrs[f] (host): header of file f.  raw_base[f]: byte offset inside the raw device buffer at
 * which byte 0 of file f lands when files are resident; a tensor's bytes then start at raw +
 * raw_base[f] + 8 + N_f + begin, at whatever alignment that gives.  Any value is allowed, and
 * raw_base[f] % FST_RAW_ALIGN is the phase of file f in every layout: file byte x sits at an
 * address congruent to x + raw_base[f] modulo FST_RAW_ALIGN, staged resident, in a slot or
 * packed.  A multiple of FST_RAW_ALIGN keeps the alignment the bytes have in the file; a caller
 * that wants the tensor data itself aligned (the kernels read 4-byte aligned sources with fewer
 * loads) picks raw_base[f] congruent to -(8 + N_f): fst_aligned_phase(hdr).  names[i] (host, NUL-terminated UTF-8) with reqs[i]; a name must exist in
 * exactly one file (FST_E_NOT_FOUND / FST_E_DUP_NAME).  The plan copies what it needs; hdrs may
 * be freed afterwards.  Output i of the plan belongs to names[i].
 */
int fst_plan_create(const fst_header *const *hdrs, const uint64_t *raw_base, size_t n_files,
                    const char *const *names, const fst_request *reqs, size_t n_names,
                    int32_t rank, int32_t world, fst_plan **out);

/* Same request for every name: fst_plan(names, target dtype, shard dim, rank, world). */
int fst_plan_uniform(const fst_header *const *hdrs, const uint64_t *raw_base, size_t n_files,
                     const char *const *names, size_t n_names, int32_t dst_dtype,
                     int32_t shard_dim, int32_t rank, int32_t world, fst_plan **out);

typedef struct fst_output_info {
    int32_t dtype;
    int32_t ndim;
    uint64_t shape[FST_MAX_DIMS];    /* shape of the rank's result */
    uint64_t nbytes;                 /* contiguous, row-major */
    uint32_t align;                  /* FST_OUTPUT_ALIGN */
    uint32_t file;                   /* file that stores the tensor */
} fst_output_info;

size_t fst_plan_output_count(const fst_plan *p);
int fst_plan_output(const fst_plan *p, size_t i, fst_output_info *out);

/*
 * Groups.  A group is a byte range [lo, hi) of one file together with the copy work whose source
 * bytes all lie inside it.  Groups are the unit that is staged and then materialized, so that
 * kernels run while later bytes are still in flight.  A new plan has one group per file.
 * fst_plan_set_groups re-cuts: tensors are taken in file order and a group is closed before it
 * would exceed max_group_bytes; a tensor larger than that is cut between source rows (and inside
 * a row, at multiples of 256 elements, when one row alone is too large).  max_group_bytes = 0
 * means one group per file.  Invalidates earlier group indices.
 *
 * Resident layout: byte o of file f is at raw + raw_base[f] + o.
 * Slot layout: the group's staged bytes are alone in a slot.  A group stages one or more extents
 *   (byte ranges of its file); byte o of extent e is at slot + e.slot_offset + (o - e.lo), where
 *   e.slot_offset % FST_RAW_ALIGN == (e.lo + raw_base[f]) % FST_RAW_ALIGN, so every source has the
 *   alignment it has in the resident layout; the slot must hold slot_bytes.
 *
 * Packed layout: the slot images of all groups side by side in one buffer of
 *   fst_plan_packed_bytes: group g's image starts at fst_group_info.packed_offset (a multiple of
 *   FST_RAW_ALIGN).  What the slot layout is to a checkpoint that streams through device memory,
 *   the packed layout is to one whose staged bytes stay: only what is staged takes room.
 *
 * fst_plan_set_groups stages, per group, everything from its first to its last needed byte as one
 * extent (whole files when every tensor is requested: Section III-A).  fst_plan_set_groups_sparse
 * additionally leaves out file ranges that no requested piece reads when they are longer than
 * min_gap_bytes -- the other ranks' shares of dim-0 partitions, unrequested tensors.  Section
 * III-B warns that selecting each rank's ranges degrades into many small scattered reads: a large
 * min_gap_bytes (megabytes) keeps every extent large.  In the resident layout the skipped ranges
 * of the raw buffer are simply never written nor read.
 *
 * fst_plan_set_groups_compact goes one step further for strided shares (a partition along an inner
 * dimension: one segment per row; the blocks of a fused matrix): when a row segment is at least
 * min_segment_bytes long, the stager reads the segments one by one and puts them back to back into
 * the slot image (a compacted extent), so that nothing of the other ranks' columns crosses the bus
 * and the kernels find one contiguous run.  One read per segment is what Section III-B warns
 * against for storage: use it when the source serves small reads well (the page cache, a
 * generator) and keep min_segment_bytes at a few KiB, or pass UINT64_MAX to switch it off.
 * Groups with compacted extents exist in the slot and packed layouts only (FST_E_ARG in the
 * resident layout, whose raw buffer mirrors the files).
 */
int fst_plan_set_groups(fst_plan *p, uint64_t max_group_bytes, size_t *n_groups);
int fst_plan_set_groups_sparse(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes,
                               size_t *n_groups);
int fst_plan_set_groups_compact(fst_plan *p, uint64_t max_group_bytes, uint64_t min_gap_bytes,
                                uint64_t min_segment_bytes, size_t *n_groups);

typedef struct fst_group_info {
    uint32_t file;
    uint32_t n_descriptors;
    uint32_t n_extents;
    uint32_t reserved;
    uint64_t lo, hi;                 /* first staged file byte, last staged file byte + 1 */
    uint64_t slot_bytes;             /* slot layout: bytes of slot the group needs */
    uint64_t staged_bytes;           /* sum of the extents' lengths */
    uint64_t read_bytes;             /* source bytes the kernels read for this group */
    uint64_t write_bytes;            /* output bytes they write */
    uint64_t packed_offset;          /* packed layout: where the group's slot image starts */
} fst_group_info;

/*
 * A plain extent (n_rows == 1) stages file bytes [lo, hi) verbatim; its image is hi - lo bytes.
 * A compacted extent (n_rows > 1) stages n_rows segments of row_bytes, segment r being file bytes
 * [lo + r*stride, lo + r*stride + row_bytes), and its image holds them back to back
 * (n_rows*row_bytes bytes); hi is the end of the last segment.  Either image starts at slot_offset,
 * with slot_offset % FST_RAW_ALIGN == (lo + raw_base[file]) % FST_RAW_ALIGN.  Plain extents of a group are ascending
 * and disjoint; compacted ones may lie inside the file range of others.
 */
typedef struct fst_extent {
    uint64_t lo, hi;                 /* file byte range the extent spans */
    uint64_t slot_offset;            /* slot layout: where byte lo sits in the slot */
    uint64_t row_bytes, n_rows, stride;
} fst_extent;

size_t fst_plan_group_count(const fst_plan *p);
int fst_plan_group(const fst_plan *p, size_t g, fst_group_info *out);
int fst_plan_group_extent(const fst_plan *p, size_t g, size_t i, fst_extent *out);

/*
 * Copy descriptors, exposed for inspection and tests.  One descriptor copies n_rows rows of
 * row_elems elements: row r is read at file offset src_file_off + r*src_stride (bytes) of file
 * `file` and written, converted, at byte dst_off + r*row_elems*sizeof(dst_dtype) of output
 * `output`.  A whole tensor or a dim-0 share is one row; a dim-d share has one row per index
 * combination of the dims before d; a blocked share one row per block.
 */
typedef struct fst_descriptor {
    uint32_t output, file, group;
    int32_t src_dtype, dst_dtype;
    uint64_t src_file_off, src_stride, dst_off, row_elems, n_rows;
} fst_descriptor;

size_t fst_plan_descriptor_count(const fst_plan *p);
int fst_plan_descriptor(const fst_plan *p, size_t i, fst_descriptor *out);

/* Totals over all groups: bytes read from the raw buffer and bytes written to outputs. */
uint64_t fst_plan_read_bytes(const fst_plan *p);
uint64_t fst_plan_write_bytes(const fst_plan *p);
/* Packed layout: bytes of one buffer that holds every group's slot image. */
uint64_t fst_plan_packed_bytes(const fst_plan *p);

/* Device workspace (bytes) that fst_materialize* needs for its tables, for any group or all. */
size_t fst_plan_workspace_bytes(const fst_plan *p);
void fst_plan_free(fst_plan *p);

/* ---------------------------------------------------------------- materialize (Section III-B)
 *
 * Enqueue on `stream` (a hipStream_t; NULL = the default stream) the kernels that turn raw bytes
 * into the plan's outputs for group `group`, or for every group with FST_ALL_GROUPS.  One small
 * host-to-device copy of the tables into dev_workspace precedes the launches; nothing is
 * synchronised.  out_ptrs (host array of output_count device pointers): out_ptrs[i] receives
 * output i, must be FST_OUTPUT_ALIGN-aligned (FST_E_ALIGN) and hold nbytes; outputs of zero bytes
 * may be NULL.  dev_workspace (device): workspace_len >= fst_plan_workspace_bytes, 256-aligned;
 * each call overwrites it, so calls in flight on different streams need separate workspaces.
 * The plan keeps the host copy of the uploaded table: keep the plan alive, and do not re-cut its
 * groups, until the stream has passed this call.
 *
 * fst_materialize: resident layout; raw_dev (device, FST_RAW_ALIGN-aligned) must cover every
 * byte the group reads (FST_E_RANGE if raw_len is too small) and be readable up to the next
 * multiple of 4 bytes.  fst_materialize_slot: slot layout for one group (not FST_ALL_GROUPS).
 * The kernels only read the raw bytes and only write the outputs named by the group.
 */
int fst_materialize(const void *raw_dev, size_t raw_len, const fst_plan *p, size_t group,
                    void *const *out_ptrs, void *dev_workspace, size_t workspace_len, void *stream);
int fst_materialize_slot(const void *slot_dev, size_t slot_len, const fst_plan *p, size_t group,
                         void *const *out_ptrs, void *dev_workspace, size_t workspace_len,
                         void *stream);

/*
 * fst_materialize (resident layout) for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The tables go into a
 * workspace of FST_STATIC_WORKSPACE_BYTES that is built into the library (one per GPU, held until
 * the process ends) instead of a caller-allocated one; the call allocates and frees no device
 * memory.  FST_E_RANGE, before anything is enqueued, when the tables of `group` (or of all groups)
 * may not fit: a piece takes 96 bytes and every MiB of output 8 more.  Every call on a GPU uses
 * that GPU's one workspace and overwrites what the previous call left there: calls on one stream
 * are ordered; calls that overlap on different streams of one GPU race, as do calls from several
 * threads.  Everything else (arguments, checks, kernels, results) is fst_materialize's.
 */
#define FST_STATIC_WORKSPACE_BYTES (4u << 20)
int fst_materialize_static(const void *raw_dev, size_t raw_len, const fst_plan *p, size_t group,
                           void *const *out_ptrs, void *stream);

/*
 * The two halves of fst_materialize, for callers that launch a group more than once or want the
 * launch apart from the table upload (timing the kernels alone; a ring of device slots that all
 * hold the same group layout).
 *
 * fst_prepare builds the table of `group` (or FST_ALL_GROUPS, in the resident and packed layouts)
 * for the given layout and output pointers, checks every source range against src_len exactly as
 * fst_materialize does, and enqueues the upload into dev_workspace on `stream`.  The workspace
 * then belongs to that group until it is prepared again or the groups are re-cut.
 *
 * fst_launch enqueues only the kernels of a prepared group on `stream`: no copy, no allocation,
 * no memset, so the call may be recorded into a HIP graph and replayed whenever new raw bytes have
 * landed in the same buffer.
 * The stream must be the one given to fst_prepare or be ordered after it.  src_dev may differ
 * from call to call (FST_RAW_ALIGN-aligned, device) as long as it holds the same layout and
 * src_len is at least the length the group was prepared with (FST_E_RANGE otherwise); a group
 * that was not prepared is FST_E_ARG.  A group without work is a successful no-op in both.
 */
#define FST_LAYOUT_RESIDENT 0
#define FST_LAYOUT_SLOT 1
#define FST_LAYOUT_PACKED 2
int fst_prepare(const fst_plan *p, size_t group, int32_t layout, size_t src_len, void *const *out_ptrs,
                void *dev_workspace, size_t workspace_len, void *stream);
int fst_launch(const fst_plan *p, size_t group, const void *src_dev, size_t src_len, void *stream);

/* ---------------------------------------------------------------- staging (Section III-A)
 *
 * The fallback path of the paper: file bytes are read into a small DMA-able (pinned) bounce
 * buffer in host memory and copied to the device from there.  Here the bounce buffer is a ring
 * of pinned slots filled by reader threads; hipMemcpyAsync on a copy stream drains it, and each
 * group is materialized on a compute stream as soon as its last byte has landed, so kernels
 * overlap the copies of later groups.  Both streams belong to the stager and are not ordered with
 * any stream of the caller: work the caller has queued on the raw, output, slot or workspace
 * buffers must have finished before fst_stage_* is called (the calls themselves return only after
 * everything they queued has finished).
 */

/* Read callback: fill dst[0..len) with bytes [off, off+len) of file `file`; 0 on success. */
typedef int (*fst_read_fn)(void *ctx, int32_t file, uint64_t off, void *dst, uint64_t len);

typedef struct fst_stager_config {
    uint32_t n_slots;        /* pinned ring slots (0 = 8) */
    uint32_t n_threads;      /* reader threads (0 = 8) */
    uint64_t slot_bytes;     /* bytes per slot (0 = 64 MiB); one host-to-device copy per slot */
} fst_stager_config;

typedef struct fst_stage_stats {
    uint64_t staged_bytes;   /* bytes copied host -> device */
    uint64_t n_copies;
    double seconds_total;    /* wall clock of the call, including the final synchronisation */
    double seconds_read;     /* summed over reader threads: time inside the read callback */
} fst_stage_stats;

/* Allocates the pinned ring (hipHostMalloc) and two streams of default priority. */
int fst_stager_create(const fst_stager_config *cfg, fst_stager **out);
void fst_stager_destroy(fst_stager *s);

/* A ready-made callback over open file descriptors: ctx = (const int *) array of fds, pread. */
int fst_read_fds(void *ctx, int32_t file, uint64_t off, void *dst, uint64_t len);

#define FST_STAGE_NO_KERNELS 1u   /* copy only (measures the pure staging time) */
#define FST_STAGE_NO_READ 2u      /* skip the read callback: copy whatever the slots hold
                                     (measures the pure host-to-device time) */

/*
 * Resident load: stage every group's extents to raw_dev + raw_base[file] + lo and materialize
 * group after group.  Blocks until all work has finished on the device.
 */
int fst_stage_resident(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx,
                       void *raw_dev, size_t raw_len, void *const *out_ptrs,
                       void *dev_workspace, size_t workspace_len, uint32_t flags,
                       fst_stage_stats *stats);

/*
 * Packed load: stage every group's extents into its slot image inside one buffer of
 * fst_plan_packed_bytes (packed_dev, FST_RAW_ALIGN-aligned; FST_E_RANGE if packed_len is less) and
 * materialize group after group.  The buffer then holds exactly what was staged -- with sparse and
 * compacted groups a fraction of the files -- and can be materialized again with
 * fst_prepare/fst_launch in FST_LAYOUT_PACKED.  Blocks until all work has finished on the device.
 */
int fst_stage_packed(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx,
                     void *packed_dev, size_t packed_len, void *const *out_ptrs,
                     void *dev_workspace, size_t workspace_len, uint32_t flags,
                     fst_stage_stats *stats);

/*
 * Streamed load for checkpoints larger than device memory: the raw buffer is a ring of
 * n_dev_slots device slots of dev_slot_bytes each (slot_dev[i], FST_RAW_ALIGN-aligned); group g
 * goes to slot g % n_dev_slots in slot layout and the slot is reused once the kernels of its
 * previous group have finished.  Every group must fit (FST_E_RANGE): cut the plan with
 * fst_plan_set_groups first.  dev_workspace must hold fst_plan_workspace_bytes.
 */
int fst_stage_streamed(fst_stager *s, const fst_plan *p, fst_read_fn read, void *read_ctx,
                       void *const *slot_dev, size_t n_dev_slots, size_t dev_slot_bytes,
                       void *const *out_ptrs, void *dev_workspace, size_t workspace_len,
                       uint32_t flags, fst_stage_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* FST_H */
