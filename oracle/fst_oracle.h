/*
 * CPU oracle for device-side safetensors deserialization -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar reader of the safetensors container (paper Section II-A, Fig. 1) that
 * materializes one tensor at a time: locate its bytes, keep one rank's partition along one
 * dimension (Section II-A last paragraph; Section III-B: equal, same-shaped partitions), convert
 * the element type (Section III-B: conversion in the pass that fixes the alignment) and write the
 * result contiguously in row-major order (Section III-A: strides follow from dtype and shape).
 * Everything is exact, so the oracle is the definition written out.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may use this library.  It
 * shares no code, header, table or helper with the GPU path.
 */
#ifndef FST_ORACLE_H
#define FST_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* result classes */
enum {
    ORC_OK = 0,
    ORC_TRUNCATED = 1,      /* fewer than 8 bytes, or fewer than 8+N header bytes given */
    ORC_HEADER_SIZE = 2,    /* N < 2, N > ORC_MAX_HEADER, or 8+N beyond the file size */
    ORC_JSON = 3,           /* not well-formed JSON / UTF-8 */
    ORC_SCHEMA = 4,         /* well-formed JSON that is not a layout definition */
    ORC_DTYPE = 5,          /* unknown dtype string */
    ORC_SIZE_MISMATCH = 6,  /* end - begin != prod(shape) * sizeof(dtype) */
    ORC_OFFSETS = 7,        /* tensors do not tile the body exactly */
    ORC_DUPLICATE = 8,      /* the same key twice */
    ORC_NOT_FOUND = 9,
    ORC_SHARD = 10,         /* bad dim / rank / world / blocks, or dim not divisible */
    ORC_CAST = 11,          /* conversion outside {F64, F32, F16, BF16} */
    ORC_RANGE = 12,         /* output buffer too small, too many dims */
    ORC_IO = 13,
    ORC_NOMEM = 14
};

#define ORC_MAX_HEADER 100000000ull
#define ORC_MAX_DIMS 8

/* dtype ids of the oracle (its own numbering) */
enum {
    ORC_BOOL = 0, ORC_U8, ORC_I8, ORC_F8_E5M2, ORC_F8_E4M3,
    ORC_I16, ORC_U16, ORC_F16, ORC_BF16,
    ORC_I32, ORC_U32, ORC_F32,
    ORC_I64, ORC_U64, ORC_F64,
    ORC_NDTYPES
};

typedef struct {
    char *name;                      /* decoded key, UTF-8, NUL-terminated */
    size_t name_len;
    int dtype;
    int ndim;
    uint64_t shape[ORC_MAX_DIMS];
    uint64_t begin, end;             /* byte offsets relative to the first body byte */
} orc_tensor;

typedef struct {
    uint64_t n_json;                 /* N: length of the JSON text */
    uint64_t body_off;               /* 8 + N */
    uint64_t body_len;               /* file size - body_off */
    size_t count;
    orc_tensor *tensors;             /* in order of `begin` (ties: zero-byte tensors first) */
    size_t n_meta;                   /* __metadata__ entries (string -> string) */
    char **meta_keys, **meta_vals;
} orc_table;

int orc_dtype_from_name(const char *s, size_t len);     /* -1 if unknown */
const char *orc_dtype_name(int dtype);
uint64_t orc_dtype_size(int dtype);

/* N = little-endian u64 in the first 8 bytes. */
int orc_header_len(const uint8_t *bytes, size_t nbytes, uint64_t *n_out);

/* Parse and validate the first 8+N bytes of a file of `file_size` bytes. */
int orc_parse(const uint8_t *bytes, size_t nbytes, uint64_t file_size, orc_table **out);
void orc_table_free(orc_table *t);
const orc_tensor *orc_find(const orc_table *t, const char *name);

/* Element conversions on bit patterns (round to nearest, ties to even). */
uint32_t orc_bf16_to_f32(uint16_t x);
uint32_t orc_f16_to_f32(uint16_t h);
uint16_t orc_f32_to_bf16(uint32_t x);
uint16_t orc_f32_to_f16(uint32_t x);
uint64_t orc_f32_to_f64(uint32_t x);
uint32_t orc_f64_to_f32(uint64_t x);
uint16_t orc_f64_to_f16(uint64_t x);      /* one rounding from 53 bits, not via binary32 */
uint16_t orc_f64_to_bf16(uint64_t x);
uint64_t orc_f16_to_f64(uint16_t h);      /* exact */
uint64_t orc_bf16_to_f64(uint16_t b);
uint32_t orc_f8e5m2_to_f32(uint8_t b);      /* exact; E5M2 keeps IEEE infinities and NaNs */
uint32_t orc_f8e4m3_to_f32(uint8_t b);      /* exact; E4M3 has no infinity, S.1111.111 is its NaN */
/* n elements of src_dtype at src -> dst_dtype at dst. */
int orc_cast_array(const uint8_t *src, uint64_t n, int src_dtype, int dst_dtype, uint8_t *dst);

/*
 * One stored tensor (its end-begin bytes at `stored`, row-major, little-endian) -> one rank's
 * partition, converted, contiguous.  shard_dim < 0: whole tensor.  blocks > 1 (dim 0 only): dim 0
 * is `blocks` stacked sub-tensors, each partitioned, results concatenated in block order.
 * dst_dtype < 0: keep.  out_shape gets ndim entries.
 */
int orc_materialize(const uint8_t *stored, int src_dtype, int ndim, const uint64_t *shape,
                    int dst_dtype, int shard_dim, int blocks, int rank, int world,
                    uint8_t *out, uint64_t out_cap, uint64_t *out_shape, uint64_t *out_nbytes);

/* Size/shape of the result without computing it. */
int orc_result_info(int src_dtype, int ndim, const uint64_t *shape, int dst_dtype, int shard_dim,
                    int blocks, int rank, int world, uint64_t *out_shape, uint64_t *out_nbytes);

/* Plain reader: open `path`, parse its header, read the named tensor's bytes with fread and
 * materialize it.  *out is malloc'ed (free with orc_free). */
int orc_load(const char *path, const char *name, int dst_dtype, int shard_dim, int blocks,
             int rank, int world, uint8_t **out, uint64_t *out_shape, int *out_ndim,
             int *out_dtype, uint64_t *out_nbytes);
void orc_free(void *p);

/* The same scalar code fanned out over jobs with plain threads (for the CPU baseline). */
typedef struct {
    const uint8_t *stored;
    int src_dtype, ndim;
    uint64_t shape[ORC_MAX_DIMS];
    int dst_dtype, shard_dim, blocks, rank, world;
    uint8_t *out;
    uint64_t out_cap;
    int rc;
} orc_job;
int orc_materialize_jobs(orc_job *jobs, size_t njobs, int nthreads);

#ifdef __cplusplus
}
#endif
#endif
