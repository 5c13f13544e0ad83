/*
 * Procedural file source for the large synthetic checkpoints (seeded input generators, part 2).
 *
 * A checkpoint of 13 GB .. 352 GB is never stored: the bytes of file f at offset o are a pure
 * function of (model, f, o).  The header bytes are kept verbatim; the body of tensor k is a
 * window into a small value pool, body byte j of the tensor = pool[(start_k + j) mod pool_len],
 * or a repeated constant pattern (norm weights = 1.0).  Pool lengths are 2 * prime so that the
 * period never lines up with a row or a tile of any tensor.
 *
 * This file holds no parsing, slicing or casting: it only produces input bytes, for the CPU
 * oracle's tests and for the GPU path alike.  syn_read has the signature of a stager read
 * callback, so the staging ring can be fed by generation instead of pread.
 */
#define _GNU_SOURCE
#include <errno.h>
#include <fcntl.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

enum { SYN_POOL = 0, SYN_PATTERN = 1 };

typedef struct {
    uint64_t begin, end;     /* absolute file offsets of the tensor's bytes */
    int32_t kind;            /* SYN_POOL or SYN_PATTERN */
    int32_t pool;            /* which pool (SYN_POOL) */
    uint64_t pool_start;     /* byte offset into that pool of the tensor's byte 0 */
    uint8_t pat[8];          /* SYN_PATTERN: repeated pattern of patlen bytes */
    int32_t patlen;
} syn_tensor;

typedef struct {
    uint8_t *header;         /* first 8+N bytes of the file */
    uint64_t header_len;
    uint64_t size;
    int64_t n;
    syn_tensor *t;           /* sorted by begin, tiling [header_len, size) */
} syn_file;

#define SYN_MAX_POOLS 8
typedef struct {
    int32_t nfiles;
    syn_file *f;
    uint8_t *pool[SYN_MAX_POOLS];
    uint64_t pool_len[SYN_MAX_POOLS];
} syn_model;

syn_model *syn_create(int32_t nfiles)
{
    syn_model *m = (syn_model *)calloc(1, sizeof(*m));
    if (!m) return NULL;
    m->nfiles = nfiles;
    m->f = (syn_file *)calloc((size_t)nfiles, sizeof(syn_file));
    return m;
}

int syn_set_pool(syn_model *m, int32_t id, const uint8_t *bytes, uint64_t len)
{
    if (id < 0 || id >= SYN_MAX_POOLS || len == 0) return -1;
    free(m->pool[id]);
    m->pool[id] = (uint8_t *)malloc(len);
    if (!m->pool[id]) return -1;
    memcpy(m->pool[id], bytes, len);
    m->pool_len[id] = len;
    return 0;
}

int syn_set_file(syn_model *m, int32_t fi, const uint8_t *header, uint64_t header_len,
                 int64_t n, const uint64_t *begin, const uint64_t *end, const int32_t *kind,
                 const int32_t *pool, const uint64_t *pool_start, const uint8_t *pat8,
                 const int32_t *patlen)
{
    if (fi < 0 || fi >= m->nfiles) return -1;
    syn_file *f = &m->f[fi];
    f->header = (uint8_t *)malloc(header_len);
    memcpy(f->header, header, header_len);
    f->header_len = header_len;
    f->n = n;
    f->t = (syn_tensor *)calloc((size_t)(n ? n : 1), sizeof(syn_tensor));
    uint64_t at = header_len;
    for (int64_t i = 0; i < n; i++) {
        if (begin[i] != at || end[i] < begin[i]) return -2;   /* must tile the body */
        f->t[i].begin = begin[i];
        f->t[i].end = end[i];
        f->t[i].kind = kind[i];
        f->t[i].pool = pool[i];
        f->t[i].pool_start = pool_start[i];
        memcpy(f->t[i].pat, pat8 + 8 * i, 8);
        f->t[i].patlen = patlen[i];
        at = end[i];
    }
    f->size = at;
    return 0;
}

uint64_t syn_file_size(const syn_model *m, int32_t fi) { return m->f[fi].size; }

/* Fill dst[0..len) with bytes [off, off+len) of file fi.  Returns 0, or -1 if out of range. */
int syn_read(void *ctx, int32_t fi, uint64_t off, void *dstv, uint64_t len)
{
    const syn_model *m = (const syn_model *)ctx;
    if (fi < 0 || fi >= m->nfiles) return -1;
    const syn_file *f = &m->f[fi];
    if (off > f->size || len > f->size - off) return -1;
    uint8_t *dst = (uint8_t *)dstv;
    uint64_t pos = off, stop = off + len;
    if (pos < f->header_len) {
        uint64_t n = f->header_len - pos;
        if (n > stop - pos) n = stop - pos;
        memcpy(dst, f->header + pos, n);
        dst += n;
        pos += n;
    }
    if (pos >= stop) return 0;
    /* first tensor whose end is beyond pos */
    int64_t lo = 0, hi = f->n;
    while (lo < hi) {
        int64_t mid = (lo + hi) / 2;
        if (f->t[mid].end <= pos) lo = mid + 1; else hi = mid;
    }
    for (int64_t k = lo; k < f->n && pos < stop; k++) {
        const syn_tensor *t = &f->t[k];
        if (t->end <= pos) continue;
        uint64_t n = (t->end < stop ? t->end : stop) - pos;
        uint64_t j = pos - t->begin;           /* byte index inside the tensor */
        if (t->kind == SYN_POOL) {
            const uint8_t *pool = m->pool[t->pool];
            uint64_t plen = m->pool_len[t->pool];
            uint64_t p = (t->pool_start + j) % plen;
            uint64_t left = n;
            while (left) {
                uint64_t run = plen - p;
                if (run > left) run = left;
                memcpy(dst, pool + p, run);
                dst += run;
                left -= run;
                p = 0;
            }
        } else {
            uint64_t pl = (uint64_t)t->patlen;
            for (uint64_t i = 0; i < n; i++) dst[i] = t->pat[(j + i) % pl];
            dst += n;
        }
        pos += n;
    }
    return pos == stop ? 0 : -1;
}

typedef struct {
    const syn_model *m;
    int32_t fi;
    int fd;
    uint64_t lo, hi;
    int rc;
} syn_wjob;

static void *syn_write_worker(void *arg)
{
    syn_wjob *j = (syn_wjob *)arg;
    const uint64_t CH = 32u << 20;
    uint8_t *buf = (uint8_t *)malloc(CH);
    if (!buf) { j->rc = -1; return NULL; }
    for (uint64_t o = j->lo; o < j->hi; o += CH) {
        uint64_t n = j->hi - o < CH ? j->hi - o : CH;
        if (syn_read((void *)j->m, j->fi, o, buf, n)) { j->rc = -1; break; }
        uint64_t done = 0;
        while (done < n) {
            ssize_t w = pwrite(j->fd, buf + done, n - done, (off_t)(o + done));
            if (w < 0) { if (errno == EINTR) continue; j->rc = -1; break; }
            done += (uint64_t)w;
        }
        if (j->rc) break;
    }
    free(buf);
    return NULL;
}

/* Write file fi to `path` with `nthreads` writers.  Returns 0 or -1. */
int syn_write_file(const syn_model *m, int32_t fi, const char *path, int32_t nthreads)
{
    if (fi < 0 || fi >= m->nfiles) return -1;
    int fd = open(path, O_CREAT | O_TRUNC | O_WRONLY, 0644);
    if (fd < 0) return -1;
    uint64_t size = m->f[fi].size;
    if (ftruncate(fd, (off_t)size)) { close(fd); return -1; }
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 64) nthreads = 64;
    pthread_t th[64];
    syn_wjob job[64];
    uint64_t per = (size / (uint64_t)nthreads + 4095) & ~(uint64_t)4095;
    if (per == 0) per = 4096;
    int used = 0;
    for (int i = 0; i < nthreads; i++) {
        uint64_t lo = per * (uint64_t)i;
        if (lo >= size) break;
        uint64_t hi = lo + per < size ? lo + per : size;
        job[used] = (syn_wjob){m, fi, fd, lo, hi, 0};
        pthread_create(&th[used], NULL, syn_write_worker, &job[used]);
        used++;
    }
    int rc = 0;
    for (int i = 0; i < used; i++) {
        pthread_join(th[i], NULL);
        if (job[i].rc) rc = -1;
    }
    if (close(fd)) rc = -1;
    return rc;
}

void syn_free(syn_model *m)
{
    if (!m) return;
    for (int i = 0; i < m->nfiles; i++) {
        free(m->f[i].header);
        free(m->f[i].t);
    }
    for (int i = 0; i < SYN_MAX_POOLS; i++) free(m->pool[i]);
    free(m->f);
    free(m);
}
