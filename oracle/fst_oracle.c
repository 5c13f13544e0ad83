/*
 * CPU oracle -- TEST INFRASTRUCTURE ONLY (see fst_oracle.h).  Plain C, scalar loops, no blocking,
 * no vectorization, nothing shared with the GPU path.
 *
 * Parity pins (tests/test_oracle_*.py): hand-built files whose bytes are written out in the test,
 * files written and read back by the independent `safetensors` package, numpy slicing for the
 * partitions, hand-derived partitions and conversions of a hand-typed file, numpy float16 /
 * float64 and torch bfloat16 / float32 conversions for every non-NaN input; binary64 -> 16-bit
 * types against numpy's direct float64 -> float16 conversion, against round-half-even on exact
 * rationals, and on inputs built a hair beside every tie (where rounding twice goes wrong).  NaN payload
 * handling follows the written rule below and is pinned by properties only (sign, quiet bit,
 * leading payload bits): the libraries disagree with each other there -- library parity unpinned
 * for NaN payloads.
 */
#define _FILE_OFFSET_BITS 64
#define _POSIX_C_SOURCE 200809L
#include "fst_oracle.h"

#include <pthread.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/types.h>

/* ------------------------------------------------------------------ dtypes */

static const struct { const char *name; uint64_t size; } k_dtypes[ORC_NDTYPES] = {
    {"BOOL", 1}, {"U8", 1}, {"I8", 1}, {"F8_E5M2", 1}, {"F8_E4M3", 1},
    {"I16", 2}, {"U16", 2}, {"F16", 2}, {"BF16", 2},
    {"I32", 4}, {"U32", 4}, {"F32", 4},
    {"I64", 8}, {"U64", 8}, {"F64", 8},
};

int orc_dtype_from_name(const char *s, size_t len)
{
    for (int i = 0; i < ORC_NDTYPES; i++)
        if (strlen(k_dtypes[i].name) == len && memcmp(k_dtypes[i].name, s, len) == 0) return i;
    return -1;
}

const char *orc_dtype_name(int d) { return (d >= 0 && d < ORC_NDTYPES) ? k_dtypes[d].name : "?"; }
uint64_t orc_dtype_size(int d) { return (d >= 0 && d < ORC_NDTYPES) ? k_dtypes[d].size : 0; }

/* ------------------------------------------------------------------ JSON tree */

typedef enum { J_OBJ, J_ARR, J_STR, J_NUM, J_LIT } jkind;

typedef struct jnode {
    jkind kind;
    char *str;              /* J_STR: decoded bytes */
    size_t len;
    int is_u64;             /* J_NUM: plain non-negative integer that fits 64 bits */
    uint64_t u;
    size_t n;               /* containers */
    struct jnode **item;
    char **key;             /* J_OBJ */
    size_t *keylen;
} jnode;

typedef struct {
    const uint8_t *p, *end;
    int err;                /* ORC_JSON / ORC_SCHEMA / ORC_NOMEM once set */
} jparser;

static void jfree(jnode *v)
{
    if (!v) return;
    for (size_t i = 0; i < v->n; i++) {
        jfree(v->item[i]);
        if (v->key) free(v->key[i]);
    }
    free(v->item);
    free(v->key);
    free(v->keylen);
    free(v->str);
    free(v);
}

static void jskip(jparser *ps)
{
    while (ps->p < ps->end && (*ps->p == ' ' || *ps->p == '\t' || *ps->p == '\n' || *ps->p == '\r'))
        ps->p++;
}

static int hexval(uint8_t c)
{
    if (c >= '0' && c <= '9') return c - '0';
    if (c >= 'a' && c <= 'f') return c - 'a' + 10;
    if (c >= 'A' && c <= 'F') return c - 'A' + 10;
    return -1;
}

static int read_u4(jparser *ps, unsigned *out)
{
    if (ps->end - ps->p < 4) return 0;
    unsigned v = 0;
    for (int i = 0; i < 4; i++) {
        int h = hexval(ps->p[i]);
        if (h < 0) return 0;
        v = v * 16 + (unsigned)h;
    }
    ps->p += 4;
    *out = v;
    return 1;
}

static size_t put_utf8(char *dst, unsigned cp)
{
    if (cp < 0x80) { dst[0] = (char)cp; return 1; }
    if (cp < 0x800) { dst[0] = (char)(0xC0 | (cp >> 6)); dst[1] = (char)(0x80 | (cp & 0x3F)); return 2; }
    if (cp < 0x10000) {
        dst[0] = (char)(0xE0 | (cp >> 12)); dst[1] = (char)(0x80 | ((cp >> 6) & 0x3F));
        dst[2] = (char)(0x80 | (cp & 0x3F));
        return 3;
    }
    dst[0] = (char)(0xF0 | (cp >> 18)); dst[1] = (char)(0x80 | ((cp >> 12) & 0x3F));
    dst[2] = (char)(0x80 | ((cp >> 6) & 0x3F)); dst[3] = (char)(0x80 | (cp & 0x3F));
    return 4;
}

/* Length of the well-formed UTF-8 sequence at p (multi-byte only), 0 if ill-formed. */
static size_t utf8_seq(const uint8_t *p, const uint8_t *end)
{
    uint8_t c = p[0];
    size_t n;
    unsigned cp, min;
    if (c >= 0xC2 && c <= 0xDF) { n = 2; cp = c & 0x1F; min = 0x80; }
    else if (c >= 0xE0 && c <= 0xEF) { n = 3; cp = c & 0x0F; min = 0x800; }
    else if (c >= 0xF0 && c <= 0xF4) { n = 4; cp = c & 0x07; min = 0x10000; }
    else return 0;
    if ((size_t)(end - p) < n) return 0;
    for (size_t i = 1; i < n; i++) {
        if ((p[i] & 0xC0) != 0x80) return 0;
        cp = (cp << 6) | (p[i] & 0x3F);
    }
    if (cp < min || cp > 0x10FFFF || (cp >= 0xD800 && cp <= 0xDFFF)) return 0;
    return n;
}

/* p is just after the opening quote; returns decoded string. */
static char *jstring(jparser *ps, size_t *len_out)
{
    size_t cap = (size_t)(ps->end - ps->p) + 1;   /* decoding never grows the text */
    char *buf = (char *)malloc(cap);
    if (!buf) { ps->err = ORC_NOMEM; return NULL; }
    size_t n = 0;
    for (;;) {
        if (ps->p >= ps->end) goto bad;
        uint8_t c = *ps->p;
        if (c == '"') { ps->p++; break; }
        if (c < 0x20) goto bad;
        if (c == '\\') {
            ps->p++;
            if (ps->p >= ps->end) goto bad;
            uint8_t e = *ps->p++;
            switch (e) {
            case '"': buf[n++] = '"'; break;
            case '\\': buf[n++] = '\\'; break;
            case '/': buf[n++] = '/'; break;
            case 'b': buf[n++] = '\b'; break;
            case 'f': buf[n++] = '\f'; break;
            case 'n': buf[n++] = '\n'; break;
            case 'r': buf[n++] = '\r'; break;
            case 't': buf[n++] = '\t'; break;
            case 'u': {
                unsigned cp;
                if (!read_u4(ps, &cp)) goto bad;
                if (cp >= 0xDC00 && cp <= 0xDFFF) goto bad;          /* lone low surrogate */
                if (cp >= 0xD800 && cp <= 0xDBFF) {                   /* needs a low surrogate */
                    unsigned lo;
                    if (ps->end - ps->p < 2 || ps->p[0] != '\\' || ps->p[1] != 'u') goto bad;
                    ps->p += 2;
                    if (!read_u4(ps, &lo) || lo < 0xDC00 || lo > 0xDFFF) goto bad;
                    cp = 0x10000 + ((cp - 0xD800) << 10) + (lo - 0xDC00);
                }
                n += put_utf8(buf + n, cp);
                break;
            }
            default: goto bad;
            }
        } else if (c < 0x80) {
            buf[n++] = (char)c;
            ps->p++;
        } else {
            size_t k = utf8_seq(ps->p, ps->end);
            if (!k) goto bad;
            memcpy(buf + n, ps->p, k);
            n += k;
            ps->p += k;
        }
    }
    buf[n] = 0;
    *len_out = n;
    return buf;
bad:
    free(buf);
    ps->err = ORC_JSON;
    return NULL;
}

static jnode *jnew(jparser *ps, jkind k)
{
    jnode *v = (jnode *)calloc(1, sizeof(jnode));
    if (!v) ps->err = ORC_NOMEM; else v->kind = k;
    return v;
}

static int jpush(jparser *ps, jnode *c, jnode *item, char *key, size_t keylen)
{
    size_t n = c->n + 1;
    jnode **ni = (jnode **)realloc(c->item, n * sizeof(*ni));
    if (!ni) { ps->err = ORC_NOMEM; return 0; }
    c->item = ni;
    if (c->kind == J_OBJ) {
        char **nk = (char **)realloc(c->key, n * sizeof(*nk));
        if (!nk) { ps->err = ORC_NOMEM; return 0; }
        c->key = nk;
        size_t *nl = (size_t *)realloc(c->keylen, n * sizeof(*nl));
        if (!nl) { ps->err = ORC_NOMEM; return 0; }
        c->keylen = nl;
        c->key[c->n] = key;
        c->keylen[c->n] = keylen;
    }
    c->item[c->n] = item;
    c->n = n;
    return 1;
}

static jnode *jvalue(jparser *ps, int depth);

static jnode *jnumber(jparser *ps)
{
    const uint8_t *s = ps->p;
    int plain = 1, overflow = 0;
    uint64_t u = 0;
    if (ps->p < ps->end && *ps->p == '-') { plain = 0; ps->p++; }
    if (ps->p >= ps->end || *ps->p < '0' || *ps->p > '9') { ps->err = ORC_JSON; return NULL; }
    if (*ps->p == '0') {
        ps->p++;
        if (ps->p < ps->end && *ps->p >= '0' && *ps->p <= '9') { ps->err = ORC_JSON; return NULL; }
    } else {
        while (ps->p < ps->end && *ps->p >= '0' && *ps->p <= '9') {
            unsigned d = (unsigned)(*ps->p - '0');
            if (u > (UINT64_MAX - d) / 10) overflow = 1; else u = u * 10 + d;
            ps->p++;
        }
    }
    if (ps->p < ps->end && *ps->p == '.') {
        plain = 0;
        ps->p++;
        if (ps->p >= ps->end || *ps->p < '0' || *ps->p > '9') { ps->err = ORC_JSON; return NULL; }
        while (ps->p < ps->end && *ps->p >= '0' && *ps->p <= '9') ps->p++;
    }
    if (ps->p < ps->end && (*ps->p == 'e' || *ps->p == 'E')) {
        plain = 0;
        ps->p++;
        if (ps->p < ps->end && (*ps->p == '+' || *ps->p == '-')) ps->p++;
        if (ps->p >= ps->end || *ps->p < '0' || *ps->p > '9') { ps->err = ORC_JSON; return NULL; }
        while (ps->p < ps->end && *ps->p >= '0' && *ps->p <= '9') ps->p++;
    }
    (void)s;
    jnode *v = jnew(ps, J_NUM);
    if (!v) return NULL;
    v->is_u64 = plain && !overflow;
    v->u = u;
    return v;
}

static jnode *jvalue(jparser *ps, int depth)
{
    jskip(ps);
    if (ps->p >= ps->end) { ps->err = ORC_JSON; return NULL; }
    uint8_t c = *ps->p;
    if (c == '{' || c == '[') {
        if (depth >= 3) { ps->err = ORC_SCHEMA; return NULL; }   /* a layout definition is 3 deep */
        jnode *v = jnew(ps, c == '{' ? J_OBJ : J_ARR);
        if (!v) return NULL;
        uint8_t close = c == '{' ? '}' : ']';
        ps->p++;
        jskip(ps);
        if (ps->p < ps->end && *ps->p == close) { ps->p++; return v; }
        for (;;) {
            char *key = NULL;
            size_t keylen = 0;
            if (v->kind == J_OBJ) {
                jskip(ps);
                if (ps->p >= ps->end || *ps->p != '"') { ps->err = ORC_JSON; jfree(v); return NULL; }
                ps->p++;
                key = jstring(ps, &keylen);
                if (!key) { jfree(v); return NULL; }
                jskip(ps);
                if (ps->p >= ps->end || *ps->p != ':') { ps->err = ORC_JSON; free(key); jfree(v); return NULL; }
                ps->p++;
            }
            jnode *item = jvalue(ps, depth + 1);
            if (!item) { free(key); jfree(v); return NULL; }
            if (!jpush(ps, v, item, key, keylen)) { free(key); jfree(item); jfree(v); return NULL; }
            jskip(ps);
            if (ps->p >= ps->end) { ps->err = ORC_JSON; jfree(v); return NULL; }
            if (*ps->p == ',') { ps->p++; continue; }
            if (*ps->p == close) { ps->p++; return v; }
            ps->err = ORC_JSON;
            jfree(v);
            return NULL;
        }
    }
    if (c == '"') {
        ps->p++;
        size_t len;
        char *s = jstring(ps, &len);
        if (!s) return NULL;
        jnode *v = jnew(ps, J_STR);
        if (!v) { free(s); return NULL; }
        v->str = s;
        v->len = len;
        return v;
    }
    if (c == '-' || (c >= '0' && c <= '9')) return jnumber(ps);
    static const char *lits[3] = {"true", "false", "null"};
    for (int i = 0; i < 3; i++) {
        size_t l = strlen(lits[i]);
        if ((size_t)(ps->end - ps->p) >= l && memcmp(ps->p, lits[i], l) == 0) {
            ps->p += l;
            return jnew(ps, J_LIT);
        }
    }
    ps->err = ORC_JSON;
    return NULL;
}

static int key_is(const jnode *o, size_t i, const char *s)
{
    return o->keylen[i] == strlen(s) && memcmp(o->key[i], s, o->keylen[i]) == 0;
}

static int has_dup_keys(const jnode *o)
{
    for (size_t i = 0; i < o->n; i++)
        for (size_t j = i + 1; j < o->n; j++)
            if (o->keylen[i] == o->keylen[j] && memcmp(o->key[i], o->key[j], o->keylen[i]) == 0) return 1;
    return 0;
}

/* ------------------------------------------------------------------ header */

int orc_header_len(const uint8_t *bytes, size_t nbytes, uint64_t *n_out)
{
    if (nbytes < 8) return ORC_TRUNCATED;
    uint64_t n = 0;
    for (int i = 7; i >= 0; i--) n = (n << 8) | bytes[i];      /* little-endian */
    *n_out = n;
    return ORC_OK;
}

void orc_table_free(orc_table *t)
{
    if (!t) return;
    for (size_t i = 0; i < t->count; i++) free(t->tensors[i].name);
    free(t->tensors);
    for (size_t i = 0; i < t->n_meta; i++) { free(t->meta_keys[i]); free(t->meta_vals[i]); }
    free(t->meta_keys);
    free(t->meta_vals);
    free(t);
}

static char *dupn(const char *s, size_t n)
{
    char *r = (char *)malloc(n + 1);
    if (r) { memcpy(r, s, n); r[n] = 0; }
    return r;
}

typedef struct { orc_tensor t; size_t order; } sort_item;

static int by_offset(const void *a, const void *b)
{
    const sort_item *x = (const sort_item *)a, *y = (const sort_item *)b;
    if (x->t.begin != y->t.begin) return x->t.begin < y->t.begin ? -1 : 1;
    if (x->t.end != y->t.end) return x->t.end < y->t.end ? -1 : 1;     /* zero-byte first */
    return x->order < y->order ? -1 : (x->order > y->order);
}

int orc_parse(const uint8_t *bytes, size_t nbytes, uint64_t file_size, orc_table **out)
{
    *out = NULL;
    uint64_t n;
    int rc = orc_header_len(bytes, nbytes, &n);
    if (rc) return rc;
    if (n < 2 || n > ORC_MAX_HEADER) return ORC_HEADER_SIZE;
    if (8 + n > file_size) return ORC_HEADER_SIZE;
    if (nbytes < 8 + n) return ORC_TRUNCATED;

    jparser ps = {bytes + 8, bytes + 8 + n, 0};
    if (*ps.p != '{') return ORC_JSON;                      /* no leading white space */
    jnode *root = jvalue(&ps, 0);
    if (!root) return ps.err;
    jskip(&ps);                                             /* writers pad with spaces */
    if (ps.p != ps.end) { jfree(root); return ORC_JSON; }

    orc_table *t = (orc_table *)calloc(1, sizeof(*t));
    sort_item *items = (sort_item *)calloc(root->n ? root->n : 1, sizeof(*items));
    size_t cnt = 0;
    rc = ORC_OK;
    if (!t || !items) { rc = ORC_NOMEM; goto done; }
    t->n_json = n;
    t->body_off = 8 + n;
    t->body_len = file_size - t->body_off;
    if (has_dup_keys(root)) { rc = ORC_DUPLICATE; goto done; }

    for (size_t i = 0; i < root->n && rc == ORC_OK; i++) {
        const jnode *v = root->item[i];
        if (key_is(root, i, "__metadata__")) {
            if (v->kind != J_OBJ) { rc = ORC_SCHEMA; break; }
            if (has_dup_keys(v)) { rc = ORC_DUPLICATE; break; }
            t->meta_keys = (char **)calloc(v->n ? v->n : 1, sizeof(char *));
            t->meta_vals = (char **)calloc(v->n ? v->n : 1, sizeof(char *));
            if (!t->meta_keys || !t->meta_vals) { rc = ORC_NOMEM; break; }
            for (size_t j = 0; j < v->n; j++) {
                if (v->item[j]->kind != J_STR) { rc = ORC_SCHEMA; break; }
                t->meta_keys[j] = dupn(v->key[j], v->keylen[j]);
                t->meta_vals[j] = dupn(v->item[j]->str, v->item[j]->len);
                t->n_meta = j + 1;
            }
            continue;
        }
        if (v->kind != J_OBJ) { rc = ORC_SCHEMA; break; }
        if (has_dup_keys(v)) { rc = ORC_DUPLICATE; break; }
        const jnode *jd = NULL, *js = NULL, *jo = NULL;
        for (size_t j = 0; j < v->n; j++) {
            if (key_is(v, j, "dtype")) jd = v->item[j];
            else if (key_is(v, j, "shape")) js = v->item[j];
            else if (key_is(v, j, "data_offsets")) jo = v->item[j];
            else { rc = ORC_SCHEMA; break; }                /* unknown field */
        }
        if (rc) break;
        if (!jd || !js || !jo || jd->kind != J_STR || js->kind != J_ARR || jo->kind != J_ARR ||
            jo->n != 2) { rc = ORC_SCHEMA; break; }
        orc_tensor *e = &items[cnt].t;
        for (size_t j = 0; j < js->n; j++)
            if (js->item[j]->kind != J_NUM || !js->item[j]->is_u64) { rc = ORC_SCHEMA; break; }
        for (size_t j = 0; j < 2 && !rc; j++)
            if (jo->item[j]->kind != J_NUM || !jo->item[j]->is_u64) { rc = ORC_SCHEMA; break; }
        if (rc) break;
        e->dtype = orc_dtype_from_name(jd->str, jd->len);
        if (e->dtype < 0) { rc = ORC_DTYPE; break; }
        if (js->n > ORC_MAX_DIMS) { rc = ORC_RANGE; break; }
        e->ndim = (int)js->n;
        uint64_t numel = 1;
        int ovf = 0;
        for (int j = 0; j < e->ndim; j++) {
            e->shape[j] = js->item[j]->u;
            if (e->shape[j] && numel > UINT64_MAX / e->shape[j]) ovf = 1; else numel *= e->shape[j];
        }
        /* a zero dimension makes the tensor empty whatever the other dims are */
        for (int j = 0; j < e->ndim; j++) if (e->shape[j] == 0) { numel = 0; ovf = 0; }
        e->begin = jo->item[0]->u;
        e->end = jo->item[1]->u;
        if (e->begin > e->end) { rc = ORC_OFFSETS; break; }
        uint64_t es = orc_dtype_size(e->dtype);
        if (ovf || numel > UINT64_MAX / es || e->end - e->begin != numel * es) { rc = ORC_SIZE_MISMATCH; break; }
        e->name = dupn(root->key[i], root->keylen[i]);
        e->name_len = root->keylen[i];
        if (!e->name) { rc = ORC_NOMEM; break; }
        items[cnt].order = cnt;
        cnt++;
    }
    if (rc) goto done;

    /* the tensors must tile the body exactly: contiguous, no holes, no overlaps */
    qsort(items, cnt, sizeof(*items), by_offset);
    {
        uint64_t at = 0;
        for (size_t i = 0; i < cnt; i++) {
            if (items[i].t.begin != at) { rc = ORC_OFFSETS; goto done; }
            at = items[i].t.end;
        }
        if (at != t->body_len) { rc = ORC_OFFSETS; goto done; }
    }
    t->tensors = (orc_tensor *)calloc(cnt ? cnt : 1, sizeof(orc_tensor));
    if (!t->tensors) { rc = ORC_NOMEM; goto done; }
    for (size_t i = 0; i < cnt; i++) t->tensors[i] = items[i].t;
    t->count = cnt;
    cnt = 0;    /* names now owned by the table */

done:
    for (size_t i = 0; i < cnt; i++) free(items[i].t.name);
    free(items);
    jfree(root);
    if (rc) { orc_table_free(t); return rc; }
    *out = t;
    return ORC_OK;
}

const orc_tensor *orc_find(const orc_table *t, const char *name)
{
    size_t l = strlen(name);
    for (size_t i = 0; i < t->count; i++)
        if (t->tensors[i].name_len == l && memcmp(t->tensors[i].name, name, l) == 0) return &t->tensors[i];
    return NULL;
}

/* ------------------------------------------------------------------ conversions
 * All on unsigned bit patterns; round to nearest, ties to even; overflow to infinity; gradual
 * underflow; the sign of zero is kept.  NaN: sign kept, leading payload bits kept, quiet bit set.
 */

/* bfloat16 is the upper half of binary32: widening appends 16 zero bits. */
uint32_t orc_bf16_to_f32(uint16_t x)
{
    uint32_t y = (uint32_t)x << 16;
    if ((y & 0x7FFFFFFFu) > 0x7F800000u) y |= 0x00400000u;
    return y;
}

/* binary16 (1-5-10, bias 15) -> binary32 (1-8-23, bias 127): always exact. */
uint32_t orc_f16_to_f32(uint16_t h)
{
    uint32_t s = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 31u;
    uint32_t m = h & 0x3FFu;
    if (e == 0) {
        if (m == 0) return s;                                    /* +-0 */
        /* subnormal: value = m * 2^-24; normalize so that the leading 1 becomes implicit */
        int k = 9;
        while (!((m >> k) & 1u)) k--;
        return s | ((uint32_t)(103 + k) << 23) | ((m << (23 - k)) & 0x7FFFFFu);
    }
    if (e == 31) {
        if (m == 0) return s | 0x7F800000u;                      /* infinity */
        return s | 0x7F800000u | (m << 13) | 0x00400000u;        /* NaN */
    }
    return s | ((e + 112u) << 23) | (m << 13);
}

/* binary32 -> bfloat16: drop 16 mantissa bits with RNE. */
uint16_t orc_f32_to_bf16(uint32_t x)
{
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((x >> 16) | 0x0040u);
    uint32_t lsb = (x >> 16) & 1u;
    return (uint16_t)((x + 0x7FFFu + lsb) >> 16);                /* max finite carries into inf */
}

/* binary32 -> binary16 with RNE. */
uint16_t orc_f32_to_f16(uint32_t x)
{
    uint32_t s = (x >> 16) & 0x8000u;
    uint32_t a = x & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(s | 0x7C00u | 0x0200u | ((a >> 13) & 0x3FFu));
    if (a >= 0x477FF000u) return (uint16_t)(s | 0x7C00u);        /* >= 65520 rounds to infinity */
    if (a <= 0x33000000u) return (uint16_t)s;                    /* <= 2^-25 rounds to zero */
    if (a >= 0x38800000u) {                                      /* result is normal */
        uint32_t r = a - 0x38000000u;                            /* rebias 127 -> 15 */
        return (uint16_t)(s | ((r + 0xFFFu + ((r >> 13) & 1u)) >> 13));
    }
    /* result is subnormal: q = round(value / 2^-24) */
    uint32_t e = a >> 23;                                        /* 102 .. 112 */
    uint32_t m = (a & 0x7FFFFFu) | 0x800000u;
    uint32_t sh = 126u - e;                                      /* 14 .. 24 */
    uint32_t q = m >> sh;
    uint32_t rem = m & ((1u << sh) - 1u);
    uint32_t half = 1u << (sh - 1);
    if (rem > half || (rem == half && (q & 1u))) q++;
    return (uint16_t)(s | q);
}

/* binary32 (1-8-23, bias 127) -> binary64 (1-11-52, bias 1023): always exact. */
uint64_t orc_f32_to_f64(uint32_t x)
{
    uint64_t s = (uint64_t)(x >> 31) << 63;
    uint64_t e = (x >> 23) & 0xFFu;
    uint64_t m = x & 0x7FFFFFu;
    if (e == 0) {
        if (m == 0) return s;                                    /* +-0 */
        /* subnormal: value = m * 2^-149; normalize so that the leading 1 becomes implicit */
        int k = 22;
        while (!((m >> k) & 1u)) k--;
        return s | ((uint64_t)(874 + k) << 52) | ((m << (52 - k)) & 0xFFFFFFFFFFFFFull);
    }
    if (e == 255) {
        if (m == 0) return s | 0x7FF0000000000000ull;            /* infinity */
        return s | 0x7FF0000000000000ull | (m << 29) | 0x0008000000000000ull;   /* NaN */
    }
    return s | ((e + 896u) << 52) | (m << 29);
}

/* binary64 -> binary32 with RNE. */
uint32_t orc_f64_to_f32(uint64_t x)
{
    uint32_t s = (uint32_t)(x >> 32) & 0x80000000u;
    uint64_t a = x & 0x7FFFFFFFFFFFFFFFull;
    uint64_t e = a >> 52;
    uint64_t m = a & 0xFFFFFFFFFFFFFull;
    if (a > 0x7FF0000000000000ull) return s | 0x7F800000u | 0x00400000u | (uint32_t)((a >> 29) & 0x3FFFFFu);
    if (e > 1023u + 127u) return s | 0x7F800000u;                /* 2^128 and above, infinity */
    if (e >= 897u) {                                             /* result is normal (or rounds up to infinity) */
        uint32_t r = (uint32_t)((e - 896u) << 23) | (uint32_t)(m >> 29);
        uint64_t rem = m & 0x1FFFFFFFull, half = 0x10000000ull;
        if (rem > half || (rem == half && (r & 1u))) r++;        /* a carry moves the exponent up, to infinity at most */
        return s | r;
    }
    if (e < 872u) return s;                                      /* below 2^-151: rounds to zero */
    /* result is subnormal: q = round(value / 2^-149), value = M * 2^(e-1075) */
    uint64_t M = m | 0x10000000000000ull;
    uint64_t sh = 926u - e;                                      /* 30 .. 54 */
    uint64_t q = M >> sh;
    uint64_t rem = M & (((uint64_t)1 << sh) - 1u);
    uint64_t half = (uint64_t)1 << (sh - 1);
    if (rem > half || (rem == half && (q & 1u))) q++;
    return s | (uint32_t)q;
}

/* binary64 -> a 16-bit format with `mb` stored mantissa bits and exponent bias `bias` (binary16:
 * 10 and 15; bfloat16: 7 and 127), rounded ONCE from the 53-bit significand.  Going through
 * binary32 would round twice and differ on values that the first rounding moves onto a tie. */
static uint16_t f64_to_16bit(uint64_t x, int mb, int bias)
{
    uint16_t s = (uint16_t)((x >> 48) & 0x8000u);
    uint64_t a = x & 0x7FFFFFFFFFFFFFFFull;
    int64_t e = (int64_t)(a >> 52);
    uint64_t m = a & 0xFFFFFFFFFFFFFull;
    uint16_t inf = (uint16_t)(0x7FFFu & ~((1u << mb) - 1u));     /* exponent field all ones */
    uint16_t quiet = (uint16_t)(1u << (mb - 1));
    if (a > 0x7FF0000000000000ull) return (uint16_t)(s | inf | quiet | ((m >> (52 - mb)) & (quiet - 1u)));
    int64_t E = e - 1023 + bias;                                 /* exponent field of a normal result */
    if (E >= (inf >> mb)) return (uint16_t)(s | inf);            /* too large (and infinity) */
    if (E >= 1) {                                                /* normal, or rounds up to infinity */
        uint32_t r = (uint32_t)(E << mb) | (uint32_t)(m >> (52 - mb));
        uint64_t rem = m & (((uint64_t)1 << (52 - mb)) - 1u), half = (uint64_t)1 << (51 - mb);
        if (rem > half || (rem == half && (r & 1u))) r++;        /* a carry moves the exponent up */
        return (uint16_t)(s | r);
    }
    /* subnormal result: q = round(value / 2^(1-bias-mb)), value = M * 2^(e-1075) */
    int64_t sh = 1076 - e - bias - mb;                           /* at least 53 - mb */
    if (e == 0 || sh > 54) return s;                             /* below half the smallest subnormal */
    uint64_t M = m | 0x10000000000000ull;
    uint64_t q = M >> sh;
    uint64_t rem = M & (((uint64_t)1 << sh) - 1u);
    uint64_t half = (uint64_t)1 << (sh - 1);
    if (rem > half || (rem == half && (q & 1u))) q++;
    return (uint16_t)(s | q);
}

uint16_t orc_f64_to_f16(uint64_t x) { return f64_to_16bit(x, 10, 15); }
uint16_t orc_f64_to_bf16(uint64_t x) { return f64_to_16bit(x, 7, 127); }
/* 16-bit -> binary64: two exact widenings in a row. */
uint64_t orc_f16_to_f64(uint16_t h) { return orc_f32_to_f64(orc_f16_to_f32(h)); }
uint64_t orc_bf16_to_f64(uint16_t b) { return orc_f32_to_f64(orc_bf16_to_f32(b)); }

/* An 8-bit float with `mb` stored mantissa bits (7 - mb exponent bits) and exponent bias `bias` ->
 * binary32: always exact.  Two layouts exist (Section VI names the 8-bit types; their definition is
 * the one of the FP8 formats the paper cites there):
 *   E5M2 (mb 2, bias 15) follows IEEE 754: exponent field all ones = infinity (mantissa 0) or NaN;
 *   E4M3 (mb 3, bias 7) has no infinity: exponent field all ones holds ordinary values (up to
 *   1.75 * 2^8 = 448), except that mantissa all ones there is the NaN.
 * NaN by the rule above: sign kept, the mantissa field moved to the leading mantissa bits, quiet bit set. */
static uint32_t f8_to_f32(uint8_t b, int mb, int bias, int ieee_specials)
{
    uint32_t s = ((uint32_t)b & 0x80u) << 24;
    uint32_t emax = (1u << (7 - mb)) - 1u, mmax = (1u << mb) - 1u;
    uint32_t e = ((uint32_t)b >> mb) & emax;
    uint32_t m = (uint32_t)b & mmax;
    if (e == emax && (ieee_specials ? m != 0 : m == mmax))
        return s | 0x7F800000u | (m << (23 - mb)) | 0x00400000u;  /* NaN */
    if (e == emax && ieee_specials) return s | 0x7F800000u;       /* infinity */
    if (e == 0) {
        if (m == 0) return s;                                     /* +-0 */
        /* subnormal: value = m * 2^(1 - bias - mb); normalize so that the leading 1 becomes implicit */
        int k = mb - 1;
        while (!((m >> k) & 1u)) k--;
        return s | ((uint32_t)(127 + 1 - bias - mb + k) << 23) | ((m << (23 - k)) & 0x7FFFFFu);
    }
    return s | ((e + 127u - (uint32_t)bias) << 23) | (m << (23 - mb));
}

uint32_t orc_f8e5m2_to_f32(uint8_t b) { return f8_to_f32(b, 2, 15, 1); }
uint32_t orc_f8e4m3_to_f32(uint8_t b) { return f8_to_f32(b, 3, 7, 0); }

static int is_float_dtype(int d) { return d == ORC_F64 || d == ORC_F32 || d == ORC_F16 || d == ORC_BF16; }
static int is_f8_dtype(int d) { return d == ORC_F8_E5M2 || d == ORC_F8_E4M3; }

/* Conversions that exist: among F64, F32, F16 and BF16, and the widenings of the two 8-bit floats to
 * F16, BF16 and F32 (every 8-bit value is exact in each of them). */
static int can_convert(int sd, int dd)
{
    if (sd == dd) return 1;
    if (is_f8_dtype(sd)) return dd == ORC_F16 || dd == ORC_BF16 || dd == ORC_F32;
    return is_float_dtype(sd) && is_float_dtype(dd);
}

static uint64_t load_le(const uint8_t *p, uint64_t es)
{
    uint64_t v = 0;
    for (uint64_t i = es; i-- > 0;) v = (v << 8) | p[i];
    return v;
}

static void store_le(uint8_t *p, uint64_t es, uint64_t v)
{
    for (uint64_t i = 0; i < es; i++) { p[i] = (uint8_t)(v & 0xFF); v >>= 8; }
}

/* One element.  Narrow-to-narrow goes through binary32, which holds every 16-bit value exactly,
 * so the result is rounded once; binary64 to a 16-bit type is rounded once from 53 bits. */
static uint64_t convert(uint64_t v, int sd, int dd)
{
    if (sd == dd) return v;
    if (sd == ORC_F64) return dd == ORC_F32 ? orc_f64_to_f32(v) : dd == ORC_F16 ? orc_f64_to_f16(v) : orc_f64_to_bf16(v);
    if (dd == ORC_F64)
        return sd == ORC_F32 ? orc_f32_to_f64((uint32_t)v) : sd == ORC_F16 ? orc_f16_to_f64((uint16_t)v) : orc_bf16_to_f64((uint16_t)v);
    uint32_t f;
    if (sd == ORC_F32) f = (uint32_t)v;
    else if (sd == ORC_F8_E5M2) f = orc_f8e5m2_to_f32((uint8_t)v);
    else if (sd == ORC_F8_E4M3) f = orc_f8e4m3_to_f32((uint8_t)v);
    else if (sd == ORC_F16) f = orc_f16_to_f32((uint16_t)v);
    else f = orc_bf16_to_f32((uint16_t)v);
    if (dd == ORC_F32) return f;
    if (dd == ORC_F16) return orc_f32_to_f16(f);
    return orc_f32_to_bf16(f);
}

int orc_cast_array(const uint8_t *src, uint64_t n, int sd, int dd, uint8_t *dst)
{
    if (sd < 0 || sd >= ORC_NDTYPES || dd < 0 || dd >= ORC_NDTYPES) return ORC_DTYPE;
    if (!can_convert(sd, dd)) return ORC_CAST;
    uint64_t ss = orc_dtype_size(sd), ds = orc_dtype_size(dd);
    for (uint64_t i = 0; i < n; i++) store_le(dst + i * ds, ds, convert(load_le(src + i * ss, ss), sd, dd));
    return ORC_OK;
}

/* ------------------------------------------------------------------ partition + convert */

int orc_result_info(int sd, int ndim, const uint64_t *shape, int dd, int shard_dim, int blocks,
                    int rank, int world, uint64_t *out_shape, uint64_t *out_nbytes)
{
    if (sd < 0 || sd >= ORC_NDTYPES) return ORC_DTYPE;
    if (dd < 0) dd = sd;
    if (dd >= ORC_NDTYPES) return ORC_DTYPE;
    if (ndim < 0 || ndim > ORC_MAX_DIMS) return ORC_RANGE;
    if (!can_convert(sd, dd)) return ORC_CAST;
    if (world < 1 || rank < 0 || rank >= world || blocks < 1) return ORC_SHARD;
    if (shard_dim < 0 && blocks != 1) return ORC_SHARD;
    if (shard_dim >= ndim) return ORC_SHARD;                     /* e.g. dim 1 of a vector */
    if (blocks > 1 && shard_dim != 0) return ORC_SHARD;
    uint64_t numel = 1;
    for (int d = 0; d < ndim; d++) {
        uint64_t s = shape[d];
        if (d == shard_dim) {
            uint64_t parts = (uint64_t)blocks * (uint64_t)world;
            if (s % parts) return ORC_SHARD;                     /* partitions must be same-shaped */
            s = s / (uint64_t)world;
        }
        if (out_shape) out_shape[d] = s;
        numel *= s;
    }
    if (out_nbytes) *out_nbytes = numel * orc_dtype_size(dd);
    return ORC_OK;
}

int orc_materialize(const uint8_t *stored, int sd, int ndim, const uint64_t *shape, int dd,
                    int shard_dim, int blocks, int rank, int world, uint8_t *out, uint64_t out_cap,
                    uint64_t *out_shape, uint64_t *out_nbytes)
{
    uint64_t oshape[ORC_MAX_DIMS + 1], onb;
    int rc = orc_result_info(sd, ndim, shape, dd, shard_dim, blocks, rank, world, oshape, &onb);
    if (rc) return rc;
    if (dd < 0) dd = sd;
    if (out_shape) for (int d = 0; d < ndim; d++) out_shape[d] = oshape[d];
    if (out_nbytes) *out_nbytes = onb;
    if (onb > out_cap) return ORC_RANGE;
    if (onb == 0) return ORC_OK;

    uint64_t ss = orc_dtype_size(sd), ds = orc_dtype_size(dd);
    /* row-major element strides of the stored tensor */
    uint64_t stride[ORC_MAX_DIMS + 1];
    uint64_t acc = 1;
    for (int d = ndim - 1; d >= 0; d--) { stride[d] = acc; acc *= shape[d]; }
    /* per = rows of one block that one rank keeps; blk_len = rows of one block as stored */
    uint64_t per = 0, blk_len = 0;
    if (shard_dim >= 0) {
        blk_len = shape[shard_dim] / (uint64_t)blocks;
        per = blk_len / (uint64_t)world;
    }

    uint64_t idx[ORC_MAX_DIMS + 1];
    for (int d = 0; d < ndim; d++) idx[d] = 0;
    uint64_t total = onb / ds;
    for (uint64_t k = 0; k < total; k++) {
        /* source element of output multi-index idx */
        uint64_t lin = 0;
        for (int d = 0; d < ndim; d++) {
            uint64_t i = idx[d];
            if (d == shard_dim) i = (i / per) * blk_len + (uint64_t)rank * per + (i % per);
            lin += i * stride[d];
        }
        store_le(out + k * ds, ds, convert(load_le(stored + lin * ss, ss), sd, dd));
        /* next multi-index in row-major order */
        for (int d = ndim - 1; d >= 0; d--) {
            if (++idx[d] < oshape[d]) break;
            idx[d] = 0;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ plain file reader */

void orc_free(void *p) { free(p); }

int orc_load(const char *path, const char *name, int dd, int shard_dim, int blocks, int rank,
             int world, uint8_t **out, uint64_t *out_shape, int *out_ndim, int *out_dtype,
             uint64_t *out_nbytes)
{
    *out = NULL;
    FILE *f = fopen(path, "rb");
    if (!f) return ORC_IO;
    int rc = ORC_OK;
    uint8_t first[8];
    uint8_t *head = NULL, *stored = NULL, *res = NULL;
    orc_table *tab = NULL;
    uint64_t n = 0;
    if (fseeko(f, 0, SEEK_END)) { rc = ORC_IO; goto done; }
    uint64_t fsize = (uint64_t)ftello(f);
    if (fseeko(f, 0, SEEK_SET)) { rc = ORC_IO; goto done; }
    size_t got = fread(first, 1, 8, f);
    if ((rc = orc_header_len(first, got, &n))) goto done;
    if (n < 2 || n > ORC_MAX_HEADER || 8 + n > fsize) { rc = ORC_HEADER_SIZE; goto done; }
    head = (uint8_t *)malloc(8 + n);
    if (!head) { rc = ORC_NOMEM; goto done; }
    memcpy(head, first, 8);
    if (fread(head + 8, 1, n, f) != n) { rc = ORC_TRUNCATED; goto done; }
    if ((rc = orc_parse(head, 8 + n, fsize, &tab))) goto done;
    const orc_tensor *t = orc_find(tab, name);
    if (!t) { rc = ORC_NOT_FOUND; goto done; }
    uint64_t oshape[ORC_MAX_DIMS], onb;
    if ((rc = orc_result_info(t->dtype, t->ndim, t->shape, dd, shard_dim, blocks, rank, world, oshape, &onb))) goto done;
    uint64_t nb = t->end - t->begin;
    stored = (uint8_t *)malloc(nb ? nb : 1);
    res = (uint8_t *)malloc(onb ? onb : 1);
    if (!stored || !res) { rc = ORC_NOMEM; goto done; }
    if (fseeko(f, (off_t)(tab->body_off + t->begin), SEEK_SET)) { rc = ORC_IO; goto done; }
    if (fread(stored, 1, nb, f) != nb) { rc = ORC_IO; goto done; }
    rc = orc_materialize(stored, t->dtype, t->ndim, t->shape, dd, shard_dim, blocks, rank, world,
                         res, onb, out_shape, out_nbytes);
    if (rc) goto done;
    if (out_ndim) *out_ndim = t->ndim;
    if (out_dtype) *out_dtype = dd < 0 ? t->dtype : dd;
    *out = res;
    res = NULL;
done:
    free(res);
    free(stored);
    free(head);
    orc_table_free(tab);
    fclose(f);
    return rc;
}

/* ------------------------------------------------------------------ thread fan-out */

typedef struct { orc_job *jobs; size_t njobs; size_t next; pthread_mutex_t mu; } job_queue;

static void *job_worker(void *arg)
{
    job_queue *q = (job_queue *)arg;
    for (;;) {
        pthread_mutex_lock(&q->mu);
        size_t i = q->next++;
        pthread_mutex_unlock(&q->mu);
        if (i >= q->njobs) return NULL;
        orc_job *j = &q->jobs[i];
        j->rc = orc_materialize(j->stored, j->src_dtype, j->ndim, j->shape, j->dst_dtype, j->shard_dim,
                                j->blocks, j->rank, j->world, j->out, j->out_cap, NULL, NULL);
    }
}

int orc_materialize_jobs(orc_job *jobs, size_t njobs, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    job_queue q = {jobs, njobs, 0, PTHREAD_MUTEX_INITIALIZER};
    pthread_t th[256];
    int started = 0;
    for (int i = 0; i < nthreads; i++)
        if (pthread_create(&th[started], NULL, job_worker, &q) == 0) started++;
    if (!started) job_worker(&q);
    for (int i = 0; i < started; i++) pthread_join(th[i], NULL);
    for (size_t i = 0; i < njobs; i++) if (jobs[i].rc) return jobs[i].rc;
    return ORC_OK;
}
