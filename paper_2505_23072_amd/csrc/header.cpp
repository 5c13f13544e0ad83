// Host-side reader of the safetensors header (paper Section II-A, Fig. 1): 8 bytes of header
// size, then a JSON layout definition {key: {dtype, shape, data_offsets}}.  A single-pass parser
// specialised to that schema fills the tensor table directly; nothing here touches the GPU.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <unordered_set>

#include "fst_internal.h"

namespace fst {

static thread_local char g_error[512] = "";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return status;
}

namespace {

struct DtypeRow { const char *name; uint32_t size; };
// indexed by fst_dtype
const DtypeRow kDtypes[FST_DTYPE_COUNT] = {
    {"F64", 8}, {"F32", 4}, {"F16", 2}, {"BF16", 2}, {"F8_E5M2", 1}, {"F8_E4M3", 1},
    {"I64", 8}, {"I32", 4}, {"I16", 2}, {"I8", 1},
    {"U64", 8}, {"U32", 4}, {"U16", 2}, {"U8", 1},
    {"BOOL", 1},
};

// Cursor over the header text.  Every method returns FST_OK or the status to report.
class Cursor {
public:
    Cursor(const uint8_t *b, const uint8_t *e) : p_(b), e_(e) {}

    void ws()
    {
        while (p_ < e_ && (*p_ == 0x20 || *p_ == 0x09 || *p_ == 0x0A || *p_ == 0x0D)) ++p_;
    }
    bool at_end() const { return p_ == e_; }
    int peek() const { return p_ < e_ ? *p_ : -1; }
    bool eat(uint8_t c)
    {
        if (p_ < e_ && *p_ == c) { ++p_; return true; }
        return false;
    }
    size_t pos(const uint8_t *base) const { return size_t(p_ - base); }

    // A JSON string, cursor on the opening quote; appends the decoded UTF-8 to out.
    int string(std::string &out)
    {
        if (!eat('"')) return FST_E_JSON;
        while (true) {
            if (p_ >= e_) return FST_E_JSON;
            uint8_t c = *p_++;
            if (c == '"') return FST_OK;
            if (c < 0x20) return FST_E_JSON;
            if (c == '\\') {
                if (p_ >= e_) return FST_E_JSON;
                uint8_t esc = *p_++;
                switch (esc) {
                case '"': case '\\': case '/': out.push_back(char(esc)); break;
                case 'b': out.push_back('\b'); break;
                case 'f': out.push_back('\f'); break;
                case 'n': out.push_back('\n'); break;
                case 'r': out.push_back('\r'); break;
                case 't': out.push_back('\t'); break;
                case 'u': {
                    uint32_t cp;
                    if (!hex4(cp)) return FST_E_JSON;
                    if ((cp & 0xFC00) == 0xDC00) return FST_E_JSON;
                    if ((cp & 0xFC00) == 0xD800) {
                        uint32_t lo;
                        if (!(eat('\\') && eat('u') && hex4(lo)) || (lo & 0xFC00) != 0xDC00) return FST_E_JSON;
                        cp = 0x10000 + ((cp & 0x3FF) << 10) + (lo & 0x3FF);
                    }
                    encode(cp, out);
                    break;
                }
                default: return FST_E_JSON;
                }
            } else if (c < 0x80) {
                out.push_back(char(c));
            } else {
                // multi-byte UTF-8: lead byte fixes the length and the smallest legal code point
                int extra;
                uint32_t cp, least;
                if (c >= 0xC2 && c <= 0xDF) { extra = 1; cp = c & 0x1F; least = 0x80; }
                else if ((c & 0xF0) == 0xE0) { extra = 2; cp = c & 0x0F; least = 0x800; }
                else if (c >= 0xF0 && c <= 0xF4) { extra = 3; cp = c & 0x07; least = 0x10000; }
                else return FST_E_JSON;
                if (e_ - p_ < extra) return FST_E_JSON;
                out.push_back(char(c));
                for (int i = 0; i < extra; ++i) {
                    uint8_t t = *p_++;
                    if ((t & 0xC0) != 0x80) return FST_E_JSON;
                    cp = (cp << 6) | (t & 0x3F);
                    out.push_back(char(t));
                }
                if (cp < least || cp > 0x10FFFF || (cp >= 0xD800 && cp < 0xE000)) return FST_E_JSON;
            }
        }
    }

    // A JSON number.  FST_E_JSON if malformed; FST_E_SCHEMA if well-formed but not a plain
    // non-negative integer that fits 64 bits.
    int u64(uint64_t &out)
    {
        bool plain = true;
        if (eat('-')) plain = false;
        if (p_ >= e_ || *p_ < '0' || *p_ > '9') return FST_E_JSON;
        uint64_t v = 0;
        if (*p_ == '0') {
            ++p_;
            if (p_ < e_ && *p_ >= '0' && *p_ <= '9') return FST_E_JSON;   // leading zero
        } else {
            while (p_ < e_ && *p_ >= '0' && *p_ <= '9') {
                uint64_t d = uint64_t(*p_++ - '0');
                if (v > (UINT64_MAX - d) / 10) plain = false; else v = v * 10 + d;
            }
        }
        if (eat('.')) {
            plain = false;
            if (!digits()) return FST_E_JSON;
        }
        if (p_ < e_ && (*p_ == 'e' || *p_ == 'E')) {
            plain = false;
            ++p_;
            if (p_ < e_ && (*p_ == '+' || *p_ == '-')) ++p_;
            if (!digits()) return FST_E_JSON;
        }
        if (!plain) return FST_E_SCHEMA;
        out = v;
        return FST_OK;
    }

private:
    bool digits()
    {
        const uint8_t *s = p_;
        while (p_ < e_ && *p_ >= '0' && *p_ <= '9') ++p_;
        return p_ != s;
    }
    bool hex4(uint32_t &v)
    {
        if (e_ - p_ < 4) return false;
        v = 0;
        for (int i = 0; i < 4; ++i) {
            uint8_t c = *p_++;
            uint32_t d;
            if (c >= '0' && c <= '9') d = c - '0';
            else if (c >= 'a' && c <= 'f') d = c - 'a' + 10;
            else if (c >= 'A' && c <= 'F') d = c - 'A' + 10;
            else return false;
            v = (v << 4) | d;
        }
        return true;
    }
    static void encode(uint32_t cp, std::string &out)
    {
        if (cp < 0x80) {
            out.push_back(char(cp));
        } else if (cp < 0x800) {
            out.push_back(char(0xC0 | (cp >> 6)));
            out.push_back(char(0x80 | (cp & 0x3F)));
        } else if (cp < 0x10000) {
            out.push_back(char(0xE0 | (cp >> 12)));
            out.push_back(char(0x80 | ((cp >> 6) & 0x3F)));
            out.push_back(char(0x80 | (cp & 0x3F)));
        } else {
            out.push_back(char(0xF0 | (cp >> 18)));
            out.push_back(char(0x80 | ((cp >> 12) & 0x3F)));
            out.push_back(char(0x80 | ((cp >> 6) & 0x3F)));
            out.push_back(char(0x80 | (cp & 0x3F)));
        }
    }

    const uint8_t *p_, *e_;
};

// What kind of value starts here, for error classification: a container or scalar of the wrong
// type is a schema error, anything that cannot start a JSON value is a syntax error.
int wrong_type(const Cursor &c)
{
    int ch = c.peek();
    if (ch == '{' || ch == '[' || ch == '"' || ch == '-' || (ch >= '0' && ch <= '9') || ch == 't' ||
        ch == 'f' || ch == 'n')
        return FST_E_SCHEMA;
    return FST_E_JSON;
}

// "[" u64 ("," u64)* "]" or "[]"; at most `cap` entries are kept, n counts all of them.
int u64_array(Cursor &c, uint64_t *vals, size_t cap, size_t &n)
{
    n = 0;
    if (!c.eat('[')) return wrong_type(c);
    c.ws();
    if (c.eat(']')) return FST_OK;
    while (true) {
        c.ws();
        int ch = c.peek();
        if (ch == '{' || ch == '[' ) return FST_E_SCHEMA;          // a fourth level of nesting
        if (!(ch == '-' || (ch >= '0' && ch <= '9'))) return wrong_type(c);
        uint64_t v = 0;
        if (int rc = c.u64(v)) return rc;
        if (n < cap) vals[n] = v;
        ++n;
        c.ws();
        if (c.eat(',')) continue;
        if (c.eat(']')) return FST_OK;
        return FST_E_JSON;
    }
}

int metadata_object(Cursor &c, fst_header &h)
{
    if (!c.eat('{')) return wrong_type(c);
    std::unordered_set<std::string> seen;
    c.ws();
    if (c.eat('}')) return FST_OK;
    while (true) {
        c.ws();
        std::string k, v;
        if (int rc = c.string(k)) return rc;
        c.ws();
        if (!c.eat(':')) return FST_E_JSON;
        c.ws();
        if (c.peek() != '"') return wrong_type(c);
        if (int rc = c.string(v)) return rc;
        if (!seen.insert(k).second) return FST_E_DUP_NAME;
        h.metadata.emplace_back(std::move(k), std::move(v));
        c.ws();
        if (c.eat(',')) continue;
        if (c.eat('}')) return FST_OK;
        return FST_E_JSON;
    }
}

struct RawEntry {
    bool has_dtype = false, has_shape = false, has_offsets = false;
    std::string dtype;
    uint64_t shape[FST_MAX_DIMS] = {};
    size_t ndim = 0;
    uint64_t offs[2] = {};
    size_t noffs = 0;
};

int tensor_object(Cursor &c, RawEntry &e)
{
    if (!c.eat('{')) return wrong_type(c);
    c.ws();
    if (c.eat('}')) return FST_E_SCHEMA;
    while (true) {
        c.ws();
        std::string k;
        if (int rc = c.string(k)) return rc;
        c.ws();
        if (!c.eat(':')) return FST_E_JSON;
        c.ws();
        if (k == "dtype") {
            if (e.has_dtype) return FST_E_DUP_NAME;
            if (c.peek() != '"') return wrong_type(c);
            if (int rc = c.string(e.dtype)) return rc;
            e.has_dtype = true;
        } else if (k == "shape") {
            if (e.has_shape) return FST_E_DUP_NAME;
            if (int rc = u64_array(c, e.shape, FST_MAX_DIMS, e.ndim)) return rc;
            e.has_shape = true;
        } else if (k == "data_offsets") {
            if (e.has_offsets) return FST_E_DUP_NAME;
            if (int rc = u64_array(c, e.offs, 2, e.noffs)) return rc;
            e.has_offsets = true;
        } else {
            return FST_E_SCHEMA;    // a layout entry has exactly three fields
        }
        c.ws();
        if (c.eat(',')) continue;
        if (c.eat('}')) break;
        return FST_E_JSON;
    }
    if (!(e.has_dtype && e.has_shape && e.has_offsets) || e.noffs != 2) return FST_E_SCHEMA;
    return FST_OK;
}

}  // namespace
}  // namespace fst

using namespace fst;

extern "C" {

const char *fst_last_error(void) { return g_error; }

const char *fst_status_name(int s)
{
    switch (s) {
    case FST_OK: return "FST_OK";
    case FST_E_TRUNCATED: return "FST_E_TRUNCATED";
    case FST_E_HEADER_SIZE: return "FST_E_HEADER_SIZE";
    case FST_E_JSON: return "FST_E_JSON";
    case FST_E_SCHEMA: return "FST_E_SCHEMA";
    case FST_E_DTYPE: return "FST_E_DTYPE";
    case FST_E_SIZE_MISMATCH: return "FST_E_SIZE_MISMATCH";
    case FST_E_OFFSETS: return "FST_E_OFFSETS";
    case FST_E_DUP_NAME: return "FST_E_DUP_NAME";
    case FST_E_NOT_FOUND: return "FST_E_NOT_FOUND";
    case FST_E_SHARD: return "FST_E_SHARD";
    case FST_E_CAST: return "FST_E_CAST";
    case FST_E_ALIGN: return "FST_E_ALIGN";
    case FST_E_RANGE: return "FST_E_RANGE";
    case FST_E_HIP: return "FST_E_HIP";
    case FST_E_NOMEM: return "FST_E_NOMEM";
    case FST_E_IO: return "FST_E_IO";
    case FST_E_ARG: return "FST_E_ARG";
    default: return "FST_E_?";
    }
}

const char *fst_dtype_name(int d) { return d >= 0 && d < FST_DTYPE_COUNT ? kDtypes[d].name : nullptr; }
size_t fst_dtype_size(int d) { return d >= 0 && d < FST_DTYPE_COUNT ? kDtypes[d].size : 0; }

int fst_dtype_from_name(const char *s, size_t len)
{
    if (s)
        for (int d = 0; d < FST_DTYPE_COUNT; ++d)
            if (strlen(kDtypes[d].name) == len && memcmp(kDtypes[d].name, s, len) == 0) return d;
    return FST_E_DTYPE;
}

int fst_header_len(const void *first8, size_t nbytes, uint64_t *n_out)
{
    if (!first8 || !n_out) return fail(FST_E_ARG, "fst_header_len: NULL argument");
    if (nbytes < 8) return fail(FST_E_TRUNCATED, "need 8 bytes for the header size, got %zu", nbytes);
    const uint8_t *b = static_cast<const uint8_t *>(first8);
    uint64_t n = 0;
    for (int i = 0; i < 8; ++i) n |= uint64_t(b[i]) << (8 * i);
    *n_out = n;
    return FST_OK;
}

static int parse_header_impl(const void *bytes, size_t nbytes, uint64_t file_size, fst_header **out)
{
    if (!out) return fail(FST_E_ARG, "fst_parse_header: out is NULL");
    *out = nullptr;
    if (!bytes) return fail(FST_E_ARG, "fst_parse_header: bytes is NULL");
    uint64_t n = 0;
    if (int rc = fst_header_len(bytes, nbytes, &n)) return rc;
    if (n < 2 || n > FST_MAX_HEADER_BYTES)
        return fail(FST_E_HEADER_SIZE, "header size %llu outside [2, %llu]", (unsigned long long)n,
                    (unsigned long long)FST_MAX_HEADER_BYTES);
    if (n > file_size || 8 > file_size - n)
        return fail(FST_E_HEADER_SIZE, "header (8+%llu bytes) is longer than the file (%llu bytes)",
                    (unsigned long long)n, (unsigned long long)file_size);
    if (nbytes < 8 + n)
        return fail(FST_E_TRUNCATED, "header needs %llu bytes, %zu given", (unsigned long long)(8 + n), nbytes);

    // owned here until handed to the caller: an exception on the way (out of memory in a container)
    // frees the half-built header
    std::unique_ptr<fst_header> owner(new (std::nothrow) fst_header);
    fst_header *h = owner.get();
    if (!h) return fail(FST_E_NOMEM, "out of memory");
    h->n_json = n;
    h->file_size = file_size;
    const uint64_t body_len = file_size - 8 - n;
    const uint8_t *text = static_cast<const uint8_t *>(bytes) + 8;
    Cursor c(text, text + n);
    int rc = FST_OK;
    std::string key;
    auto bail = [&](int status, const char *what) {
        fail(status, "%s (near header byte %zu%s%s)", what, c.pos(text), key.empty() ? "" : ", key ",
             key.c_str());
        return status;
    };

    if (!c.eat('{')) return bail(FST_E_JSON, "header text does not start with '{'");
    c.ws();
    bool closed = c.eat('}');
    while (!closed) {
        c.ws();
        key.clear();
        if ((rc = c.string(key))) return bail(rc, "bad key");
        c.ws();
        if (!c.eat(':')) return bail(FST_E_JSON, "expected ':'");
        c.ws();
        if (key == "__metadata__") {
            if (!h->metadata.empty() || h->index.count(key)) return bail(FST_E_DUP_NAME, "key appears twice");
            h->index.emplace(key, SIZE_MAX);           // remembered only to catch a repeat
            if ((rc = metadata_object(c, *h))) return bail(rc, "bad __metadata__");
        } else {
            RawEntry e;
            if ((rc = tensor_object(c, e))) return bail(rc, "bad layout entry");
            if (h->index.count(key)) return bail(FST_E_DUP_NAME, "key appears twice");
            Tensor t;
            int dt = fst_dtype_from_name(e.dtype.data(), e.dtype.size());
            if (dt < 0) return bail(FST_E_DTYPE, "unknown dtype");
            if (e.ndim > FST_MAX_DIMS) return bail(FST_E_RANGE, "more than FST_MAX_DIMS dimensions");
            t.dtype = dt;
            t.ndim = int32_t(e.ndim);
            bool empty = false, overflow = false;
            uint64_t numel = 1;
            for (size_t d = 0; d < e.ndim; ++d) {
                t.shape[d] = e.shape[d];
                if (e.shape[d] == 0) empty = true;
                else if (numel > UINT64_MAX / e.shape[d]) overflow = true;
                else numel *= e.shape[d];
            }
            if (empty) { numel = 0; overflow = false; }
            t.begin = e.offs[0];
            t.end = e.offs[1];
            if (t.begin > t.end) return bail(FST_E_OFFSETS, "data_offsets run backwards");
            const uint64_t es = kDtypes[dt].size;
            if (overflow || numel > UINT64_MAX / es || t.end - t.begin != numel * es)
                return bail(FST_E_SIZE_MISMATCH, "data_offsets do not match shape and dtype");
            t.name = key;
            h->index.emplace(key, h->tensors.size());
            h->tensors.push_back(std::move(t));
        }
        c.ws();
        if (c.eat(',')) continue;
        if (c.eat('}')) break;
        return bail(FST_E_JSON, "expected ',' or '}'");
    }
    c.ws();
    key.clear();
    if (!c.at_end()) return bail(FST_E_JSON, "text after the closing brace");
    h->index.erase("__metadata__");

    // order by offset (empty tensors first on a shared boundary) and require an exact tiling
    std::stable_sort(h->tensors.begin(), h->tensors.end(), [](const Tensor &a, const Tensor &b) {
        return a.begin != b.begin ? a.begin < b.begin : a.end < b.end;
    });
    uint64_t at = 0;
    for (size_t i = 0; i < h->tensors.size(); ++i) {
        const Tensor &t = h->tensors[i];
        if (t.begin != at) {
            key = t.name;
            return bail(FST_E_OFFSETS, t.begin < at ? "tensor overlaps its predecessor" : "hole before tensor");
        }
        at = t.end;
        h->index[t.name] = i;
    }
    if (at != body_len) return bail(FST_E_OFFSETS, "tensors do not end where the file ends");
    *out = owner.release();
    return FST_OK;
}

int fst_parse_header(const void *bytes, size_t nbytes, uint64_t file_size, fst_header **out)
{
    try {
        return parse_header_impl(bytes, nbytes, file_size, out);
    } catch (const std::bad_alloc &) {
        if (out) *out = nullptr;     // the half-built header is lost only when memory ran out
        return fail(FST_E_NOMEM, "out of memory");
    } catch (...) {
        if (out) *out = nullptr;
        return fail(FST_E_ARG, "unexpected internal error");
    }
}

size_t fst_header_count(const fst_header *h) { return h ? h->tensors.size() : 0; }

int fst_header_tensor(const fst_header *h, size_t i, fst_tensor_info *out)
{
    if (!h || !out) return fail(FST_E_ARG, "fst_header_tensor: NULL argument");
    if (i >= h->tensors.size()) return fail(FST_E_RANGE, "tensor index %zu out of range", i);
    const Tensor &t = h->tensors[i];
    out->name = t.name.c_str();
    out->name_len = t.name.size();
    out->dtype = t.dtype;
    out->ndim = t.ndim;
    for (int d = 0; d < FST_MAX_DIMS; ++d) out->shape[d] = d < t.ndim ? t.shape[d] : 0;
    out->begin = t.begin;
    out->end = t.end;
    return FST_OK;
}

int64_t fst_header_find(const fst_header *h, const char *name)
{
    if (!h || !name) return fail(FST_E_ARG, "fst_header_find: NULL argument");
    auto it = h->index.find(name);
    if (it == h->index.end()) return fail(FST_E_NOT_FOUND, "no tensor named %s", name);
    return int64_t(it->second);
}

uint64_t fst_header_body_offset(const fst_header *h) { return h ? 8 + h->n_json : 0; }
uint64_t fst_aligned_phase(const fst_header *h)
{
    return h ? (FST_RAW_ALIGN - (8 + h->n_json) % FST_RAW_ALIGN) % FST_RAW_ALIGN : 0;
}
uint64_t fst_header_file_size(const fst_header *h) { return h ? h->file_size : 0; }
size_t fst_header_metadata_count(const fst_header *h) { return h ? h->metadata.size() : 0; }

int fst_header_metadata(const fst_header *h, size_t i, const char **key, const char **value)
{
    if (!h || !key || !value) return fail(FST_E_ARG, "fst_header_metadata: NULL argument");
    if (i >= h->metadata.size()) return fail(FST_E_RANGE, "metadata index %zu out of range", i);
    *key = h->metadata[i].first.c_str();
    *value = h->metadata[i].second.c_str();
    return FST_OK;
}

void fst_header_free(fst_header *h) { delete h; }

}  // extern "C"
