// Drives the staging ring on the fake runtime: synthetic files of many small tensors (vectors and
// matrices of which one rank's column share is taken) held in memory, small ring slots that several
// reader threads fill together; resident, streamed, packed and compacted runs.  Checks that the
// staged bytes are the file's bytes and that the first byte of every output arrived; the race
// detector watches the rest.  Exit code 0 = all checks passed.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "fst.h"

namespace {

struct MemFile { std::vector<uint8_t> bytes; };

int read_mem(void *ctx, int32_t file, uint64_t off, void *dst, uint64_t len)
{
    const MemFile *f = static_cast<const MemFile *>(ctx) + file;
    if (off + len > f->bytes.size()) return -1;
    std::memcpy(dst, f->bytes.data() + off, len);
    return 0;
}

// Every third tensor is a matrix [rows, 2*seg] (its second column half is what rank 1 of 2 takes).
MemFile make_file(int n_tensors, uint32_t seed, std::vector<std::string> &names, const char *prefix,
                  std::vector<uint64_t> *share_begin = nullptr)
{
    std::string json = "{";
    std::vector<uint64_t> sizes;
    uint64_t at = 0;
    for (int i = 0; i < n_tensors; ++i) {
        seed = seed * 1664525u + 1013904223u;
        uint64_t n = 1 + (seed >> 8) % 9000;
        const std::string name = std::string(prefix) + std::to_string(i);
        names.push_back(name);
        std::string shape = std::to_string(n);
        uint64_t first = at;                              // body offset of the first byte rank 1 of 2 keeps
        if (share_begin && i % 3 == 0) {
            const uint64_t rows = 3 + (seed >> 4) % 60, seg = 8 + (seed >> 12) % 150;
            n = rows * 2 * seg;
            shape = std::to_string(rows) + "," + std::to_string(2 * seg);
            first = at + seg;
        }
        if (share_begin) share_begin->push_back(first);
        json += (i ? "," : "") + ("\"" + name + "\":{\"dtype\":\"U8\",\"shape\":[" + shape + "],\"data_offsets\":[" +
                                  std::to_string(at) + "," + std::to_string(at + n) + "]}");
        at += n;
        sizes.push_back(n);
    }
    json += "}";
    MemFile f;
    f.bytes.resize(8 + json.size() + at);
    uint64_t n_json = json.size();
    for (int k = 0; k < 8; ++k) f.bytes[k] = uint8_t(n_json >> (8 * k));
    std::memcpy(f.bytes.data() + 8, json.data(), json.size());
    for (uint64_t i = 0; i < at; ++i) { seed = seed * 1664525u + 1013904223u; f.bytes[8 + json.size() + i] = uint8_t(seed >> 24); }
    return f;
}

#define CHECK(cond)                                                                   \
    do { if (!(cond)) { std::fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, fst_last_error()); std::exit(1); } } while (0)

}  // namespace

int main()
{
    std::vector<std::string> names;
    std::vector<MemFile> files;
    files.push_back(make_file(60, 1, names, "a."));
    files.push_back(make_file(45, 2, names, "b."));
    std::vector<fst_header *> hdrs(files.size());
    std::vector<uint64_t> bases;
    uint64_t raw_len = 0;
    for (size_t f = 0; f < files.size(); ++f) {
        uint64_t n = 0;
        CHECK(fst_header_len(files[f].bytes.data(), 8, &n) == FST_OK);
        CHECK(fst_parse_header(files[f].bytes.data(), 8 + n, files[f].bytes.size(), &hdrs[f]) == FST_OK);
        bases.push_back(raw_len);
        raw_len += (files[f].bytes.size() + 255) / 256 * 256;
    }
    std::vector<const char *> cnames;
    for (const std::string &s : names) cnames.push_back(s.c_str());

    for (int pass = 0; pass < 2; ++pass) {
        const bool streamed = pass == 1;
        std::vector<uint64_t> zero(files.size(), 0);
        fst_plan *plan = nullptr;
        CHECK(fst_plan_uniform(hdrs.data(), streamed ? zero.data() : bases.data(), files.size(), cnames.data(), cnames.size(),
                               FST_KEEP, -1, 0, 1, &plan) == FST_OK);
        size_t ng = 0;
        CHECK(fst_plan_set_groups(plan, 65536, &ng) == FST_OK && ng > 5);
        const size_t n_out = fst_plan_output_count(plan);
        std::vector<std::vector<uint8_t>> outs(n_out);
        std::vector<void *> ptrs(n_out);
        for (size_t i = 0; i < n_out; ++i) {
            fst_output_info info;
            CHECK(fst_plan_output(plan, i, &info) == FST_OK);
            outs[i].assign(info.nbytes + 512, 0);
            ptrs[i] = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(outs[i].data()) + 255) / 256 * 256);
        }
        std::vector<uint8_t> ws_store(fst_plan_workspace_bytes(plan) + 256);
        void *ws = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(ws_store.data()) + 255) / 256 * 256);
        fst_stager_config cfg{3, 6, 16384};      // blocks of up to 16 KiB, read in four parts
        fst_stager *st = nullptr;
        CHECK(fst_stager_create(&cfg, &st) == FST_OK);
        fst_stage_stats stats{};
        if (!streamed) {
            std::vector<uint8_t> raw_store(raw_len + 256, 0xEE);
            uint8_t *raw = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(raw_store.data()) + 255) / 256 * 256);
            for (int rep = 0; rep < 3; ++rep)
                CHECK(fst_stage_resident(st, plan, read_mem, files.data(), raw, raw_len, ptrs.data(), ws,
                                         fst_plan_workspace_bytes(plan), 0, &stats) == FST_OK);
            for (size_t f = 0; f < files.size(); ++f) {
                uint64_t n = 0;
                fst_header_len(files[f].bytes.data(), 8, &n);
                CHECK(std::memcmp(raw + bases[f] + 8 + n, files[f].bytes.data() + 8 + n, files[f].bytes.size() - 8 - n) == 0);
            }
        } else {
            std::vector<std::vector<uint8_t>> slot_store(3, std::vector<uint8_t>(65536 + 512));
            std::vector<void *> slots;
            for (auto &s : slot_store) slots.push_back(reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(s.data()) + 255) / 256 * 256));
            for (int rep = 0; rep < 3; ++rep)
                CHECK(fst_stage_streamed(st, plan, read_mem, files.data(), slots.data(), slots.size(), 65536, ptrs.data(), ws,
                                         fst_plan_workspace_bytes(plan), 0, &stats) == FST_OK);
        }
        // the stand-in for a kernel copies the first source byte of every piece to its output
        size_t at = 0;
        for (size_t f = 0; f < files.size(); ++f) {
            uint64_t n = 0;
            fst_header_len(files[f].bytes.data(), 8, &n);
            const size_t cnt = fst_header_count(hdrs[f]);
            for (size_t i = 0; i < cnt; ++i, ++at) {
                fst_tensor_info ti;
                CHECK(fst_header_tensor(hdrs[f], i, &ti) == FST_OK);
                size_t oi = 0;
                while (oi < names.size() && names[oi] != std::string(ti.name, ti.name_len)) ++oi;
                CHECK(oi < names.size());
                CHECK(*static_cast<uint8_t *>(ptrs[oi]) == files[f].bytes[8 + n + ti.begin]);
            }
        }
        std::printf("%s: %llu bytes in %llu copies, %zu groups\n", streamed ? "streamed" : "resident",
                    (unsigned long long)stats.staged_bytes, (unsigned long long)stats.n_copies, ng);
        fst_stager_destroy(st);
        fst_plan_free(plan);
    }
    // column shares (rank 1 of 2 along dim 1 of every matrix), staged sparsely and with the row segments
    // compacted: packed into one buffer, and streamed through three device slots
    {
        std::vector<std::string> mnames;
        std::vector<uint64_t> first;
        std::vector<MemFile> mfiles;
        mfiles.push_back(make_file(40, 7, mnames, "m.", &first));
        fst_header *mh = nullptr;
        uint64_t n = 0;
        CHECK(fst_header_len(mfiles[0].bytes.data(), 8, &n) == FST_OK);
        CHECK(fst_parse_header(mfiles[0].bytes.data(), 8 + n, mfiles[0].bytes.size(), &mh) == FST_OK);
        std::vector<const char *> cn;
        std::vector<fst_request> reqs;
        for (size_t i = 0; i < mnames.size(); ++i) {
            cn.push_back(mnames[i].c_str());
            reqs.push_back(fst_request{FST_KEEP, i % 3 == 0 ? 1 : -1, 1, -1});
        }
        const uint64_t zero = 0;
        for (int pass = 0; pass < 2; ++pass) {
            fst_plan *plan = nullptr;
            CHECK(fst_plan_create(&mh, &zero, 1, cn.data(), reqs.data(), cn.size(), 1, 2, &plan) == FST_OK);
            size_t ng = 0;
            CHECK(fst_plan_set_groups_compact(plan, 32768, 64, 8, &ng) == FST_OK && ng > 3);
            const size_t n_out = fst_plan_output_count(plan);
            std::vector<std::vector<uint8_t>> outs(n_out);
            std::vector<void *> ptrs(n_out);
            for (size_t i = 0; i < n_out; ++i) {
                fst_output_info info;
                CHECK(fst_plan_output(plan, i, &info) == FST_OK);
                outs[i].assign(info.nbytes + 512, 0);
                ptrs[i] = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(outs[i].data()) + 255) / 256 * 256);
            }
            std::vector<uint8_t> ws_store(fst_plan_workspace_bytes(plan) + 256);
            void *ws = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(ws_store.data()) + 255) / 256 * 256);
            fst_stager_config cfg{3, 6, 4096};
            fst_stager *st = nullptr;
            CHECK(fst_stager_create(&cfg, &st) == FST_OK);
            fst_stage_stats stats{};
            if (pass == 0) {
                std::vector<uint8_t> store(fst_plan_packed_bytes(plan) + 256, 0xEE);
                uint8_t *packed = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(store.data()) + 255) / 256 * 256);
                for (int rep = 0; rep < 3; ++rep)
                    CHECK(fst_stage_packed(st, plan, read_mem, mfiles.data(), packed, fst_plan_packed_bytes(plan), ptrs.data(), ws,
                                           fst_plan_workspace_bytes(plan), 0, &stats) == FST_OK);
            } else {
                std::vector<std::vector<uint8_t>> slot_store(3, std::vector<uint8_t>(32768 + 512));
                std::vector<void *> slots;
                for (auto &s : slot_store) slots.push_back(reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(s.data()) + 255) / 256 * 256));
                for (int rep = 0; rep < 3; ++rep)
                    CHECK(fst_stage_streamed(st, plan, read_mem, mfiles.data(), slots.data(), slots.size(), 32768, ptrs.data(), ws,
                                             fst_plan_workspace_bytes(plan), 0, &stats) == FST_OK);
            }
            // what is staged is what the rank reads: half of every matrix, all of every vector
            CHECK(stats.staged_bytes == fst_plan_read_bytes(plan));
            for (size_t i = 0; i < n_out; ++i)
                CHECK(*static_cast<uint8_t *>(ptrs[i]) == mfiles[0].bytes[8 + n + first[i]]);
            std::printf("%s, compacted: %llu bytes in %llu copies, %zu groups\n", pass ? "streamed" : "packed",
                        (unsigned long long)stats.staged_bytes, (unsigned long long)stats.n_copies, ng);
            fst_stager_destroy(st);
            fst_plan_free(plan);
        }
        fst_header_free(mh);
    }
    for (fst_header *h : hdrs) fst_header_free(h);
    std::puts("ok");
    return 0;
}
