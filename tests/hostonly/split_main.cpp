// Host-side check of how a launch class is cut into dispatches and of the permutation of the
// workgroups inside a dispatch: together they must visit every workgroup position of the class
// exactly once, and no dispatch may exceed what a grid can hold.  Compiled with g++ (no GPU).
#include <cstdio>
#include <vector>

#include "fst_internal.h"

using namespace fst;

static int check(uint32_t n_tiles, uint32_t max_tiles, bool visit)
{
    const std::vector<LaunchPart> parts = split_launch(n_tiles, max_tiles);
    uint64_t at = 0;
    std::vector<uint8_t> seen(visit ? n_tiles : 0, 0);
    for (size_t i = 0; i < parts.size(); ++i) {
        const LaunchPart &p = parts[i];
        if (p.wg_base != at || p.n_wg == 0 || p.n_wg > max_tiles) return 1;
        if (uint64_t(p.n_wg) * VEC_BLOCK_THREADS > 0xFFFFFFFFull) return 2;        // work-items of one dispatch
        if (i + 1 < parts.size() && p.n_wg % (XCD_COUNT * XCD_RUN)) return 3;    // whole spans but for the last
        if (visit)
            for (uint32_t wg = 0; wg < p.n_wg; ++wg) {
                const uint32_t t = p.wg_base + tile_of_workgroup(wg, p.n_wg);
                if (t >= n_tiles || seen[t]++) return 4;
            }
        at += p.n_wg;
    }
    if (at != n_tiles) return 5;
    for (uint8_t s : seen)
        if (s != 1) return 6;
    return 0;
}

int main()
{
    if (MAX_LAUNCH_WORKGROUPS % (XCD_COUNT * XCD_RUN) || uint64_t(MAX_LAUNCH_WORKGROUPS) * VEC_BLOCK_THREADS > 0xFFFFFFFFull ||
        uint64_t(MAX_LAUNCH_WORKGROUPS + XCD_COUNT * XCD_RUN) * VEC_BLOCK_THREADS <= 0xFFFFFFFFull) {
        std::printf("MAX_LAUNCH_WORKGROUPS = %u is not the largest whole number of spans that fits\n", MAX_LAUNCH_WORKGROUPS);
        return 1;
    }
    // every tile visited once, with a small limit so that many dispatches occur
    for (uint32_t max_tiles : {256u, 512u, 1024u})
        for (uint32_t n = 0; n < 3000; ++n)
            if (int rc = check(n, max_tiles, true)) { std::printf("n=%u max=%u rc=%d\n", n, max_tiles, rc); return 1; }
    // the real limit: sizes around it and the largest tile count a table can hold
    for (uint64_t n : {uint64_t(1), uint64_t(MAX_LAUNCH_WORKGROUPS) - 1, uint64_t(MAX_LAUNCH_WORKGROUPS), uint64_t(MAX_LAUNCH_WORKGROUPS) + 1,
                       2 * uint64_t(MAX_LAUNCH_WORKGROUPS) + 255, uint64_t(0x7FFFFFFF)})
        if (int rc = check(uint32_t(n), MAX_LAUNCH_WORKGROUPS, n < 3 * uint64_t(MAX_LAUNCH_WORKGROUPS))) {
            std::printf("n=%llu rc=%d\n", (unsigned long long)n, rc);
            return 1;
        }
    std::printf("ok\n");
    return 0;
}
