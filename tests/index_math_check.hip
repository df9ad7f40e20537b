// Host-side check of the index arithmetic the kernels use to map a thread number to (row, position)
// or (bag, word): compiled with hipcc and run on the CPU by tests/test_index_math.py.  Every value is
// compared with plain 64-bit (or 128-bit) integer division around the 2^32 boundary, where the
// kernels switch from 32-bit to 64-bit division.
#include <cstdint>
#include <cstdio>

#include "../paper_1911_02079_amd/csrc/e4q_index.h"

static int failures = 0;

static void check_item(int64_t t, int64_t n_items, uint32_t per)
{
    const int64_t want_group = (int64_t)((unsigned __int128)t / per);
    const uint32_t want_off = (uint32_t)((unsigned __int128)t % per);
    const int64_t g = e4q::group_of(t, n_items, per);
    const int64_t gt = e4q::needs_wide_index(n_items) ? e4q::group_of<true>(t, per) : e4q::group_of<false>(t, per);
    const uint32_t off = e4q::offset_in_group(t, g, per);
    if (g != want_group || gt != want_group || off != want_off) {
        if (failures++ < 20)
            std::printf("MISMATCH t=%lld n=%lld per=%u: group %lld/%lld want %lld, offset %u want %u\n", (long long)t,
                        (long long)n_items, per, (long long)g, (long long)gt, (long long)want_group, off, want_off);
    }
}

int main()
{
    const int64_t two32 = 0x100000000LL;
    const uint32_t pers[] = {1, 2, 3, 4, 7, 8, 16, 25, 32, 100, 127, 128, 255, 256, 512, 1000, 1024, 4095, 4096};
    long checked = 0;
    for (uint32_t per : pers) {
        // item counts just below, at and above 2^32 (multiples of `per`, as n_bags * per is)
        for (int64_t base : {two32 - 4096, two32 - 256, two32 - 255, two32 - 1, two32, two32 + 1, two32 + 255, two32 + 4096,
                             3 * two32 + 17, (int64_t)1 << 40}) {
            const int64_t n_items = (base + per - 1) / per * per;
            // thread numbers a padded grid of 256-thread blocks can produce, valid ones only (the
            // kernels return first for t >= n_items)
            const int64_t probes[] = {0, 1, per - 1, per, per + 1, n_items / 2, two32 - 257, two32 - 256, two32 - 2, two32 - 1,
                                      two32, two32 + 1, two32 + 255, n_items - per - 1, n_items - per, n_items - 2, n_items - 1};
            for (int64_t t : probes) {
                if (t < 0 || t >= n_items) continue;
                check_item(t, n_items, per);
                ++checked;
            }
        }
    }
    // Launch shapes: every workgroup number 0 .. n_blocks - 1 is reached exactly once by
    // y * grid.x + x, no grid dimension holds 2^32 work-items or more (a larger one-dimensional
    // launch silently runs a truncated grid), and the padding stays below one row of the grid.
    for (int64_t n_blocks : {(int64_t)1, (int64_t)255, e4q::kMaxGridX - 1, e4q::kMaxGridX, e4q::kMaxGridX + 1,
                             (int64_t)16777412 /* 2^32 / 256 + 196 */, (int64_t)0x7fffffff, e4q::kMaxGridX * e4q::kMaxGridY}) {
        const dim3 g = e4q::grid_for(n_blocks);
        const int64_t covered = (int64_t)g.x * g.y;
        if (g.z != 1 || (int64_t)g.x * 1024 >= two32 || g.y > e4q::kMaxGridY || covered < n_blocks ||
            covered - n_blocks >= (int64_t)g.x || (g.y > 1 && g.x != e4q::kMaxGridX)) {
            ++failures;
            std::printf("grid_for(%lld) = (%u, %u, %u)\n", (long long)n_blocks, g.x, g.y, g.z);
        }
    }
    for (int64_t n_items : {two32 - 100, two32 - 1, two32, two32 + 1}) {
        const int64_t last = e4q::blocks_for(n_items, 256) * 256 - 1;
        if (!(last >= n_items - 1 && last < n_items + 255)) { ++failures; std::printf("blocks_for wrong at %lld\n", (long long)n_items); }
    }
    if (e4q::blocks_for(e4q::kMaxGridX * e4q::kMaxGridY * 256 + 1, 256) != -1) { ++failures; std::printf("blocks_for must refuse an oversized grid\n"); }
    if (e4q::blocks_for(e4q::kMaxGridX * e4q::kMaxGridY * 256, 256) != e4q::kMaxGridX * e4q::kMaxGridY) { ++failures; std::printf("blocks_for largest grid\n"); }
    if (e4q::needs_wide_index(two32) || !e4q::needs_wide_index(two32 + 1)) { ++failures; std::printf("needs_wide_index boundary\n"); }
    std::printf("checked %ld items, %d failures\n", checked, failures);
    return failures == 0 ? 0 : 1;
}
