// Host-side brute force over the index arithmetic of the tile kernel's launches, under the sanitizers: the walk
// of the workgroup ids over the tiles, the planner that shares a ragged last round of tiles among the compute
// units, and the walk of the quantize kernel's workgroups over the blocks of its tensor.  Every tile, and every K step of every shared tile, must be computed exactly once, and every partial
// result must have a slot of its own inside the scratch the plan asks for.
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../../paper_2512_15306_amd/csrc/gemm_tile.h"
#include "../../paper_2512_15306_amd/csrc/llmq_device.h"

using namespace llmq;

static int g_fail = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            if (g_fail < 20) { printf("FAIL %s:%d %s: ", __FILE__, __LINE__, #cond); printf(__VA_ARGS__); printf("\n"); } \
            ++g_fail;                                     \
        }                                                 \
    } while (0)

static void check_walk(int n) {
    const int grid = ((n + kXcds - 1) / kXcds) * kXcds;
    std::vector<int> seen(n, 0);
    for (int pid = 0; pid < grid; ++pid) {
        const int pos = walk_position(pid, n);
        CHECK(pos >= -1 && pos < n, "n=%d pid=%d pos=%d", n, pid, pos);
        if (pos >= 0) ++seen[pos];
    }
    for (int p = 0; p < n; ++p) CHECK(seen[p] == 1, "n=%d position %d taken %d times", n, p, seen[p]);
    // workgroups of one XCD (ids congruent modulo the XCD count) take neighbouring positions in id order
    for (int pid = kXcds; pid < grid; ++pid) {
        const int a = walk_position(pid - kXcds, n), b = walk_position(pid, n);
        if (a >= 0 && b >= 0) CHECK(b == a + 1, "n=%d pid=%d: %d after %d", n, pid, b, a);
    }
}

static void check_tiles(int tiles_r, int tiles_c, int band) {
    const int nt = tiles_r * tiles_c;
    std::vector<int> seen(nt, 0);
    for (int pos = 0; pos < nt; ++pos) {
        int tr = -1, tc = -1;
        tile_of_position(pos, tiles_r, tiles_c, band, tr, tc);
        CHECK(tr >= 0 && tr < tiles_r && tc >= 0 && tc < tiles_c, "%d x %d band %d pos %d -> (%d, %d)", tiles_r, tiles_c, band, pos, tr, tc);
        if (tr >= 0 && tr < tiles_r && tc >= 0 && tc < tiles_c) ++seen[tr * tiles_c + tc];
    }
    for (int t = 0; t < nt; ++t) CHECK(seen[t] == 1, "%d x %d band %d: tile %d computed %d times", tiles_r, tiles_c, band, t, seen[t]);
}

// The walk of the quantize kernel's workgroups over the blocks of its tensor (band_walk): a bijection, also for the
// grids of very tall tensors, where band x grid_rows comes close to 2^32.
static void check_bands(unsigned gr, unsigned gc, unsigned band) {
    if (band > gc) band = gc;                      // as the launcher does
    const unsigned long long n = (unsigned long long)gr * gc;
    std::vector<unsigned char> seen(n, 0);
    for (unsigned long long id = 0; id < n; ++id) {
        unsigned br = ~0u, bc = ~0u;
        band_walk((unsigned)id, gr, gc, band, br, bc);
        CHECK(br < gr && bc < gc, "grid %u x %u band %u: id %llu -> (%u, %u)", gr, gc, band, id, br, bc);
        if (br < gr && bc < gc) {
            CHECK(seen[(size_t)br * gc + bc] == 0, "grid %u x %u band %u: block (%u, %u) twice", gr, gc, band, br, bc);
            seen[(size_t)br * gc + bc] = 1;
        }
    }
}

// Replays what the three launches of a contraction do with the plan, as the kernel's prologue does.
static void check_plan(int nt, int nk, int slots, size_t scratch_bytes, const char* mode) {
    const SplitChoice c = choose_split(nt, nk, slots, 4, 4, scratch_bytes);
    const size_t tile_bytes = 4u * 256 * 256;
    CHECK(c.n_whole >= 0 && c.n_whole <= nt, "nt=%d nk=%d %s: n_whole %d", nt, nk, mode, c.n_whole);
    if (c.n_groups == 0) {
        CHECK(c.n_whole == nt, "nt=%d nk=%d %s: nothing shared but n_whole %d", nt, nk, mode, c.n_whole);
        return;
    }
    CHECK(c.n_whole % slots == 0, "nt=%d nk=%d %s: n_whole %d is not whole rounds", nt, nk, mode, c.n_whole);
    CHECK(c.n_whole + c.shared_tiles == nt, "nt=%d nk=%d %s: %d + %d tiles", nt, nk, mode, c.n_whole, c.shared_tiles);
    CHECK(c.n_groups <= kMaxSplitGroups, "groups %d", c.n_groups);
    CHECK(c.slots * tile_bytes <= scratch_bytes, "nt=%d nk=%d %s: %zu slots do not fit %zu bytes", nt, nk, mode, c.slots, scratch_bytes);
    std::vector<int> slot_used(c.slots, 0);
    // steps[t][k]: how often K step k of shared tile t is computed
    std::vector<std::vector<int>> steps(c.shared_tiles, std::vector<int>(nk, 0));
    int tile_at = 0, wg_at = 0;
    bool any_cut = false;
    for (int g = 0; g < c.n_groups; ++g) {
        const SplitGroup& grp = c.group[g];
        CHECK(grp.tile_begin == tile_at && grp.wg_begin == wg_at, "nt=%d nk=%d %s group %d starts at tile %d wg %d, expected %d %d", nt, nk, mode, g, grp.tile_begin, grp.wg_begin, tile_at, wg_at);
        CHECK(grp.tiles >= 1 && grp.pieces >= 1 && grp.steps >= 1, "group %d empty", g);
        CHECK(grp.wgs % kXcds == 0 && grp.wgs >= grp.tiles * grp.pieces, "group %d: %d workgroups for %d x %d", g, grp.wgs, grp.tiles, grp.pieces);
        CHECK(grp.pieces == 1 || grp.tiles * grp.pieces <= slots, "nt=%d nk=%d %s group %d: %d pieces at once on %d slots", nt, nk, mode, g, grp.tiles * grp.pieces, slots);
        CHECK((grp.pieces - 1) * grp.steps < nk && grp.pieces * grp.steps >= nk, "nt=%d nk=%d %s group %d: %d pieces of %d steps", nt, nk, mode, g, grp.pieces, grp.steps);
        any_cut = any_cut || grp.pieces > 1;
        // the pieces launch
        for (int q = grp.wg_begin; q < grp.wg_begin + grp.wgs; ++q) {
            const int w = walk_position(q - grp.wg_begin, grp.tiles * grp.pieces);
            if (w < 0) continue;
            const int piece = w / grp.tiles, j = w - piece * grp.tiles;
            const int kb = piece * grp.steps;
            int n = nk - kb < grp.steps ? nk - kb : grp.steps;
#ifdef LLMQ_PLANT_SHORT_PIECES      // a replay that drops the last K step of every last piece: the checks must notice
            if (grp.pieces > 1 && piece == grp.pieces - 1) --n;
#endif
            CHECK(n >= 0, "nt=%d nk=%d %s group %d: empty piece %d", nt, nk, mode, g, piece);
#ifndef LLMQ_PLANT_SHORT_PIECES
            CHECK(n > 0, "nt=%d nk=%d %s group %d: empty piece %d", nt, nk, mode, g, piece);
#endif
            const int slot = grp.wg_begin + j * grp.pieces + piece;
            CHECK(slot >= 0 && (size_t)slot < c.slots, "slot %d of %zu", slot, c.slots);
            if (slot >= 0 && (size_t)slot < c.slots) ++slot_used[slot];
            for (int k = kb; k < kb + n && k < nk; ++k) ++steps[grp.tile_begin + j][k];
        }
        // the fix-up launch reads slots [first, first + pieces) of tile j in this order
        for (int j = 0; j < grp.tiles; ++j) {
            const int first = grp.wg_begin + j * grp.pieces;
            for (int p = 0; p < grp.pieces; ++p) CHECK(slot_used[first + p] == 1, "nt=%d nk=%d %s group %d tile %d piece %d: slot written %d times", nt, nk, mode, g, j, p, slot_used[first + p]);
        }
        tile_at += grp.tiles;
        wg_at += grp.wgs;
    }
    CHECK(tile_at == c.shared_tiles && wg_at == c.share_wgs, "nt=%d nk=%d %s: groups hold %d tiles %d workgroups, plan says %d %d", nt, nk, mode, tile_at, wg_at, c.shared_tiles, c.share_wgs);
    CHECK(any_cut, "nt=%d nk=%d %s: a plan that cuts nothing", nt, nk, mode);
    for (int t = 0; t < c.shared_tiles; ++t)
        for (int k = 0; k < nk; ++k) CHECK(steps[t][k] == 1, "nt=%d nk=%d %s: K step %d of shared tile %d computed %d times", nt, nk, mode, k, t, steps[t][k]);
}

int main() {
    for (int n = 1; n <= 1100; n += (n < 300 ? 1 : 37)) check_walk(n);
    check_walk(13824);
    const int bands[] = {1, 2, 3, 4, 8, 64};
    for (int r = 1; r <= 40; r += (r < 10 ? 1 : 7))
        for (int c = 1; c <= 220; c += (c < 10 ? 1 : 23))
            for (int b : bands) check_tiles(r, c, b);
    check_tiles(64, 216, 4);
    const unsigned band_sizes[] = {1, 2, 3, 7, 16, 1u << 20};
    for (unsigned gr : {1u, 2u, 5u, 64u, 130u})
        for (unsigned gc : {1u, 2u, 3u, 14u, 20u, 33u})
            for (unsigned b : band_sizes) check_bands(gr, gc, b);
    for (unsigned b : band_sizes) {
        check_bands(4096, 20, b);                  // 524288 rows: 2^20 x 4096 would wrap to 0 without the clamp
        check_bands(3 * 4096 + 1, 7, b);
        check_bands(1u << 20, 2, b);               // 2^27 rows
    }
    const char* modes[] = {nullptr, "1", "a2", "a3", "a5", "a16", "0"};
    const int nks[] = {1, 2, 7, 8, 15, 16, 28, 40, 63, 64, 65, 108, 128, 216, 432};
    const int slot_counts[] = {256, 64, 8};
    for (const char* mode : modes) {
        if (mode) setenv("LLMQ_GEMM_SPLIT", mode, 1);
        else unsetenv("LLMQ_GEMM_SPLIT");
        for (int slots : slot_counts)
            for (int nk : nks)
                for (int nt = 1; nt <= 3 * slots + 5; nt += (slots > 64 && nt > 20 ? 3 : 1)) {
                    check_plan(nt, nk, slots, (size_t)1 << 40, mode ? mode : "default");
                    check_plan(nt, nk, slots, (size_t)64 << 20, mode ? mode : "default");      // 256 binary32 tiles
                    check_plan(nt, nk, slots, 0, mode ? mode : "default");
                }
    }
    unsetenv("LLMQ_GEMM_SPLIT");
    // what the default rule shares: long contractions whose left-over tiles fit one group
    CHECK(choose_split(560, 128, 256, 4, 4, (size_t)1 << 40).n_groups == 1, "560 tiles x 128 steps");
    CHECK(choose_split(560, 128, 256, 4, 4, 0).n_groups == 0, "no scratch, no sharing");
    CHECK(choose_split(448, 296, 256, 4, 4, (size_t)1 << 40).n_groups == 0, "192 left-over tiles need two groups");
    CHECK(choose_split(560, 40, 256, 4, 4, (size_t)1 << 40).n_groups == 0, "short contraction");
    CHECK(choose_split(512, 128, 256, 4, 4, (size_t)1 << 40).n_groups == 0, "whole rounds");
    if (g_fail) { printf("%d checks failed\n", g_fail); return 1; }
    printf("planner driver ok\n");
    return 0;
}
