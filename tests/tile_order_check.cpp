// CPU check of the workgroup order used by the row x tile kernels.  For many
// (rows, tiles, super, chunk):
//  - every (row, tile) pair is decoded by exactly one workgroup of the planned
//    grid, and at most 7 workgroups per row have no tile;
//  - the XCD (wg & 7) that owns a tile is the one a greedy dealer gives it:
//    rounds of eight equal chunks, largest size first, each smaller power of
//    two while it still fits, single tiles at the end;
//  - an XCD walks the tiles of a row in address order, takes the rows of a tile
//    in order, and comes back to a tile for the next row after at most one
//    super-chunk of other work;
//  - decoded as a single row (the gbest copy does that), the same order gives
//    every tile once, on the XCD that owns it in the K-row pass.
// Built by tests/test_tile_order.py against the library's own header.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "tile_order.h"

static int check(int rows, unsigned long long tiles, unsigned long long super, unsigned long long chunk) {
    TileOrder ord;
    unsigned long long grid = 0;
    if (!plan_tile_order(rows, tiles, super, chunk, &ord, &grid)) return 1;
    if (grid % 8 != 0 || grid < (unsigned long long)rows * tiles) return 2;
    if (grid > (unsigned long long)rows * (tiles + 7)) return 3;

    // Owner of every tile by the greedy dealer.
    std::vector<int> owner((size_t)tiles, -1);
    {
        unsigned long long size = chunk > super ? super : chunk, pos = 0;
        for (; size >= 1; size >>= 1)
            while (tiles - pos >= 8 * size)
                for (int x = 0; x < 8; ++x)
                    for (unsigned long long k = 0; k < size; ++k) owner[(size_t)pos++] = x;
        for (int x = 0; pos < tiles; ++x) owner[(size_t)pos++] = x;
    }

    std::vector<unsigned char> seen((size_t)rows * tiles, 0);
    std::vector<int> next_row((size_t)tiles, 0);
    std::vector<unsigned long long> first_visit((size_t)tiles, 0);
    std::vector<long long> prev_tile((size_t)rows * 8, -1);  // per (XCD, row): last tile taken
    for (unsigned long long wg = 0; wg < grid; ++wg) {
        unsigned row = ~0u, tile = ~0u;
        const bool live = decode_tile_order(ord, (unsigned)rows, (unsigned)wg, &row, &tile);
        if (!live) {
            if (row < (unsigned)rows && tile < tiles) return 4;  // a live pair reported as idle
            continue;
        }
        if (row >= (unsigned)rows || tile >= tiles) return 5;
        unsigned char& s = seen[(size_t)row * tiles + tile];
        if (s) return 6;  // handled twice
        s = 1;
        if (next_row[tile] != (int)row) return 7;  // rows of a tile not in order
        next_row[tile] = (int)row + 1;
        if (owner[tile] != (int)(wg & 7u)) return 8;  // not the greedy dealer's XCD
        long long& prev = prev_tile[(size_t)(wg & 7u) * rows + row];
        if ((long long)tile <= prev) return 10;  // an XCD's tiles of a row not in address order
        prev = (long long)tile;
        const unsigned long long j = wg >> 3;
        if (row == 0) first_visit[tile] = j;
        else if (j - first_visit[tile] > (unsigned long long)row << ord.super_log2) return 11;
    }
    for (unsigned char s : seen)
        if (!s) return 9;  // skipped

    // The gbest copy decodes the order of the K-row pass as a single row: the
    // plan must not depend on the number of rows, and every tile must come up
    // once, on the XCD that owns it in the K-row pass.
    TileOrder one;
    unsigned long long grid1 = 0;
    if (!plan_tile_order(1, tiles, super, chunk, &one, &grid1)) return 12;
    if (std::memcmp(&one, &ord, sizeof ord) != 0 || grid1 * (unsigned long long)rows != grid) return 13;
    std::vector<unsigned char> seen1((size_t)tiles, 0);
    for (unsigned long long wg = 0; wg < grid1; ++wg) {
        unsigned row = ~0u, tile = ~0u;
        if (!decode_tile_order(ord, 1u, (unsigned)wg, &row, &tile)) continue;
        if (row != 0 || tile >= tiles || seen1[tile]) return 14;
        seen1[tile] = 1;
        if (owner[tile] != (int)(wg & 7u)) return 15;
    }
    for (unsigned char s : seen1)
        if (!s) return 16;
    return 0;
}

int main() {
    unsigned long long state = 88172645463325252ull;
    auto rnd = [&](unsigned long long m) {
        state ^= state << 13; state ^= state >> 7; state ^= state << 17;
        return state % m;
    };
    int cases = 0;
    const unsigned long long fixed[][4] = {
        {1, 1, 1, 1}, {4, 199, 1024, 128}, {32, 49917, 1024, 128}, {8, 28767, 1024, 128},
        {5, 7, 2, 1}, {9, 274, 2, 1}, {9, 274, 8, 2}, {9, 1094, 32, 8}, {3, 4096, 16, 16},
        {130, 3, 1024, 128}, {16, 16 * 1024, 1024, 128}, {16, 16 * 1024 - 1, 1024, 128},
        {2, 100000, 1048576, 1}, {2, 100000, 1048576, 512}, {3, 8 * 1023, 1024, 128},
        {3, 8 * 1023 + 7, 1024, 128}, {3, 8 * 128, 1024, 128}, {3, 8 * 128 - 1, 1024, 128},
        {7, 8, 4, 4}, {7, 9, 4, 4}, {7, 15, 4, 4}, {7, 16, 4, 4}, {2, 1ull << 20, 1ull << 30, 1}};
    for (const auto& f : fixed) {
        const int rc = check((int)f[0], f[1], f[2], f[3]);
        if (rc) { std::printf("FAIL rc=%d rows=%llu tiles=%llu super=%llu chunk=%llu\n", rc, f[0], f[1], f[2], f[3]); return 1; }
        ++cases;
    }
    for (int it = 0; it < 3000; ++it) {
        const int rows = 1 + (int)rnd(40);
        const unsigned long long tiles = 1 + rnd(it % 3 ? 3000 : 60000);
        const unsigned long long super = 1ull << rnd(12);
        const unsigned long long chunk = 1ull << rnd(10);
        const int rc = check(rows, tiles, super, chunk);
        if (rc) { std::printf("FAIL rc=%d rows=%d tiles=%llu super=%llu chunk=%llu\n", rc, rows, tiles, super, chunk); return 1; }
        ++cases;
    }
    TileOrder ord; unsigned long long grid;
    if (plan_tile_order(64, (1ull << 31), 512, 64, &ord, &grid)) { std::printf("FAIL: oversized grid accepted\n"); return 1; }
    if (plan_tile_order(1 << 12, (1ull << 20), 512, 64, &ord, &grid)) { std::printf("FAIL: oversized grid accepted\n"); return 1; }
    std::printf("tile order ok: %d cases\n", cases);
    return 0;
}
