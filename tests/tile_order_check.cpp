// CPU check of the workgroup order used by the row x tile kernels: for many
// (rows, tiles, super, chunk) every (row, tile) pair must be decoded by exactly
// one workgroup of the planned grid, padding workgroups must say so, and each
// XCD (wg & 7) must see a tile for all rows before it leaves a super-chunk.
// Built by tests/test_tile_order.py against the library's own header.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "tile_order.h"

static int check(int rows, unsigned long long tiles, unsigned long long super, unsigned long long chunk,
                 bool explicit_super) {
    TileOrder ord;
    unsigned long long grid = 0;
    if (!plan_tile_order(rows, tiles, super, chunk, explicit_super, &ord, &grid)) return 1;
    if (grid % 8 != 0 || grid < (unsigned long long)rows * tiles) return 2;
    if (grid > (unsigned long long)rows * (tiles + 8ull * (1ull << ord.chunk_log2)) + 8ull * rows) return 3;
    std::vector<unsigned char> seen((size_t)rows * tiles, 0);
    // per XCD: the sequence of rows for one tile must be 0,1,..,rows-1 in order of wg
    std::vector<int> next_row((size_t)tiles, 0);
    for (unsigned long long wg = 0; wg < grid; ++wg) {
        unsigned row = ~0u, tile = ~0u;
        const bool live = decode_tile_order(ord, (unsigned)rows, (unsigned)wg, &row, &tile);
        if (!live) {
            if (row < (unsigned)rows && tile < tiles) return 4;  // a live pair reported as padding
            continue;
        }
        if (row >= (unsigned)rows || tile >= tiles) return 5;
        unsigned char& s = seen[(size_t)row * tiles + tile];
        if (s) return 6;  // handled twice
        s = 1;
        if (next_row[tile] != (int)row) return 7;  // rows of a tile not in order
        next_row[tile] = (int)row + 1;
        // the tile belongs to the XCD that runs this workgroup
        if (((tile >> ord.chunk_log2) & 7u) != (wg & 7u)) return 8;
    }
    for (unsigned char s : seen)
        if (!s) return 9;  // skipped
    return 0;
}

int main() {
    unsigned long long state = 88172645463325252ull;
    auto rnd = [&](unsigned long long m) {
        state ^= state << 13; state ^= state >> 7; state ^= state << 17;
        return state % m;
    };
    int cases = 0;
    const unsigned long long fixed[][5] = {
        {1, 1, 1, 1, 0}, {4, 199, 1024, 128, 0}, {32, 49917, 1024, 128, 0}, {8, 28767, 1024, 128, 0},
        {5, 7, 2, 1, 1}, {9, 274, 2, 1, 1}, {9, 274, 8, 2, 1}, {9, 1094, 32, 8, 1}, {3, 4096, 16, 16, 1},
        {130, 3, 1024, 128, 0}, {16, 16 * 1024, 1024, 128, 0}, {16, 16 * 1024 - 1, 1024, 128, 0},
        {2, 100000, 1048576, 1, 1}, {2, 100000, 1048576, 512, 1}};
    for (const auto& f : fixed) {
        const int rc = check((int)f[0], f[1], f[2], f[3], f[4] != 0);
        if (rc) { std::printf("FAIL rc=%d rows=%llu tiles=%llu super=%llu chunk=%llu\n", rc, f[0], f[1], f[2], f[3]); return 1; }
        ++cases;
    }
    for (int it = 0; it < 3000; ++it) {
        const int rows = 1 + (int)rnd(40);
        const unsigned long long tiles = 1 + rnd(it % 3 ? 3000 : 60000);
        const unsigned long long super = 1ull << rnd(12);
        const unsigned long long chunk = 1ull << rnd(10);
        const bool explicit_super = rnd(2) != 0;
        const int rc = check(rows, tiles, super, chunk, explicit_super);
        if (rc) { std::printf("FAIL rc=%d rows=%d tiles=%llu super=%llu chunk=%llu explicit=%d\n", rc, rows, tiles, super, chunk, (int)explicit_super); return 1; }
        ++cases;
    }
    TileOrder ord; unsigned long long grid;
    if (plan_tile_order(64, (1ull << 31), 512, 64, false, &ord, &grid)) { std::printf("FAIL: oversized grid accepted\n"); return 1; }
    if (plan_tile_order(1 << 12, (1ull << 20), 512, 64, false, &ord, &grid)) { std::printf("FAIL: oversized grid accepted\n"); return 1; }
    std::printf("tile order ok: %d cases\n", cases);
    return 0;
}
