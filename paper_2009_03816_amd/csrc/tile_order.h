// Workgroup order of the row x tile passes (update, broadcast), shared by the
// host planner and the device decoder; plain C++ so that the index arithmetic
// can also be checked exhaustively on the CPU.
//
// Workgroup wg runs on XCD wg & 7 (workgroups are dealt round-robin to the
// eight XCDs) and is the (wg >> 3)-th of that XCD.  A row's tiles are cut into
// chunks of consecutive tiles, every chunk size being dealt once to each of the
// eight XCDs: first as many rounds of the largest chunk (2^chunk_log2 tiles)
// as fit, then the rest by the binary digits of what is left - one round of
// each smaller power of two that still fits - and at last one tile each for
// the final fewer than eight.  All XCDs therefore get the same number of tiles
// of any row (up to that last one) in pieces as long as the row allows.  The
// tiles of one XCD, in address order, are its list u = 0 .. per_xcd-1.  The
// list is cut into super-chunks of 2^super_log2 entries (the last one may be
// shorter); within a super-chunk the order is row-major: all its tiles for
// row 0, then for row 1, ...  A gbest tile is therefore re-read by the same
// XCD, K times in a row, while its slice of gbest still sits in that XCD's L2,
// and the chip works on few rows at once.
#ifndef PSO_PS_TILE_ORDER_H
#define PSO_PS_TILE_ORDER_H

#if defined(__HIPCC__) || defined(__HIP__)
#define PSO_PS_HD __host__ __device__
#else
#define PSO_PS_HD
#endif

struct TileOrder {
    unsigned tiles;       // tiles per row (address-aligned tiles, first/last partial)
    unsigned per_xcd;     // list length per XCD
    unsigned super_log2;
    unsigned chunk_log2;
    unsigned full;        // number of full super-chunks
    unsigned last;        // entries in the last, shorter super-chunk (0 if none)
    unsigned main;        // list entries that lie in largest-size chunks
    unsigned rest;        // list entries in smaller chunks (< 2^chunk_log2)
};

inline unsigned tile_order_ceil_log2(unsigned long long t) {
    unsigned l = 0;
    while ((1ull << l) < t) ++l;
    return l;
}

// Order for `rows` rows of `tiles` tiles.  super_tiles / chunk_tiles: powers of
// two; chunk is clamped to super.  Returns false if the launch would exceed
// 2^31 - 1 workgroups; *grid gets the number of workgroups (a multiple of 8,
// at most 7 * rows of them without a tile).
inline bool plan_tile_order(int rows, unsigned long long tiles, unsigned long long super_tiles,
                            unsigned long long chunk_tiles, TileOrder* ord,
                            unsigned long long* grid) {
    unsigned long long super = super_tiles, chunk = chunk_tiles;
    if (super < 1) super = 1;
    if (chunk < 1) chunk = 1;
    if (chunk > super) chunk = super;
    const unsigned chunk_log2 = tile_order_ceil_log2(chunk);
    const unsigned long long groups = tiles >> 3;  // whole rounds of one tile per XCD
    const unsigned long long main = (groups >> chunk_log2) << chunk_log2;
    const unsigned long long rest = groups - main;
    const unsigned long long per_xcd = groups + ((tiles & 7ull) ? 1 : 0);
    if (rows < 1 || tiles >= (1ull << 31) ||
        per_xcd * 8ull * (unsigned long long)rows >= (1ull << 31))
        return false;
    ord->tiles = (unsigned)tiles;
    ord->per_xcd = (unsigned)per_xcd;
    ord->super_log2 = tile_order_ceil_log2(super);
    ord->chunk_log2 = chunk_log2;
    ord->full = (unsigned)(per_xcd >> ord->super_log2);
    ord->last = (unsigned)(per_xcd - ((unsigned long long)ord->full << ord->super_log2));
    ord->main = (unsigned)main;
    ord->rest = (unsigned)rest;
    *grid = per_xcd * 8ull * (unsigned long long)rows;
    return true;
}

// Which (row, tile) does workgroup `wg` of a launch (or of a segment's share
// of a launch, which starts at a multiple of 8) handle?  Returns false for a
// workgroup without a tile (the last list entry of some XCDs when the number
// of tiles is not a multiple of 8).
PSO_PS_HD inline bool decode_tile_order(const TileOrder& ord, unsigned rows, unsigned wg,
                                        unsigned* row, unsigned* tile) {
    const unsigned xcd = wg & 7u;
    const unsigned j = wg >> 3;
    const unsigned super = 1u << ord.super_log2;
    const unsigned full_span = (ord.full << ord.super_log2) * rows;
    unsigned i, u;
    if (j < full_span) {
        const unsigned q = j >> ord.super_log2;  // (super-chunk, row) pair
        const unsigned sc = q / rows;
        i = q - sc * rows;
        u = (sc << ord.super_log2) + (j & (super - 1u));
    } else {
        const unsigned r = j - full_span;
        i = r / ord.last;
        u = (ord.full << ord.super_log2) + (r - i * ord.last);
    }
    if (u < ord.main) {
        const unsigned chunk_mask = (1u << ord.chunk_log2) - 1u;
        *tile = ((((u >> ord.chunk_log2) << 3) + xcd) << ord.chunk_log2) + (u & chunk_mask);
    } else {
        const unsigned t = u - ord.main;
        if (t < ord.rest) {
            // t and rest agree above their highest differing bit l, where rest has
            // a 1 and t a 0: t lies in rest's chunk of 2^l entries, which follows
            // the chunks of rest's higher 1 bits.
            const unsigned l = 31u - (unsigned)__builtin_clz(t ^ ord.rest);
            const unsigned before = ord.rest & ~((2u << l) - 1u);
            *tile = ((ord.main + before) << 3) + (xcd << l) + (t & ((1u << l) - 1u));
        } else {
            *tile = ((ord.main + ord.rest) << 3) + xcd;
        }
    }
    *row = i;
    return *tile < ord.tiles && i < rows;
}

#endif  // PSO_PS_TILE_ORDER_H
