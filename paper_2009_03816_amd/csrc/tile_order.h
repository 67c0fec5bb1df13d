// Workgroup order of the row x tile passes (update, broadcast), shared by the
// host planner and the device decoder; plain C++ so that the index arithmetic
// can also be checked exhaustively on the CPU.
//
// Workgroup wg runs on XCD wg & 7 (workgroups are dealt round-robin to the
// eight XCDs) and is the (wg >> 3)-th of that XCD.  An XCD owns the tile
// chunks m with m % 8 == xcd (a chunk is 2^chunk_log2 consecutive tiles),
// listed as u = 0 .. per_xcd-1.  The list is cut into super-chunks of
// 2^super_log2 entries (the last one may be shorter); within a super-chunk the
// order is row-major: all its tiles for row 0, then for row 1, ...  A gbest
// tile is therefore re-read by the same XCD, K times in a row, while its slice
// of gbest still sits in that XCD's L2, and the chip works on few rows at once.
#ifndef PSO_PS_TILE_ORDER_H
#define PSO_PS_TILE_ORDER_H

#if defined(__HIPCC__) || defined(__HIP__)
#define PSO_PS_HD __host__ __device__
#else
#define PSO_PS_HD
#endif

struct TileOrder {
    unsigned tiles;       // tiles per row (address-aligned tiles, first/last partial)
    unsigned per_xcd;     // list length per XCD (multiple of the chunk size)
    unsigned super_log2;
    unsigned chunk_log2;
    unsigned full;        // number of full super-chunks
    unsigned last;        // entries in the last, shorter super-chunk (0 if none)
};

inline unsigned tile_order_ceil_log2(unsigned long long t) {
    unsigned l = 0;
    while ((1ull << l) < t) ++l;
    return l;
}

// Order for `rows` rows of `tiles` tiles.  super_tiles / chunk_tiles: powers of
// two; chunk is clamped to super.  Rows with fewer than 16 super-chunks of
// tiles take the plain row-major order (chunks of one tile, one super-chunk),
// which keeps all eight XCDs evenly loaded; an explicit_super is honoured.
// Returns false if the launch would exceed 2^31 - 1 workgroups; *grid gets the
// number of workgroups (a multiple of 8).
inline bool plan_tile_order(int rows, unsigned long long tiles, unsigned long long super_tiles,
                            unsigned long long chunk_tiles, bool explicit_super, TileOrder* ord,
                            unsigned long long* grid) {
    unsigned long long super = super_tiles, chunk = chunk_tiles;
    if (super < 1) super = 1;
    if (chunk < 1) chunk = 1;
    if (chunk > super) chunk = super;
    if (tiles < 16ull * super) chunk = 1;
    const unsigned long long per_xcd = (tiles + 8 * chunk - 1) / (8 * chunk) * chunk;
    if (!explicit_super && tiles < 16ull * super) super = 1ull << tile_order_ceil_log2(per_xcd);
    if (rows < 1 || tiles >= (1ull << 31) ||
        per_xcd * 8ull * (unsigned long long)rows >= (1ull << 31))
        return false;
    ord->tiles = (unsigned)tiles;
    ord->per_xcd = (unsigned)per_xcd;
    ord->super_log2 = tile_order_ceil_log2(super);
    ord->chunk_log2 = tile_order_ceil_log2(chunk);
    ord->full = (unsigned)(per_xcd >> ord->super_log2);
    ord->last = (unsigned)(per_xcd - ((unsigned long long)ord->full << ord->super_log2));
    *grid = per_xcd * 8ull * (unsigned long long)rows;
    return true;
}

// Which (row, tile) does workgroup `wg` of a launch (or of a segment's share
// of a launch, which starts at a multiple of 8) handle?  Returns false for the
// padding workgroups at the end of an XCD's list.
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
    const unsigned chunk_mask = (1u << ord.chunk_log2) - 1u;
    *tile = ((((u >> ord.chunk_log2) << 3) + xcd) << ord.chunk_log2) + (u & chunk_mask);
    *row = i;
    return *tile < ord.tiles && i < rows;
}

#endif  // PSO_PS_TILE_ORDER_H
