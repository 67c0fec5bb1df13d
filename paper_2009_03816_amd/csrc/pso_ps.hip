// PSO-PS synchronization step for gfx950 (MI355X): HIP kernels and the C ABI
// declared in include/pso_ps.h.
//
// Two kernels per stage of a large swarm.  Flat layout without history (pso_ps_sync):
//   select_move_best_kernel  g = argmin loss (Algorithm 3), improved_i = loss_i <
//                        pbest_loss_i (Algorithm 1), and the move of the best
//                        particle itself (Eq. (6), (7)), which stores gbest =
//                        x_g, Algorithm 3's return value, on its way.
//   update_others_kernel one streaming pass over the other K-1 rows of [K, D]:
//                        conditional pbest copy, Eq. (6) velocity and Eq. (7)
//                        position update; also brings pbest_loss up to date.
// With the historical gBest of Section II-C, for K separate row arrays and for
// ragged per-tensor segments (32 per launch) the split is the copy-based one:
//   select_gbest_kernel  selection, pbest_loss update and the copy gbest = x_g
//                        (TableSource / select_gbest_segments_kernel variants),
//   update_kernel        the pass over all K rows (update_rows_kernel,
//                        update_segments_kernel).
// A small swarm (K <= 16, K * D <= 1,000,000; more on request) takes the whole
// stage in ONE launch instead, because two dependent launches are what it
// pays for: whole_stage_kernel (and its ragged and row-pointer forms), one
// wavefront per particle, a workgroup barrier between everybody's read of x_g
// and its owner's write, and ticket counters that tell the last workgroup it
// may write pbest_loss.
// Parameter averaging, the synchronization the method replaces, is
// mean_kernel + broadcast_kernel.  fused_rows_kernel is the stage as a single
// pass (one workgroup owns a tile of columns for all K rows and keeps its piece
// of gbest on chip): the fewest bytes, but slower on this chip; kept selectable
// for measurement.
//
// The update pass is bound by HBM traffic, not by arithmetic: per particle
// parameter it must read x and v, write x and v, and either read pbest (not
// improved) or write it (improved; its old value is not needed because
// pbest - x is then exactly zero): 20 bytes.  gbest costs 8 bytes per column
// (written by the first kernel, first read by the second; 12 in the copy-based
// split, which reads x_g once more); the other reads of a gbest tile are served
// by the caches.
//
// Mapping of the update pass: one workgroup = one wavefront = one row
// (particle) x one tile of 256 consecutive floats, one 128-bit access per
// thread and array, i.e. the access pattern of a plain streaming copy.  What
// makes it reach copy-like bandwidth on this chip:
//   * tiles are aligned to the ADDRESS of the row's x (not to column 0), so
//     every wavefront touches whole 128-byte lines even when the row stride is
//     not a multiple of the tile (D = 25,557,032 gives rows 160 bytes off a
//     4 KiB boundary); the ragged head and tail of a row are handled
//     element-wise; v and pbest may sit at any 4-byte alignment and a row may
//     start at an odd flat index (three Philox calls per four columns then);
//   * x, v, pbest use non-temporal accesses (each byte is touched once); gbest
//     uses ordinary cached loads so that it stays resident;
//   * the workgroup order is XCD-aware: workgroup b runs on XCD b % 8, each XCD
//     is given runs of consecutive tiles (256 KiB) and walks a "super-chunk"
//     (2 MiB) of its tiles for row 0, 1, .., K-1 before moving on, so that a
//     gbest tile is re-read from the XCD's own L2 and the DRAM pages of few
//     rows are open at a time;
//   * the Philox rounds are placed between the loads and their first use;
//   * each launch reserves LDS it never touches, which caps a compute unit at
//     about 20 resident wavefronts of the 32 it could hold: HBM serves fewer,
//     steadier request streams better than the full house.
// Because gbest is written by the first kernel, which is also the only one that
// touches row g (or, in the copy-based split, copies it out before the update
// pass starts), the in-place update of row g cannot race with anything.
//
// Compile with -ffp-contract=off: the only fused operations are the two
// explicit fmaf of the velocity update.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

#include "pso_ps.h"
#include "tile_order.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
// Same, but only promised to be 4-byte aligned (the hardware takes unaligned
// multi-dword global accesses; the compiler picks the instruction).
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// Device scratch owned by a handle.
struct Selection {
    int g;                 // index of this stage's best particle
    int replaced;          // 1 if this stage's selection (re)wrote gbest
    float gbest_loss;      // historical gBest: the loss that goes with gbest after this stage
    int reserved;
    uint64_t improved[1];  // bit i of word i/64: particle i improved (really (K+63)/64 words)
};

// One dense block of columns: rows `ld` elements apart, `n` columns, the first
// of which has flat coordinate index d0.
struct ColumnBlock {
    float* x;
    float* v;
    float* pbest;
    float* gbest;
    long long ld;
    long long n;
    unsigned long long d0;
};

// Row-pointer mode: the K particles are K separate arrays (each worker's own
// weight tensor); one launch carries at most kTableRows of them by value.
constexpr int kTableRows = 64;
struct RowTable {
    float* x[kTableRows];
    float* v[kTableRows];
    float* pbest[kTableRows];
};

// Start of one particle's row in x, v and pbest.
struct RowPtrs {
    float* x;
    float* v;
    float* pbest;
};

struct MoveParams {
    float w, c1, c2;            // inertia (paper's m), effective accelerations
    uint32_t key0, key1;        // seed halves  -> Philox key
    uint32_t step_lo, step_hi;  // step halves  -> Philox counter words 2, 3
};

// Ragged mode: up to kTableSegs dense [K, n] segments share one launch.  Each
// keeps its own workgroup order; its workgroups start at first_wg (a multiple
// of 8, so that wg & 7 is still the XCD).  The update launch and the gbest
// copy launch carry a table each.
constexpr int kTableSegs = 32;
struct SegEntry {
    float* x;
    float* v;
    float* pbest;
    float* gbest;
    long long n;
    unsigned long long d0;
    TileOrder ord;
    unsigned first_wg;
    int vec;
};
struct SegTable {
    // The first workgroups again, side by side: the lookup scans them with
    // wide scalar loads instead of touching every entry.
    unsigned first_wg[kTableSegs];
    SegEntry seg[kTableSegs];
    int count;
};
struct CopyEntry {
    const float* x;  // [K, n], dense
    float* gbest;
    long long n;
    TileOrder ord;   // copy tiles of one row
    unsigned first_wg;
    int reserved;
};
struct CopyTable {
    unsigned first_wg[kTableSegs];
    CopyEntry seg[kTableSegs];
    int count;
};

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two
// 32x32->64 multiplications and a word permutation with key injection; the
// key is bumped by two Weyl constants after every round.
// ---------------------------------------------------------------------------
struct Words4 { uint32_t s0, s1, s2, s3; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const unsigned long long pa = (unsigned long long)c0 * 0xD2511F53ull;
        const unsigned long long pb = (unsigned long long)c2 * 0xCD9E8D57ull;
        const uint32_t t0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = t0;
        c2 = t2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words4{c0, c1, c2, c3};
}

// Top 24 bits of a random word as a float in [0, 1): both steps are exact.
__device__ __forceinline__ float unit_float(uint32_t word) {
    return __uint2float_rn(word >> 8) * 0x1.0p-24f;
}

// Eq. (6), (7) for one element.  p is the personal best after the pBest test.
__device__ __forceinline__ void move_element(float& x, float& v, float p, float gb,
                                             uint32_t word1, uint32_t word2,
                                             const MoveParams& m) {
    const float r1 = unit_float(word1);
    const float r2 = unit_float(word2);
    const float dp = p - x;
    const float dg = gb - x;
    const float a1 = m.c1 * r1;
    const float a2 = m.c2 * r2;
    float acc = m.w * v;
    acc = __fmaf_rn(a1, dp, acc);
    acc = __fmaf_rn(a2, dg, acc);
    v = acc;
    x = x + acc;
}

__device__ __forceinline__ bool is_improved(const Selection* __restrict__ sel, int i) {
    return (sel->improved[i >> 6] >> (i & 63)) & 1ull;
}

// One element of one row, element-wise accesses: ragged row ends and the
// generic path.  `col` is the column inside the block.
template <bool BEST = false>
__device__ __forceinline__ void move_single(const RowPtrs& r, float* __restrict__ gbest,
                                            unsigned long long d0, long long col, unsigned i,
                                            bool improved, const MoveParams& m) {
    const unsigned long long d = d0 + (unsigned long long)col;
    const Words4 words = philox4x32_10((uint32_t)(d >> 1), i, m.step_lo, m.step_hi, m.key0, m.key1);
    float xv = r.x[col];
    float vv = r.v[col];
    const float pv = improved ? xv : r.pbest[col];
    if (improved) r.pbest[col] = xv;
    if (BEST) gbest[col] = xv;  // this row is the best particle: gbest = its position before the move
    const float gb = BEST ? xv : gbest[col];
    const bool odd = d & 1ull;
    move_element(xv, vv, pv, gb, odd ? words.s2 : words.s0, odd ? words.s3 : words.s1, m);
    r.x[col] = xv;
    r.v[col] = vv;
}

// 128-bit store of four columns that will not be touched again in this
// launch, p 4-byte aligned: the nt bit (what a non-temporal store compiles to)
// plus sc1.  On the arithmetic-free 3 reads + 2 writes stream the pair is
// 0.8 % faster than nt alone and 8 % faster than sc1 alone; on the update pass
// 0.7 % (2.506 -> 2.489 ms per stage at K = 32, D = 25.6 M).  A write-only
// stream wants nt alone (the broadcast pass of the averaging baseline loses
// 14 % with sc1), and no builtin sets the pair, hence the instruction itself.
// The stores are the last memory operations of their wavefront, so that the
// compiler's count of outstanding operations is not off for any wait.
__device__ __forceinline__ void store_streaming(float* p, f32x4 q) {
    asm volatile("global_store_dwordx4 %0, %1, off nt sc1" : : "v"(p), "v"(q) : "memory");
}

// Columns c .. c+3 of row i with 128-bit accesses.  The address of x + c is
// 16-byte aligned (tiles are aligned to the row's address); v and pbest are
// read and written at the same columns and may sit at any 4-byte alignment,
// which the hardware accepts for multi-dword global accesses.  ODD: the flat
// index d0 + c of the first column is odd, so the four columns take the second
// half of one Philox call, all of the next and the first half of a third;
// otherwise they are two whole calls.  improved (uniform over the workgroup):
// Algorithm 1 replaced this particle's personal best by its position, so pbest
// is written instead of read.
template <bool ODD, bool BEST = false>
__device__ __forceinline__ void move_quad(const RowPtrs& r, float* __restrict__ gbest,
                                          unsigned long long d0, long long c, unsigned i,
                                          bool improved, const MoveParams& m) {
    float* xp = r.x + c;
    float* vp = r.v + c;
    float* pp = r.pbest + c;
    f32x4 x_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xp));
    f32x4 v_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(vp));
    f32x4 p_old = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!improved) p_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(pp));
    f32x4 gb = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!BEST) gb = *reinterpret_cast<const f32x4_a4*>(gbest + c);
    __builtin_amdgcn_sched_barrier(0);  // all loads are issued before anything below

    // The random words need nothing from memory: compute them while the loads
    // are in flight.  The empty asm ties the loaded values to the last random
    // words, which keeps the compiler from moving any use of them (and the
    // wait that goes with it) in front of the Philox rounds.
    const uint32_t pair = (uint32_t)((d0 + (unsigned long long)c) >> 1);
    const Words4 ra = philox4x32_10(pair, i, m.step_lo, m.step_hi, m.key0, m.key1);
    const Words4 rb = philox4x32_10(pair + 1u, i, m.step_lo, m.step_hi, m.key0, m.key1);
    Words4 rc = rb;
    if (ODD) rc = philox4x32_10(pair + 2u, i, m.step_lo, m.step_hi, m.key0, m.key1);
    asm volatile("" : "+v"(x_old), "+v"(v_old), "+v"(p_old), "+v"(gb)
                 : "v"(ra.s0), "v"(rb.s0), "v"(rc.s0));

    if (BEST) {
        // this row is the best particle: gbest = its position before the move
        // (Algorithm 3), written through the caches where the other rows'
        // pass will look for it
        gb = x_old;
        *reinterpret_cast<f32x4_a4*>(gbest + c) = x_old;
    }
    const f32x4 pv = improved ? x_old : p_old;
    float xs[4] = {x_old.x, x_old.y, x_old.z, x_old.w};
    float vs[4] = {v_old.x, v_old.y, v_old.z, v_old.w};
    if (!ODD) {
        move_element(xs[0], vs[0], pv.x, gb.x, ra.s0, ra.s1, m);
        move_element(xs[1], vs[1], pv.y, gb.y, ra.s2, ra.s3, m);
        move_element(xs[2], vs[2], pv.z, gb.z, rb.s0, rb.s1, m);
        move_element(xs[3], vs[3], pv.w, gb.w, rb.s2, rb.s3, m);
    } else {
        move_element(xs[0], vs[0], pv.x, gb.x, ra.s2, ra.s3, m);
        move_element(xs[1], vs[1], pv.y, gb.y, rb.s0, rb.s1, m);
        move_element(xs[2], vs[2], pv.z, gb.z, rb.s2, rb.s3, m);
        move_element(xs[3], vs[3], pv.w, gb.w, rc.s0, rc.s1, m);
    }
    store_streaming(xp, f32x4{xs[0], xs[1], xs[2], xs[3]});
    store_streaming(vp, f32x4{vs[0], vs[1], vs[2], vs[3]});
    if (improved) store_streaming(pp, x_old);
}

// One row x one tile.  VEC: tiles are aligned to the address of the row's x
// (any 4-byte aligned row qualifies) and whole groups of four columns go
// through move_quad; the ragged first and last columns of the row, and
// everything without VEC (tiles then start at column 0), are element-wise.
template <int BLOCK, bool VEC, bool BEST = false>
__device__ __forceinline__ void update_tile(const RowPtrs& r, float* __restrict__ gbest,
                                            long long n, unsigned long long d0, unsigned i,
                                            unsigned tile, bool improved, const MoveParams& m) {
    constexpr unsigned TILE = BLOCK * 4;
    long long phase = 0;
    if (VEC) phase = (long long)((reinterpret_cast<uintptr_t>(r.x) >> 2) & (TILE - 1u));
    const long long c = (long long)tile * TILE - phase + 4 * (long long)threadIdx.x;
    if (c + 4 <= 0 || c >= n) return;
    if (VEC && c >= 0 && c + 4 <= n) {
        // parity of the flat index of every quad of this row (TILE and 4 are even)
        const bool odd = ((unsigned long long)phase + d0) & 1ull;
        if (odd)
            move_quad<true, BEST>(r, gbest, d0, c, i, improved, m);
        else
            move_quad<false, BEST>(r, gbest, d0, c, i, improved, m);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long long col = c + e;
            if (col >= 0 && col < n) move_single<BEST>(r, gbest, d0, col, i, improved, m);
        }
    }
}

// Where the runs of consecutive tiles handed to an XCD (2^chunk_log2 tiles) start.
// origin 0: counted from the row's first tile.  Otherwise at absolute multiples
// of the run's size in memory: the decoded tile index then counts from the
// last such multiple (origin 2) or the last multiple of eight runs (origin 1)
// at or below the row's first tile, and indices before the row's first tile
// name no tile.  With origin 1 a run goes to XCD (address / run size) mod 8, so
// the same columns of different rows go to different XCDs; with origin 2 the
// first run of every row goes to XCD 0 and the columns of an XCD shift by less
// than one run from row to row.
template <int BLOCK>
__device__ __forceinline__ bool tile_from_origin(const float* row_x, const TileOrder& ord,
                                                 int origin, unsigned* tile) {
    if (origin == 0) return true;
    const unsigned cycle = (origin == 2 ? 1u : 8u) << ord.chunk_log2;
    const unsigned first =
        (unsigned)((reinterpret_cast<uintptr_t>(row_x) / (BLOCK * 16u)) & (uintptr_t)(cycle - 1u));
    if (*tile < first) return false;
    *tile -= first;
    return true;
}

// Update pass over stacked [K, ld] arrays.  gbest_loss (may be null) is the
// caller's historical-gBest loss: the selection kernel only reads it, and the
// value that belongs to this stage is stored here, after that kernel is done.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_kernel(ColumnBlock b, int K,
                                                       const Selection* __restrict__ sel,
                                                       MoveParams m, TileOrder ord,
                                                       float* gbest_loss, int origin) {
    if (gbest_loss && blockIdx.x == 0 && threadIdx.x == 0) *gbest_loss = sel->gbest_loss;
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)K, blockIdx.x, &i, &tile)) return;
    const long long row = (long long)i * b.ld;
    const RowPtrs r{b.x + row, b.v + row, b.pbest + row};
    if (VEC && !tile_from_origin<BLOCK>(r.x, ord, origin, &tile)) return;
    update_tile<BLOCK, VEC>(r, b.gbest, b.n, b.d0, i, tile, is_improved(sel, (int)i), m);
}

// Update pass over `rows` separate particle arrays, particles row0 .. row0+rows-1.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_rows_kernel(RowTable tab, const float* gbest,
                                                            long long n, int row0, int rows,
                                                            const Selection* __restrict__ sel,
                                                            MoveParams m, TileOrder ord,
                                                            float* gbest_loss) {
    if (gbest_loss && blockIdx.x == 0 && threadIdx.x == 0) *gbest_loss = sel->gbest_loss;
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)rows, blockIdx.x, &i, &tile)) return;
    const RowPtrs r{tab.x[i], tab.v[i], tab.pbest[i]};
    const unsigned particle = (unsigned)row0 + i;
    // (gbest is only read on this path)
    update_tile<BLOCK, VEC>(r, const_cast<float*>(gbest), n, 0ull, particle, tile,
                            is_improved(sel, (int)particle), m);
}

// The entry of the segment that workgroup `wg` belongs to (entries are sorted
// by their first workgroup).  The table is a kernel argument: the index is
// uniform, so the entry is fetched with scalar loads from the argument segment.
template <class Table>
__device__ __forceinline__ auto segment_of(const Table& tab, unsigned wg) -> decltype(tab.seg[0])& {
    int idx = 0;
#pragma unroll
    for (int s = 1; s < kTableSegs; ++s)
        if (s < tab.count && wg >= tab.first_wg[s]) idx = s;
    return tab.seg[idx];
}

// Update pass over up to kTableSegs ragged segments in one launch.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void update_segments_kernel(SegTable tab, int K,
                                                                const Selection* __restrict__ sel,
                                                                MoveParams m, float* gbest_loss) {
    if (gbest_loss && blockIdx.x == 0 && threadIdx.x == 0) *gbest_loss = sel->gbest_loss;
    const SegEntry& e = segment_of(tab, blockIdx.x);
    unsigned i, tile;
    if (!decode_tile_order(e.ord, (unsigned)K, blockIdx.x - e.first_wg, &i, &tile)) return;
    const long long row = (long long)i * e.n;  // segments are dense: row stride = n
    const RowPtrs r{e.x + row, e.v + row, e.pbest + row};
    const bool improved = is_improved(sel, (int)i);
    if (e.vec)
        update_tile<BLOCK, true>(r, e.gbest, e.n, e.d0, i, tile, improved, m);
    else
        update_tile<BLOCK, false>(r, e.gbest, e.n, e.d0, i, tile, improved, m);
}

// Where the gbest copy finds row g: in a stacked array, or among the rows that
// a row-pointer launch carries (null if g is not one of them).
struct StackedSource {
    const float* x;
    long long ld;
    __device__ const float* row(int g) const { return x + (long long)g * ld; }
};
struct TableSource {
    const float* x[kTableRows];
    int row0, rows;
    __device__ const float* row(int g) const {
        return (g >= row0 && g < row0 + rows) ? x[g - row0] : nullptr;
    }
};

// Lexicographic minimum of (loss, index) over the K losses with NaN read as
// +inf: the first argmin of Algorithm 3.  Every lane returns the same result.
// With `publisher` the calling wavefront also applies the strict "<" test of
// Algorithm 1 against pbest_loss and stores the improved mask.
__device__ __forceinline__ void wave_argmin(int K, const float* __restrict__ loss, float* pbest_loss,
                                            Selection* sel, bool publisher, float* best_out,
                                            int* g_out, bool store_pbest_loss = true) {
    const int lane = threadIdx.x & 63;
    const float inf = __builtin_huge_valf();
    float best = inf;
    int best_i = 0x7fffffff;
    for (int base = 0; base < K; base += 64) {
        const int i = base + lane;
        bool improved = false;
        if (i < K) {
            const float l = loss[i];
            const float key = (l != l) ? inf : l;
            if (best_i == 0x7fffffff || key < best) { best = key; best_i = i; }
            if (publisher) {
                improved = l < pbest_loss[i];  // false if either is NaN
                if (improved && store_pbest_loss) pbest_loss[i] = l;
            }
        }
        const unsigned long long mask = __ballot(improved);
        if (publisher && lane == 0) sel->improved[base >> 6] = mask;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float other = __shfl_xor(best, off, 64);
        const int other_i = __shfl_xor(best_i, off, 64);
        if (other < best || (other == best && other_i < best_i)) { best = other; best_i = other_i; }
    }
    *best_out = best;
    *g_out = best_i;
}

// This stage's selection, found by every wavefront on its own.  Wavefront 0 of
// workgroup 0 also does the pBest test and publishes g, the improved mask and
// whether gbest is replaced.  Nobody but that wavefront touches pbest_loss or
// the scratch, and nobody in this launch reads what it writes, so there is no
// ordering problem.  Without do_select, g and the replace flag are read from
// the scratch (later segment groups / row groups of the same stage).
//
// gbest_loss == null: gbest = x_g always (Algorithm 3).  Otherwise historical
// gBest: gbest = x_g only if this stage's lowest loss is strictly below
// *gbest_loss, which this launch only reads.
__device__ __forceinline__ void select_or_recall(int K, const float* __restrict__ loss,
                                                 float* pbest_loss, Selection* sel,
                                                 const float* gbest_loss, int do_select, int* g,
                                                 bool* replace, bool store_pbest_loss = true) {
    if (do_select) {
        const bool publisher = blockIdx.x == 0 && threadIdx.x < 64;
        float best;
        wave_argmin(K, loss, pbest_loss, sel, publisher, &best, g, store_pbest_loss);
        const float kept = gbest_loss ? *gbest_loss : 0.0f;
        *replace = gbest_loss ? (best < kept) : true;
        if (publisher && (threadIdx.x & 63) == 0) {
            sel->g = *g;
            sel->replaced = *replace ? 1 : 0;
            sel->gbest_loss = *replace ? best : kept;
        }
    } else {
        *g = sel->g;
        *replace = sel->replaced != 0;
    }
}

// gbest[0..n) = src[0..n) for one tile of kCopyTile columns: kCopyQuads
// 128-bit loads per thread, kCopyBlock quads apart, all issued before the
// first store.  A copy has no other work to hide its memory latency behind,
// so it wants many bytes in flight per thread and the whole compute unit
// (no occupancy cap); plain cached accesses measured faster than non-temporal
// ones here.  Tiles are aligned to the address of src.
constexpr int kCopyBlock = 256;
constexpr int kCopyQuads = 4;
constexpr unsigned kCopyTile = kCopyBlock * 4 * kCopyQuads;  // 4096 floats = 16 KiB

__device__ __forceinline__ void copy_tile(const float* __restrict__ src, float* __restrict__ gbest,
                                          long long n, unsigned tile) {
    const long long phase = (long long)((reinterpret_cast<uintptr_t>(src) >> 2) & (kCopyTile - 1u));
    const long long c0 = (long long)tile * kCopyTile - phase + 4 * (long long)threadIdx.x;
    f32x4 val[kCopyQuads];
    bool whole[kCopyQuads];
#pragma unroll
    for (int u = 0; u < kCopyQuads; ++u) {
        const long long c = c0 + (long long)u * (kCopyBlock * 4);
        whole[u] = c >= 0 && c + 4 <= n;
        if (whole[u]) val[u] = *reinterpret_cast<const f32x4*>(src + c);
    }
#pragma unroll
    for (int u = 0; u < kCopyQuads; ++u) {
        const long long c = c0 + (long long)u * (kCopyBlock * 4);
        if (whole[u]) {
            *reinterpret_cast<f32x4_a4*>(gbest + c) = val[u];
        } else {
            for (int e = 0; e < 4; ++e)
                if (c + e >= 0 && c + e < n) gbest[c + e] = src[c + e];
        }
    }
}

// Selection and gbest copy.  The copy takes its tiles in chunks dealt to the
// XCDs like those of the update pass (`ord` is an order for a single row of
// copy tiles), so that the XCD that will re-read a slice of gbest K times is,
// up to a tile at the chunk borders, the one that writes it.  In row-pointer
// mode a launch carries some of the rows by value and copies only if g is one
// of them.
template <class Source>
__global__ __launch_bounds__(kCopyBlock) void select_gbest_kernel(
    int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel, Source source,
    float* __restrict__ gbest, long long n, const float* gbest_loss, int do_select, TileOrder ord) {
    int g;
    bool replace;
    select_or_recall(K, loss, pbest_loss, sel, gbest_loss, do_select, &g, &replace);
    if (!replace) return;
    const float* src = source.row(g);
    if (!src) return;
    unsigned row, tile;
    if (!decode_tile_order(ord, 1u, blockIdx.x, &row, &tile)) return;
    copy_tile(src, gbest, n, tile);
}

// Selection (if do_select) and the gbest copies of up to kTableSegs segments.
__global__ __launch_bounds__(kCopyBlock) void select_gbest_segments_kernel(
    int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel, CopyTable tab,
    const float* gbest_loss, int do_select) {
    int g;
    bool replace;
    select_or_recall(K, loss, pbest_loss, sel, gbest_loss, do_select, &g, &replace);
    if (!replace) return;
    const CopyEntry& e = segment_of(tab, blockIdx.x);
    unsigned row, tile;
    if (!decode_tile_order(e.ord, 1u, blockIdx.x - e.first_wg, &row, &tile)) return;
    copy_tile(e.x + (long long)g * e.n, e.gbest, e.n, tile);
}

// ---------------------------------------------------------------------------
// The default split of the flat stage without history ("best first"): the first
// launch does the selection and moves the best particle itself, writing
// gbest = x_g from the values it has loaded anyway; the second launch moves
// the other K-1 particles.  Against selection + copy + K-row update this reads
// row g once less (4 D (5K+2) bytes instead of 4 D (5K+3)) and turns the copy
// into streaming work of the update pass's kind.  pbest_loss is left alone by
// the first launch (its workgroups need the old pbest_loss of the best
// particle while the publisher would be overwriting it) and brought up to date
// by workgroup 0 of the second.  (The same split was built for the ragged and
// the row-pointer layouts and measured no faster there - 2.56 against 2.51-2.55
// ms with 32 separate rows, 2.56 against 2.56 with 161 tensors - so those keep
// the copy-based split.)
// ---------------------------------------------------------------------------
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void select_move_best_kernel(
    ColumnBlock b, int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel,
    MoveParams m, TileOrder ord) {
    int g;
    bool replace;
    select_or_recall(K, loss, pbest_loss, sel, nullptr, 1, &g, &replace, false);
    unsigned row, tile;
    if (!decode_tile_order(ord, 1u, blockIdx.x, &row, &tile)) return;
    const long long off = (long long)g * b.ld;
    const RowPtrs r{b.x + off, b.v + off, b.pbest + off};
    const bool improved = loss[g] < pbest_loss[g];  // Algorithm 1's test, old pbest_loss
    update_tile<BLOCK, VEC, true>(r, b.gbest, b.n, b.d0, (unsigned)g, tile, improved, m);
}

// The other K-1 particles: the grid holds K-1 rows, and row index i of it is
// particle i, or i + 1 from the best particle on.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_others_kernel(
    ColumnBlock b, int K, const float* __restrict__ loss, float* pbest_loss,
    const Selection* __restrict__ sel, MoveParams m, TileOrder ord) {
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        // Algorithm 1: pbest_loss_i = loss_i for the particles that improved
        for (int i = (int)threadIdx.x; i < K; i += 64)
            if (is_improved(sel, i)) pbest_loss[i] = loss[i];
    }
    if (K < 2) return;  // the only particle is the best one
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)K - 1u, blockIdx.x, &i, &tile)) return;
    if (i >= (unsigned)sel->g) ++i;
    const long long row = (long long)i * b.ld;
    const RowPtrs r{b.x + row, b.v + row, b.pbest + row};
    update_tile<BLOCK, VEC>(r, b.gbest, b.n, b.d0, i, tile, is_improved(sel, (int)i), m);
}

// ---------------------------------------------------------------------------
// The single-pass variant: one workgroup owns a tile of columns for ALL K
// rows.  It reads its piece of x_g once, keeps it on chip (every thread needs
// only its own four columns of it, so registers serve; staging through LDS
// would add a round trip and share nothing), writes it to gbest, and walks the
// rows with the loads of the next P rows in flight while one row is computed.
// This moves the algorithmic minimum, 4 D (5K + 1) bytes, in one launch after
// a one-wavefront selection launch, and no workgroup reads what another
// writes.  Tiles are common to all rows, so only rows whose address is
// congruent to row 0's modulo 128 bytes get line-aligned accesses.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void select_only_kernel(int K, const float* __restrict__ loss,
                                                         float* pbest_loss, Selection* sel,
                                                         const float* gbest_loss) {
    int g;
    bool replace;
    select_or_recall(K, loss, pbest_loss, sel, gbest_loss, 1, &g, &replace);
}

// Columns c .. c+3 of a row of n columns: one 128-bit access where all four
// exist (whole), else element by element.
template <bool NT = true>
__device__ __forceinline__ f32x4 load_quad(const float* __restrict__ row, long long c, long long n,
                                           bool whole) {
    if (whole) {
        if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(row + c));
        return *reinterpret_cast<const f32x4_a4*>(row + c);
    }
    f32x4 r = {0.0f, 0.0f, 0.0f, 0.0f};
    if (c >= 0 && c < n) r.x = row[c];
    if (c + 1 >= 0 && c + 1 < n) r.y = row[c + 1];
    if (c + 2 >= 0 && c + 2 < n) r.z = row[c + 2];
    if (c + 3 >= 0 && c + 3 < n) r.w = row[c + 3];
    return r;
}

template <bool NT = true>
__device__ __forceinline__ void store_quad(float* __restrict__ row, long long c, long long n,
                                           bool whole, f32x4 q) {
    if (whole) {
        if (NT) __builtin_nontemporal_store(q, reinterpret_cast<f32x4_a4*>(row + c));
        else *reinterpret_cast<f32x4_a4*>(row + c) = q;
        return;
    }
    if (c >= 0 && c < n) row[c] = q.x;
    if (c + 1 >= 0 && c + 1 < n) row[c + 1] = q.y;
    if (c + 2 >= 0 && c + 2 < n) row[c + 2] = q.z;
    if (c + 3 >= 0 && c + 3 < n) row[c + 3] = q.w;
}

// The random words of four consecutive columns of particle i.  `pair` is the
// random-number pair index (flat coordinate index / 2) of the first column;
// ODD: that column is the second of its pair, so the four columns take words
// from three Philox calls instead of two.
struct RandomFour {
    Words4 a, b, c;
};
template <bool ODD>
__device__ __forceinline__ RandomFour draw_four(uint32_t pair, uint32_t i, const MoveParams& m) {
    RandomFour r;
    r.a = philox4x32_10(pair, i, m.step_lo, m.step_hi, m.key0, m.key1);
    r.b = philox4x32_10(pair + 1u, i, m.step_lo, m.step_hi, m.key0, m.key1);
    r.c = r.b;
    if (ODD) r.c = philox4x32_10(pair + 2u, i, m.step_lo, m.step_hi, m.key0, m.key1);
    return r;
}

// Eq. (6), (7) for those four columns held in registers: xq, vq are replaced
// by the moved values.
template <bool ODD>
__device__ __forceinline__ void move_four(f32x4& xq, f32x4& vq, f32x4 pv, f32x4 gb,
                                          const RandomFour& r, const MoveParams& m) {
    float xs[4] = {xq.x, xq.y, xq.z, xq.w};
    float vs[4] = {vq.x, vq.y, vq.z, vq.w};
    if (!ODD) {
        move_element(xs[0], vs[0], pv.x, gb.x, r.a.s0, r.a.s1, m);
        move_element(xs[1], vs[1], pv.y, gb.y, r.a.s2, r.a.s3, m);
        move_element(xs[2], vs[2], pv.z, gb.z, r.b.s0, r.b.s1, m);
        move_element(xs[3], vs[3], pv.w, gb.w, r.b.s2, r.b.s3, m);
    } else {
        move_element(xs[0], vs[0], pv.x, gb.x, r.a.s2, r.a.s3, m);
        move_element(xs[1], vs[1], pv.y, gb.y, r.b.s0, r.b.s1, m);
        move_element(xs[2], vs[2], pv.z, gb.z, r.b.s2, r.b.s3, m);
        move_element(xs[3], vs[3], pv.w, gb.w, r.c.s0, r.c.s1, m);
    }
    xq = f32x4{xs[0], xs[1], xs[2], xs[3]};
    vq = f32x4{vs[0], vs[1], vs[2], vs[3]};
}

template <int BLOCK, int P, bool ODD>
__device__ __forceinline__ void fused_tile(const ColumnBlock& b, int K,
                                           const Selection* __restrict__ sel, const MoveParams& m,
                                           long long c) {
    const bool whole = c >= 0 && c + 4 <= b.n;
    const int g = sel->g;
    const bool replaced = sel->replaced != 0;

    // gbest for these columns: x_g as it is before anybody moves (Algorithm 3),
    // or the kept historical gbest.
    f32x4 gb;
    if (replaced) {
        gb = load_quad(b.x + (long long)g * b.ld, c, b.n, whole);
        store_quad(b.gbest, c, b.n, whole, gb);
    } else {
        gb = load_quad(b.gbest, c, b.n, whole);
    }

    // Flat index of column c; may be negative in the first tile, whose columns
    // below 0 do not exist (arithmetic shift keeps the pairs of the others right).
    const long long d = (long long)b.d0 + c;
    const uint32_t pair = (uint32_t)(d >> 1);

    f32x4 xq[P], vq[P], pq[P];
    auto improved_bit = [&](int i) { return (sel->improved[i >> 6] >> (i & 63)) & 1ull; };
    auto fetch = [&](int i, f32x4& xo, f32x4& vo, f32x4& po) {
        const long long row = (long long)i * b.ld;
        xo = (replaced && i == g) ? gb : load_quad(b.x + row, c, b.n, whole);
        vo = load_quad(b.v + row, c, b.n, whole);
        po = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (!improved_bit(i)) po = load_quad(b.pbest + row, c, b.n, whole);
    };
#pragma unroll
    for (int s = 0; s < P; ++s)
        if (s < K) fetch(s, xq[s], vq[s], pq[s]);

    for (int base = 0; base < K; base += P) {
#pragma unroll
        for (int s = 0; s < P; ++s) {
            const int i = base + s;
            if (i >= K) break;
            const bool improved = improved_bit(i);
            const f32x4 x_old = xq[s];
            f32x4 x_new = x_old, v_new = vq[s];
            move_four<ODD>(x_new, v_new, improved ? x_old : pq[s], gb, draw_four<ODD>(pair, (uint32_t)i, m), m);
            const long long row = (long long)i * b.ld;
            store_quad(b.x + row, c, b.n, whole, x_new);
            store_quad(b.v + row, c, b.n, whole, v_new);
            if (improved) store_quad(b.pbest + row, c, b.n, whole, x_old);
            if (i + P < K) fetch(i + P, xq[s], vq[s], pq[s]);
        }
    }
}

template <int BLOCK, int P>
__global__ __launch_bounds__(BLOCK) void fused_rows_kernel(ColumnBlock b, int K,
                                                           const Selection* __restrict__ sel,
                                                           MoveParams m, TileOrder ord,
                                                           float* gbest_loss) {
    if (gbest_loss && blockIdx.x == 0 && threadIdx.x == 0) *gbest_loss = sel->gbest_loss;
    unsigned row, tile;
    if (!decode_tile_order(ord, 1u, blockIdx.x, &row, &tile)) return;
    constexpr unsigned TILE = BLOCK * 4;
    // tiles are aligned to the address of row 0
    const long long phase = (long long)((reinterpret_cast<uintptr_t>(b.x) >> 2) & (TILE - 1u));
    const long long c = (long long)tile * TILE - phase + 4 * (long long)threadIdx.x;
    if (c + 4 <= 0 || c >= b.n) return;
    if (((unsigned long long)phase + b.d0) & 1ull)
        fused_tile<BLOCK, P, true>(b, K, sel, m, c);
    else
        fused_tile<BLOCK, P, false>(b, K, sel, m, c);
}

// ---------------------------------------------------------------------------
// The whole stage in ONE launch, for swarms so small that a stage is bound by
// its launches (two dependent launches cost about 4 us each) and not by
// memory.  A workgroup owns a tile of 256 columns for all K particles and has
// one wavefront per particle (up to kStageWaves of them; with more particles
// a wavefront takes every W-th).  Two things in a stage are read by many and
// overwritten in place:
//  * x_g, which is gbest for everybody (Algorithm 3) and is moved by the
//    wavefront that owns particle g.  Every wavefront loads its four columns
//    of x_g before a workgroup barrier, the owner stores after it; only this
//    workgroup touches these columns.
//  * pbest_loss (and the historical gbest loss), which every workgroup reads
//    for Algorithm 1's "<" test and which must end up updated.  Every
//    workgroup takes a ticket after the barrier, i.e. after all its reads have
//    returned; the workgroup that draws the last ticket knows that nobody will
//    read them again and writes them, together with the selection record.
//    Tickets are same-address atomics, which cost about 10 ns each here, so
//    they are spread over kTicketShards counters (256 bytes apart) whose last
//    drawers then draw from a top counter.  The last workgroup of all puts the
//    counters back to zero for the next stage.
// Every workgroup reaches the barrier and the ticket: no early exit.
// ---------------------------------------------------------------------------
constexpr int kStageWaves = 16;         // wavefronts per workgroup at most
constexpr int kStageMaxK = PSO_PS_SINGLE_LAUNCH_MAX_K;   // one wavefront holds the whole improved mask
static_assert(kStageMaxK <= 64, "the improved mask of the single-launch stage is one ballot");
static_assert(kStageMaxK <= kTableRows, "a row-pointer launch carries every particle of the single-launch stage");
constexpr unsigned kStageTile = 256;    // columns per workgroup: one 128-bit group per lane
constexpr bool kStageNT = false;         // cached accesses: these swarms live in L2 / Infinity Cache
constexpr unsigned kTicketShards = 16;
constexpr unsigned kTicketStride = 64;  // counters are 64 unsigned = 256 bytes apart
constexpr size_t kTicketBytes = (size_t)(kTicketShards + 1) * kTicketStride * sizeof(unsigned);

// `rows` says where particle i's x, v and pbest start (stacked with a stride,
// or K separate arrays); `b` carries gbest, the number of columns and d0.
struct StackedRows {
    float* x;
    float* v;
    float* pbest;
    long long ld;
    __device__ RowPtrs row(int i) const {
        const long long off = (long long)i * ld;
        return RowPtrs{x + off, v + off, pbest + off};
    }
};
struct TableRows {
    RowTable tab;
    __device__ RowPtrs row(int i) const { return RowPtrs{tab.x[i], tab.v[i], tab.pbest[i]}; }
};

// One tile of the single-launch stage.  Everything before the barrier is
// ordered for latency, which is all a small swarm pays: the losses are
// requested first, then this wavefront's first
// particle (pbest too, whether or not it turns out to be needed: waiting for
// the "<" test would cost a round trip); the selection runs when the losses
// are there; x_g can only be requested then; the random words are computed
// while all of that is in flight.
template <bool ODD, class Rows>
__device__ __forceinline__ void whole_stage_tile(const Rows& rows, const ColumnBlock& b, int K,
                                                 const float* __restrict__ loss, float* pbest_loss,
                                                 Selection* sel, const MoveParams& m,
                                                 float* gbest_loss, long long c, unsigned* tickets) {
    const int lane = (int)(threadIdx.x & 63);
    const int w = (int)(threadIdx.x >> 6), W = (int)(blockDim.x >> 6);
    const float inf = __builtin_huge_valf();
    float l = inf, pl = 0.0f;
    if (lane < K) { l = loss[lane]; pl = pbest_loss[lane]; }
    const float kept = gbest_loss ? *gbest_loss : 0.0f;

    const bool whole = c >= 0 && c + 4 <= b.n;
    int i = w;   // W <= K: every wavefront has a first particle
    RowPtrs r = rows.row(i);
    f32x4 xq = load_quad<kStageNT>(r.x, c, b.n, whole);
    f32x4 vq = load_quad<kStageNT>(r.v, c, b.n, whole);
    f32x4 pq = load_quad<kStageNT>(r.pbest, c, b.n, whole);

    // Algorithm 3: first argmin with NaN read as +inf (every lane gets the
    // result); Algorithm 1: the strict "<" test, false if either side is NaN
    float best = (l != l) ? inf : l;
    int g = lane < K ? lane : 0x7fffffff;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float other = __shfl_xor(best, off, 64);
        const int other_i = __shfl_xor(g, off, 64);
        if (other < best || (other == best && other_i < g)) { best = other; g = other_i; }
    }
    const unsigned long long improved_mask = __ballot(lane < K && l < pl);
    const bool replace = gbest_loss ? (best < kept) : true;

    // gbest for these columns: x_g before anybody moves, or the kept historical gbest
    const f32x4 gb =
        load_quad<kStageNT>(replace ? rows.row(g).x : b.gbest, c, b.n, whole);
    const long long d = (long long)b.d0 + c;   // may be negative in the first tile: see fused_tile
    const uint32_t pair = (uint32_t)(d >> 1);
    RandomFour rnd = draw_four<ODD>(pair, (uint32_t)i, m);
    asm volatile("" : "+v"(xq), "+v"(vq), "+v"(pq) : "v"(rnd.a.s0), "v"(rnd.b.s0), "v"(rnd.c.s0));
    __syncthreads();   // every load above has returned, in every wavefront

    // (drawing the ticket earlier, under a barrier of its own right after the
    // losses, measured no faster)
    unsigned ticket = 0;
    if (threadIdx.x == 0)
        ticket = atomicAdd(tickets + kTicketStride * (1u + blockIdx.x % kTicketShards), 1u);
    if (w == 0 && replace) store_quad<kStageNT>(b.gbest, c, b.n, whole, gb);
    for (;;) {
        const bool improved = (improved_mask >> i) & 1ull;
        const f32x4 x_old = xq;
        move_four<ODD>(xq, vq, improved ? x_old : pq, gb, rnd, m);
        store_quad<kStageNT>(r.x, c, b.n, whole, xq);
        store_quad<kStageNT>(r.v, c, b.n, whole, vq);
        if (improved) store_quad<kStageNT>(r.pbest, c, b.n, whole, x_old);
        i += W;
        if (i >= K) break;
        r = rows.row(i);
        xq = load_quad<kStageNT>(r.x, c, b.n, whole);
        vq = load_quad<kStageNT>(r.v, c, b.n, whole);
        if (!((improved_mask >> i) & 1ull)) pq = load_quad<kStageNT>(r.pbest, c, b.n, whole);
        rnd = draw_four<ODD>(pair, (uint32_t)i, m);
    }

    if (threadIdx.x != 0) return;
    const unsigned shard = blockIdx.x % kTicketShards;
    const unsigned in_shard = (gridDim.x - shard + kTicketShards - 1u) / kTicketShards;
    if (ticket != in_shard - 1u) return;
    const unsigned shards = gridDim.x < kTicketShards ? gridDim.x : kTicketShards;
    if (atomicAdd(tickets, 1u) != shards - 1u) return;
    // Last ticket of the last shard: every workgroup has its copy of the
    // losses.  Algorithm 1: pbest_loss_i = loss_i for the particles that improved.
    for (int k = 0; k < K; ++k)
        if ((improved_mask >> k) & 1ull) pbest_loss[k] = loss[k];
    sel->g = g;
    sel->replaced = replace ? 1 : 0;
    sel->gbest_loss = replace ? best : kept;
    sel->improved[0] = improved_mask;
    if (gbest_loss) *gbest_loss = replace ? best : kept;
    for (unsigned q = 0; q <= kTicketShards; ++q)
        __hip_atomic_store(tickets + kTicketStride * q, 0u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(64 * kStageWaves) void whole_stage_kernel(
    ColumnBlock b, int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel,
    MoveParams m, float* gbest_loss, unsigned* tickets) {
    // tiles are aligned to the address of row 0
    const long long phase = (long long)((reinterpret_cast<uintptr_t>(b.x) >> 2) & (kStageTile - 1u));
    const long long c =
        (long long)blockIdx.x * kStageTile - phase + 4 * (long long)(threadIdx.x & 63);
    const StackedRows rows{b.x, b.v, b.pbest, b.ld};
    if (((unsigned long long)phase + b.d0) & 1ull)
        whole_stage_tile<true>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
    else
        whole_stage_tile<false>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
}

// The same for the ragged layout, when all its segments fit one launch: a
// workgroup owns 256 columns of one segment.  The tickets are drawn over the
// whole launch, so pbest_loss is written when every segment's workgroups have
// read it.
struct StageEntry {
    float* x;
    float* v;
    float* pbest;
    float* gbest;
    long long n;
    unsigned long long d0;
    unsigned first_wg;
    unsigned reserved;
};
struct StageTable {
    unsigned first_wg[kTableSegs];
    StageEntry seg[kTableSegs];
    int count;
};

__global__ __launch_bounds__(64 * kStageWaves) void whole_stage_segments_kernel(
    StageTable tab, int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel,
    MoveParams m, float* gbest_loss, unsigned* tickets) {
    const StageEntry& e = segment_of(tab, blockIdx.x);
    const ColumnBlock b{e.x, e.v, e.pbest, e.gbest, e.n, e.n, e.d0};   // dense: row stride = n
    const long long phase = (long long)((reinterpret_cast<uintptr_t>(b.x) >> 2) & (kStageTile - 1u));
    const long long c = (long long)(blockIdx.x - e.first_wg) * kStageTile - phase +
                        4 * (long long)(threadIdx.x & 63);
    const StackedRows rows{b.x, b.v, b.pbest, b.ld};
    if (((unsigned long long)phase + b.d0) & 1ull)
        whole_stage_tile<true>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
    else
        whole_stage_tile<false>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
}

// The same for K <= kTableRows separate particle arrays (row-pointer mode).
__global__ __launch_bounds__(64 * kStageWaves) void whole_stage_rows_kernel(
    TableRows rows, float* gbest, long long n, int K, const float* __restrict__ loss,
    float* pbest_loss, Selection* sel, MoveParams m, float* gbest_loss, unsigned* tickets) {
    const ColumnBlock b{nullptr, nullptr, nullptr, gbest, 0, n, 0ull};   // gbest, n, d0 are used
    // tiles are aligned to the address of particle 0's x
    const long long phase =
        (long long)((reinterpret_cast<uintptr_t>(rows.tab.x[0]) >> 2) & (kStageTile - 1u));
    const long long c =
        (long long)blockIdx.x * kStageTile - phase + 4 * (long long)(threadIdx.x & 63);
    if ((unsigned long long)phase & 1ull)
        whole_stage_tile<true>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
    else
        whole_stage_tile<false>(rows, b, K, loss, pbest_loss, sel, m, gbest_loss, c, tickets);
}

// Parameter averaging (Section II-B, step 5) on the stacked layout, first half:
// one thread owns four columns, sums the K rows in order and divides by K.
// Reading K rows at one column is tolerant of the rows' different alignments.
// Column tiles are dealt to the XCDs in chunks like those of the update pass
// (`ord` is an order for a single row of column tiles).
constexpr int kMeanBlock = 256;
constexpr int kMeanQuads = 1;  // 128-bit groups per thread and row, kMeanBlock groups apart
                               // (2, 4 and 8 measured no faster: 1.06, 1.08, 1.05 against 1.05 ms)
constexpr unsigned kMeanTile = kMeanBlock * 4 * kMeanQuads;

__global__ __launch_bounds__(kMeanBlock) void mean_kernel(const float* __restrict__ x,
                                                          float* __restrict__ mean, long long ld,
                                                          long long n, int K, TileOrder ord) {
    unsigned row, tile;
    if (!decode_tile_order(ord, 1u, blockIdx.x, &row, &tile)) return;
    const long long c0 = (long long)tile * kMeanTile + 4 * (long long)threadIdx.x;
    const float kf = (float)K;
    f32x4 sum[kMeanQuads];
    bool whole[kMeanQuads];
#pragma unroll
    for (int u = 0; u < kMeanQuads; ++u) {
        const long long c = c0 + (long long)u * (kMeanBlock * 4);
        whole[u] = c + 4 <= n;
        if (whole[u]) sum[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(x + c));
    }
    // (issuing several rows' loads before the first add changes nothing: the
    // pass is bound by the K rows it has open at once, not by latency)
    for (int k = 1; k < K; ++k) {
#pragma unroll
        for (int u = 0; u < kMeanQuads; ++u) {
            const long long c = c0 + (long long)u * (kMeanBlock * 4);
            if (whole[u])
                sum[u] = sum[u] + __builtin_nontemporal_load(
                                      reinterpret_cast<const f32x4_a4*>(x + (long long)k * ld + c));
        }
    }
#pragma unroll
    for (int u = 0; u < kMeanQuads; ++u) {
        const long long c = c0 + (long long)u * (kMeanBlock * 4);
        if (whole[u]) {
            *reinterpret_cast<f32x4_a4*>(mean + c) =
                f32x4{sum[u].x / kf, sum[u].y / kf, sum[u].z / kf, sum[u].w / kf};
        } else {
            for (long long e = c; e < n && e < c + 4; ++e) {   // the ragged last columns
                float s1 = x[e];
                for (int k = 1; k < K; ++k) s1 = s1 + x[(long long)k * ld + e];
                mean[e] = s1 / kf;
            }
        }
    }
}

// Second half: every row becomes the mean.  Writes want whole 128-byte lines,
// so this is one row x one address-aligned tile per workgroup, in the same
// order as the update pass; the mean tile is re-read through the caches.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void broadcast_kernel(float* x, const float* __restrict__ mean,
                                                          long long ld, long long n, int K,
                                                          TileOrder ord) {
    constexpr unsigned TILE = BLOCK * 4;
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)K, blockIdx.x, &i, &tile)) return;
    float* row = x + (long long)i * ld;
    long long phase = 0;
    if (VEC) phase = (long long)((reinterpret_cast<uintptr_t>(row) >> 2) & (TILE - 1u));
    const long long c = (long long)tile * TILE - phase + 4 * (long long)threadIdx.x;
    if (c + 4 <= 0 || c >= n) return;
    if (VEC && c >= 0 && c + 4 <= n) {
        const f32x4 m = *reinterpret_cast<const f32x4_a4*>(mean + c);
        __builtin_nontemporal_store(m, reinterpret_cast<f32x4*>(row + c));
    } else {
        for (int e = 0; e < 4; ++e)
            if (c + e >= 0 && c + e < n) row[c + e] = mean[c + e];
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
bool aligned_to(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

struct pso_ps_ctx {
    int K;
    int64_t D;
    int64_t ld;
    std::vector<int64_t> seg_sizes;  // empty: one flat block
    // Work lists of pso_ps_sync_segments, sized at create so that a stage does
    // not touch the host heap.
    std::vector<ColumnBlock> seg_blocks;
    std::vector<SegTable> seg_tables;
    std::vector<CopyTable> seg_copy_tables;
    std::vector<unsigned> seg_update_wgs, seg_copy_wgs;
    int device;
    Selection* sel;        // device
    size_t sel_bytes;
    int mask_words;
    hipStream_t last_stream;
    bool have_selection;
    int block_threads;     // 0 = default
    int super_tiles;       // 0 = default; else a power of two
    int chunk_tiles;       // 0 = default; else a power of two <= super_tiles
    int wgs_per_cu;        // 0 = default; else cap on resident update workgroups per compute unit
    bool force_generic;
    int fused_rows;        // 0: selection/copy kernel + update kernel; P > 0: single pass, P rows in flight
    int chunk_origin;      // 0, 1, 2: see tile_from_origin
    bool best_first;       // flat stage without history as select_move_best_kernel + update_others_kernel
    int single_launch;     // whole_stage_kernel: -1 where it measured faster (small swarms), 0 never, 1 wherever it can run
    unsigned* tickets;     // device: the ticket counters of whole_stage_kernel, zero between stages
    bool eight_xcds;       // 256 compute units: the chip is driven as one device of 8 XCDs
    int last_hip_error;
};

// Selection scratch of pso_ps_sync_static, which must not allocate: a
// file-scope device array instead of a handle's hipMalloc.  Every GPU holds its
// own copy at its own address; host code never uses the name as an address,
// only the pointer that hipGetSymbolAddress returns for the current device.
constexpr int kStaticMaxK = PSO_PS_STATIC_MAX_K;
constexpr size_t kStaticSelectionBytes =
    (sizeof(Selection) + (size_t)((kStaticMaxK + 63) / 64 - 1) * sizeof(uint64_t) + 255) / 256 * 256;
// the selection record, then the ticket counters of whole_stage_kernel, which
// start at zero (static storage) and are put back to zero by every stage
constexpr size_t kStaticScratchBytes = kStaticSelectionBytes + kTicketBytes;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Defaults from sweeps on MI355X with K = 32, D = 25.6 M: one wavefront per
// workgroup (tile = 1 KiB; 64 threads beat 128 by just under 1 %, 256 lose 3 %),
constexpr int kDefaultBlock = 64;
constexpr int kRowsBlock = 128;                      // update_rows_kernel
constexpr unsigned kDefaultSuperBytes = 2u << 20;    // gbest footprint per XCD, in its 4 MiB L2
constexpr unsigned kDefaultChunkBytes = 256u << 10;  // consecutive addresses handed to one XCD
constexpr int kDefaultWavesPerCu = 20;               // resident wavefronts per compute unit (of 32)

// Makes the handle's device current for the lifetime of the object.
struct DeviceScope {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceScope(int device) {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != device) {
            err = hipSetDevice(device);
            switched = (err == hipSuccess);
        }
    }
    ~DeviceScope() {
        if (switched) (void)hipSetDevice(prev);
    }
};

int hip_fail(pso_ps_ctx* h, hipError_t e) {
    if (h) h->last_hip_error = (int)e;
    return PSO_PS_EHIP;
}

int check_arrays(const float* x, const float* v, const float* pbest, const float* gbest) {
    if (!x || !v || !pbest || !gbest) return PSO_PS_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(v, 4) || !aligned_to(pbest, 4) || !aligned_to(gbest, 4))
        return PSO_PS_EALIGN;
    return PSO_PS_OK;
}

int check_block(const ColumnBlock& b) {
    const int rc = check_arrays(b.x, b.v, b.pbest, b.gbest);
    if (rc != PSO_PS_OK) return rc;
    if (b.n < 0 || b.ld < b.n) return PSO_PS_EINVAL;
    // Philox counter word 0 holds the pair index: flat indices must stay below 2^33.
    if (b.d0 + (unsigned long long)b.n > (1ull << 33)) return PSO_PS_EINVAL;
    return PSO_PS_OK;
}

// Every 4-byte aligned row can take the 128-bit path (tiles are aligned to the
// row's own address, v and pbest may be off by any multiple of 4 bytes, the
// Philox parity of a row is found on the device); the element-wise path is
// only taken on request.
bool vector_path(const pso_ps_ctx* h) { return !h->force_generic; }

// Workgroup order for `rows` rows of `tiles` tiles of `tile` floats, with the
// handle's launch settings.  Returns false if the grid would be too large.
bool plan_order(const pso_ps_ctx* h, int rows, unsigned long long tiles, unsigned tile,
                TileOrder* ord, unsigned long long* grid) {
    const unsigned long long super = h->super_tiles ? (unsigned long long)h->super_tiles
                                                    : kDefaultSuperBytes / (tile * 4u);
    const unsigned long long chunk = h->chunk_tiles ? (unsigned long long)h->chunk_tiles
                                                    : kDefaultChunkBytes / (tile * 4u);
    // The chunked order is tuned for workgroups dealt round-robin to 8 XCDs.  On
    // a partitioned device (fewer compute units behind one device) fall back to
    // plain row-major order unless the caller has chosen a shape.
    if (!h->eight_xcds && !h->super_tiles && !h->chunk_tiles)
        return plan_tile_order(rows, tiles, 1ull << 30, 1, ord, grid);
    return plan_tile_order(rows, tiles, super, chunk, ord, grid);
}

// Tile indices that name no tile when runs start at absolute addresses: the
// row that starts furthest into its run (or its eight runs) needs that many more.
unsigned long long origin_slack(const pso_ps_ctx* h, unsigned tile) {
    if (h->chunk_origin == 0 || !h->eight_xcds) return 0;
    unsigned long long super = h->super_tiles ? (unsigned long long)h->super_tiles
                                              : kDefaultSuperBytes / (tile * 4u);
    unsigned long long chunk = h->chunk_tiles ? (unsigned long long)h->chunk_tiles
                                              : kDefaultChunkBytes / (tile * 4u);
    if (chunk > super) chunk = super;
    if (chunk < 1) chunk = 1;
    const unsigned long long run = 1ull << tile_order_ceil_log2(chunk);
    return (h->chunk_origin == 2 ? run : 8ull * run) - 1ull;
}

// Dynamic LDS requested for a streaming launch.  The kernels never touch it:
// the reservation only caps how many workgroups a compute unit holds at once
// (160 KiB of LDS per compute unit), which is what the memory system likes.
unsigned occupancy_cap_lds(const pso_ps_ctx* h, int block) {
    int wgs = h->wgs_per_cu;
    if (wgs == 0) {  // default: about kDefaultWavesPerCu wavefronts (sweep: 16-20 of 32 is best)
        wgs = (kDefaultWavesPerCu * 64 + block - 1) / block;
        if (wgs < 3) wgs = 3;
    }
    if (wgs >= 64) return 0;                              // no cap
    const unsigned bytes = (160u * 1024u / (unsigned)wgs) & ~511u;
    return bytes > 64u * 1024u ? 64u * 1024u : bytes;     // default dynamic-LDS limit of a kernel
}

// Tiles per row when tiles are aligned to each row's address: enough for the
// row that starts furthest into a tile.
template <class RowX>
unsigned long long tiles_per_row(int rows, long long n, bool aligned_to_rows, unsigned tile,
                                 RowX row_x) {
    unsigned long long max_phase = 0;
    if (aligned_to_rows) {
        for (int i = 0; i < rows; ++i) {
            const unsigned long long a = (reinterpret_cast<uintptr_t>(row_x(i)) >> 2) & (tile - 1u);
            if (a > max_phase) max_phase = a;
        }
    }
    return (max_phase + (unsigned long long)n + tile - 1) / tile;
}

int block_of(const pso_ps_ctx* h) { return h->block_threads ? h->block_threads : kDefaultBlock; }
// Row-pointer launches fetch their row's three pointers from the kernel
// arguments first; twice the workgroups pay that twice (2.64 against 2.51 ms).
int rows_block_of(const pso_ps_ctx* h) { return h->block_threads ? h->block_threads : kRowsBlock; }

#define PSO_PS_DISPATCH_BLOCK(h, e, CALL)   \
    switch (block_of(h)) {                  \
        case 64: e = CALL(64); break;       \
        case 128: e = CALL(128); break;     \
        case 256: e = CALL(256); break;     \
        case 512: e = CALL(512); break;     \
        case 1024: e = CALL(1024); break;   \
        default: return PSO_PS_EINVAL;      \
    }

template <int BLOCK>
hipError_t launch_update(const pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m,
                         float* gbest_loss, hipStream_t stream) {
    const bool vec = vector_path(h);
    TileOrder ord;
    unsigned long long grid = 0;
    const unsigned long long tiles =
        tiles_per_row(h->K, b.n, vec, BLOCK * 4u, [&](int i) { return b.x + (long long)i * b.ld; }) +
        (vec ? origin_slack(h, BLOCK * 4u) : 0ull);
    if (!plan_order(h, h->K, tiles, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((update_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, (const Selection*)h->sel, m, ord, gbest_loss,
                           h->chunk_origin);
    else
        hipLaunchKernelGGL((update_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, (const Selection*)h->sel, m, ord, gbest_loss, 0);
    return hipGetLastError();
}

template <int BLOCK>
hipError_t launch_update_rows(const pso_ps_ctx* h, const RowTable& tab, const float* gbest,
                              int row0, int rows, const MoveParams& m, float* gbest_loss,
                              hipStream_t stream) {
    const bool vec = vector_path(h);
    TileOrder ord;
    unsigned long long grid = 0;
    const long long n = (long long)h->D;
    const unsigned long long tiles =
        tiles_per_row(rows, n, vec, BLOCK * 4u, [&](int i) { return tab.x[i]; });
    if (!plan_order(h, rows, tiles, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((update_rows_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, tab, gbest, n, row0, rows, (const Selection*)h->sel, m, ord,
                           gbest_loss);
    else
        hipLaunchKernelGGL((update_rows_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, tab, gbest, n, row0, rows, (const Selection*)h->sel, m, ord,
                           gbest_loss);
    return hipGetLastError();
}

// Order of the gbest copy over `tiles` copy tiles of one row: chunks of the same
// bytes as the update pass's, whatever its tile size.
bool plan_copy_order(const pso_ps_ctx* h, unsigned long long tiles, TileOrder* ord,
                     unsigned long long* grid) {
    if (!h->eight_xcds) return plan_tile_order(1, tiles, 1ull << 30, 1, ord, grid);
    const unsigned long long update_tile = (unsigned long long)block_of(h) * 16u;  // bytes
    unsigned long long super = h->super_tiles ? h->super_tiles * update_tile : kDefaultSuperBytes;
    unsigned long long chunk = h->chunk_tiles ? h->chunk_tiles * update_tile : kDefaultChunkBytes;
    super /= kCopyTile * 4ull;
    chunk /= kCopyTile * 4ull;
    unsigned long long super2 = 1, chunk2 = 1;  // the planner wants powers of two
    while (super2 * 2 <= super) super2 *= 2;
    while (chunk2 * 2 <= chunk) chunk2 *= 2;
    return plan_tile_order(1, tiles, super2, chunk2, ord, grid);
}

// Selection (if do_select) and the gbest copy from `source`, whose `rows` rows
// start at row_x(0..rows-1).
template <class Source, class RowX>
int enqueue_select_gbest(pso_ps_ctx* h, float* pbest_loss, const float* loss, const Source& source,
                         int rows, RowX row_x, float* gbest, long long n, const float* gbest_loss,
                         bool do_select, hipStream_t stream) {
    TileOrder ord;
    unsigned long long grid = 0;
    const unsigned long long tiles = tiles_per_row(rows, n, true, kCopyTile, row_x);
    if (!plan_copy_order(h, tiles, &ord, &grid)) return hip_fail(h, hipErrorInvalidConfiguration);
    hipLaunchKernelGGL((select_gbest_kernel<Source>), dim3((unsigned)grid), dim3(kCopyBlock), 0,
                       stream, h->K, loss, pbest_loss, h->sel, source, gbest, n, gbest_loss,
                       do_select ? 1 : 0, ord);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    if (do_select) h->have_selection = true;
    return PSO_PS_OK;
}

// Enqueue the update pass over one dense block (already validated).
int enqueue_update(pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, float* gbest_loss,
                   hipStream_t stream) {
    if (b.n == 0) return PSO_PS_OK;
    hipError_t e;
#define CALL(B) launch_update<B>(h, b, m, gbest_loss, stream)
    PSO_PS_DISPATCH_BLOCK(h, e, CALL)
#undef CALL
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

int enqueue_update_rows(pso_ps_ctx* h, const RowTable& tab, const float* gbest, int row0, int rows,
                        const MoveParams& m, float* gbest_loss, hipStream_t stream) {
    hipError_t e;
    switch (rows_block_of(h)) {
        case 64: e = launch_update_rows<64>(h, tab, gbest, row0, rows, m, gbest_loss, stream); break;
        case 128: e = launch_update_rows<128>(h, tab, gbest, row0, rows, m, gbest_loss, stream); break;
        case 256: e = launch_update_rows<256>(h, tab, gbest, row0, rows, m, gbest_loss, stream); break;
        case 512: e = launch_update_rows<512>(h, tab, gbest, row0, rows, m, gbest_loss, stream); break;
        case 1024: e = launch_update_rows<1024>(h, tab, gbest, row0, rows, m, gbest_loss, stream); break;
        default: return PSO_PS_EINVAL;
    }
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

// The single-pass variant of the flat stage: a one-wavefront selection launch,
// then one launch that walks all K rows of each column tile.
template <int BLOCK>
hipError_t launch_fused(const pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m,
                        float* gbest_loss, hipStream_t stream) {
    TileOrder ord;
    unsigned long long grid = 0;
    const unsigned long long tiles = tiles_per_row(1, b.n, true, BLOCK * 4u, [&](int) { return b.x; });
    if (!plan_order(h, 1, tiles, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
#define PSO_PS_FUSED(P)                                                                          \
    hipLaunchKernelGGL((fused_rows_kernel<BLOCK, P>), dim3((unsigned)grid), dim3(BLOCK), lds,    \
                       stream, b, h->K, (const Selection*)h->sel, m, ord, gbest_loss)
    switch (h->fused_rows) {
        case 1: PSO_PS_FUSED(1); break;
        case 2: PSO_PS_FUSED(2); break;
        case 3: PSO_PS_FUSED(3); break;
        case 4: PSO_PS_FUSED(4); break;
        case 6: PSO_PS_FUSED(6); break;
        case 8: PSO_PS_FUSED(8); break;
        default: return hipErrorInvalidValue;
    }
#undef PSO_PS_FUSED
    return hipGetLastError();
}

int enqueue_select_only(pso_ps_ctx* h, float* pbest_loss, const float* loss, const float* gbest_loss,
                        hipStream_t stream) {
    hipLaunchKernelGGL(select_only_kernel, dim3(1), dim3(64), 0, stream, h->K, loss, pbest_loss,
                       h->sel, gbest_loss);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    h->have_selection = true;
    return PSO_PS_OK;
}

int enqueue_fused(pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, float* gbest_loss,
                  hipStream_t stream) {
    hipError_t e;
    switch (block_of(h)) {
        case 64: e = launch_fused<64>(h, b, m, gbest_loss, stream); break;
        case 128: e = launch_fused<128>(h, b, m, gbest_loss, stream); break;
        case 256: e = launch_fused<256>(h, b, m, gbest_loss, stream); break;
        default: return PSO_PS_EINVAL;
    }
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

// The two launches of the "best first" split: see select_move_best_kernel.  The
// first launch is short (one row), so it takes the whole compute unit (no
// occupancy cap: 0.383 against 0.396 ms per stage at K = 8, D = 14.7 M).
constexpr int kBestBlock = 64;

int enqueue_move_best(pso_ps_ctx* h, const ColumnBlock& b, float* pbest_loss, const float* loss,
                      const MoveParams& m, hipStream_t stream) {
    const bool vec = vector_path(h);
    TileOrder one;
    unsigned long long grid = 0;
    const unsigned long long tiles = tiles_per_row(
        h->K, b.n, vec, kBestBlock * 4u, [&](int i) { return b.x + (long long)i * b.ld; });
    if (!plan_order(h, 1, tiles, kBestBlock * 4u, &one, &grid))
        return hip_fail(h, hipErrorInvalidConfiguration);
    if (vec)
        hipLaunchKernelGGL((select_move_best_kernel<kBestBlock, true>), dim3((unsigned)grid),
                           dim3(kBestBlock), 0, stream, b, h->K, loss, pbest_loss, h->sel, m, one);
    else
        hipLaunchKernelGGL((select_move_best_kernel<kBestBlock, false>), dim3((unsigned)grid),
                           dim3(kBestBlock), 0, stream, b, h->K, loss, pbest_loss, h->sel, m, one);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    h->have_selection = true;
    return PSO_PS_OK;
}

template <int BLOCK>
hipError_t launch_update_others(const pso_ps_ctx* h, const ColumnBlock& b, float* pbest_loss,
                                const float* loss, const MoveParams& m, hipStream_t stream) {
    const bool vec = vector_path(h);
    const unsigned long long tiles = tiles_per_row(
        h->K, b.n, vec, BLOCK * 4u, [&](int i) { return b.x + (long long)i * b.ld; });
    TileOrder ord;
    unsigned long long grid = 0;
    // K = 1: only the pbest_loss update is left (an order for one row, unused)
    if (!plan_order(h, h->K > 1 ? h->K - 1 : 1, tiles, BLOCK * 4u, &ord, &grid))
        return hipErrorInvalidConfiguration;
    if (h->K == 1) grid = 8;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((update_others_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, loss, pbest_loss, (const Selection*)h->sel, m, ord);
    else
        hipLaunchKernelGGL((update_others_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, loss, pbest_loss, (const Selection*)h->sel, m, ord);
    return hipGetLastError();
}

int enqueue_update_others(pso_ps_ctx* h, const ColumnBlock& b, float* pbest_loss, const float* loss,
                          const MoveParams& m, hipStream_t stream) {
    hipError_t e;
#define CALL(B) launch_update_others<B>(h, b, pbest_loss, loss, m, stream)
    PSO_PS_DISPATCH_BLOCK(h, e, CALL)
#undef CALL
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

// The stage as one launch of whole_stage_kernel.
bool single_launch_possible(const pso_ps_ctx* h) { return h->K <= kStageMaxK && h->tickets; }

// Up to this many particle parameters (K * D) the single launch measured
// faster than two launches on MI355X.
constexpr long long kSingleLaunchMaxParams = PSO_PS_SINGLE_LAUNCH_MAX_PARAMS;

bool single_launch_chosen(const pso_ps_ctx* h) {
    if (!single_launch_possible(h) || h->single_launch == 0 || h->fused_rows > 0) return false;
    if (h->single_launch > 0) return true;
    // by itself only where it measured faster: one particle per wavefront
    return h->K <= kStageWaves && (long long)h->K * (long long)h->D <= kSingleLaunchMaxParams;
}

int enqueue_whole_stage(pso_ps_ctx* h, const ColumnBlock& b, float* pbest_loss, const float* loss,
                        const MoveParams& m, float* gbest_loss, hipStream_t stream) {
    const unsigned long long phase = (reinterpret_cast<uintptr_t>(b.x) >> 2) & (kStageTile - 1u);
    const unsigned long long grid = (phase + (unsigned long long)b.n + kStageTile - 1u) / kStageTile;
    if (grid >= (1ull << 31)) return hip_fail(h, hipErrorInvalidConfiguration);
    const int waves = h->K < kStageWaves ? h->K : kStageWaves;
    hipLaunchKernelGGL(whole_stage_kernel, dim3((unsigned)grid), dim3(64u * (unsigned)waves), 0, stream,
                       b, h->K, loss, pbest_loss, h->sel, m, gbest_loss, h->tickets);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    h->have_selection = true;
    return PSO_PS_OK;
}

// The ragged stage as one launch: every segment of `blocks` (at most kTableSegs).
int enqueue_whole_stage_segments(pso_ps_ctx* h, const std::vector<ColumnBlock>& blocks,
                                 float* pbest_loss, const float* loss, const MoveParams& m,
                                 float* gbest_loss, hipStream_t stream) {
    StageTable tab;
    tab.count = (int)blocks.size();
    unsigned long long wgs = 0;
    for (int s = 0; s < kTableSegs; ++s) {
        StageEntry& e = tab.seg[s];
        if (s >= tab.count) {
            e = tab.seg[tab.count - 1];  // never selected: segment_of stops at count
            tab.first_wg[s] = 0xffffffffu;
            continue;
        }
        const ColumnBlock& b = blocks[(size_t)s];
        e.x = b.x; e.v = b.v; e.pbest = b.pbest; e.gbest = b.gbest;
        e.n = b.n; e.d0 = b.d0; e.reserved = 0;
        e.first_wg = tab.first_wg[s] = (unsigned)wgs;
        const unsigned long long phase = (reinterpret_cast<uintptr_t>(b.x) >> 2) & (kStageTile - 1u);
        wgs += (phase + (unsigned long long)b.n + kStageTile - 1u) / kStageTile;
        if (wgs >= (1ull << 31)) return hip_fail(h, hipErrorInvalidConfiguration);
    }
    const int waves = h->K < kStageWaves ? h->K : kStageWaves;
    hipLaunchKernelGGL(whole_stage_segments_kernel, dim3((unsigned)wgs), dim3(64u * (unsigned)waves), 0,
                       stream, tab, h->K, loss, pbest_loss, h->sel, m, gbest_loss, h->tickets);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    h->have_selection = true;
    return PSO_PS_OK;
}

MoveParams make_params(float w, float c1, float c2, uint64_t seed, uint64_t step) {
    MoveParams m;
    m.w = w; m.c1 = c1; m.c2 = c2;
    m.key0 = (uint32_t)seed; m.key1 = (uint32_t)(seed >> 32);
    m.step_lo = (uint32_t)step; m.step_hi = (uint32_t)(step >> 32);
    return m;
}

bool is_pow2(int t) { return t > 0 && (t & (t - 1)) == 0; }

// The flat stage, or one of its two launches (parts & 1: the first, parts & 2:
// the second); gbest_loss == null: best of this stage, else historical gBest.
// Which kernels the two launches are:
//   default, no history   selection + move of the best particle | the other particles
//   history, or the copy-based split on request
//                         selection + gbest copy | all K particles
//   single pass on request
//                         selection (one wavefront) | all K particles, one workgroup per column tile
// A small swarm (or any of K <= 64 on request) takes the whole stage as one
// launch instead, when it is not asked for in two parts.
int sync_flat(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss, const float* loss,
              float* gbest, float* gbest_loss, const MoveParams& m, hipStream_t stream,
              int parts = 3) {
    if (!h || !pbest_loss || !loss) return PSO_PS_EINVAL;
    if (parts == 2 && !h->have_selection) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4) || !aligned_to(gbest_loss, 4))
        return PSO_PS_EALIGN;
    ColumnBlock b{x, v, pbest, gbest, (long long)h->ld, (long long)h->D, 0ull};
    int rc = check_block(b);
    if (rc != PSO_PS_OK) return rc;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    if (parts == 3 && single_launch_chosen(h))
        return enqueue_whole_stage(h, b, pbest_loss, loss, m, gbest_loss, stream);
    const bool fused = h->fused_rows > 0;
    const bool best_first = !fused && h->best_first && !gbest_loss;
    if (parts & 1) {
        if (fused)
            rc = enqueue_select_only(h, pbest_loss, loss, gbest_loss, stream);
        else if (best_first)
            rc = enqueue_move_best(h, b, pbest_loss, loss, m, stream);
        else
            rc = enqueue_select_gbest(h, pbest_loss, loss, StackedSource{x, b.ld}, h->K,
                                      [&](int i) { return x + (long long)i * b.ld; }, gbest, b.n,
                                      gbest_loss, true, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    if (parts & 2) {
        if (fused)
            rc = enqueue_fused(h, b, m, gbest_loss, stream);
        else if (best_first)
            rc = enqueue_update_others(h, b, pbest_loss, loss, m, stream);
        else
            rc = enqueue_update(h, b, m, gbest_loss, stream);
        if (rc == PSO_PS_OK) h->last_stream = stream;
    }
    return rc;
}

// The ragged stage; gbest_loss as in sync_flat.
int sync_segments(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg, float* const* pbest_seg,
                  float* pbest_loss, const float* loss, float* const* gbest_seg, float* gbest_loss,
                  const MoveParams& m, hipStream_t stream) {
    if (!h || !x_seg || !v_seg || !pbest_seg || !gbest_seg || !pbest_loss || !loss)
        return PSO_PS_EINVAL;
    if (h->seg_sizes.empty()) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4) || !aligned_to(gbest_loss, 4))
        return PSO_PS_EALIGN;
    const int n_seg = (int)h->seg_sizes.size();
    // Validate every segment before anything is enqueued.  The work lists were
    // reserved at create: no allocation happens here.
    std::vector<ColumnBlock>& blocks = h->seg_blocks;
    std::vector<SegTable>& tables = h->seg_tables;
    std::vector<CopyTable>& copy_tables = h->seg_copy_tables;
    std::vector<unsigned>& update_totals = h->seg_update_wgs;
    std::vector<unsigned>& copy_totals = h->seg_copy_wgs;
    blocks.clear(); tables.clear(); copy_tables.clear(); update_totals.clear(); copy_totals.clear();
    unsigned long long start = 0;
    for (int s = 0; s < n_seg; ++s) {
        const long long n = (long long)h->seg_sizes[s];
        if (n > 0) {
            ColumnBlock b{x_seg[s], v_seg[s], pbest_seg[s], gbest_seg[s], n, n, start};
            const int rc = check_block(b);
            if (rc != PSO_PS_OK) return rc;
            blocks.push_back(b);
        }
        start += (unsigned long long)n;
    }
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    if (single_launch_chosen(h) && !blocks.empty() && blocks.size() <= (size_t)kTableSegs)
        return enqueue_whole_stage_segments(h, blocks, pbest_loss, loss, m, gbest_loss, stream);
    const int block = block_of(h);
    const bool vec = vector_path(h);
    // Up to kTableSegs segments per launch; the selection rides on the first
    // gbest-copy launch.  All copies are enqueued before the first update.
    for (size_t first = 0; first < blocks.size(); first += kTableSegs) {
        SegTable tab;
        CopyTable ctab;
        tab.count = (int)((blocks.size() - first < (size_t)kTableSegs) ? blocks.size() - first
                                                                      : (size_t)kTableSegs);
        ctab.count = tab.count;
        unsigned long long update_wg = 0, copy_wg = 0;
        for (int s = 0; s < kTableSegs; ++s) {
            SegEntry& e = tab.seg[s];
            CopyEntry& c = ctab.seg[s];
            if (s >= tab.count) {
                e = tab.seg[tab.count - 1];  // never selected: segment_of stops at count
                c = ctab.seg[tab.count - 1];
                tab.first_wg[s] = 0xffffffffu;
                ctab.first_wg[s] = 0xffffffffu;
                continue;
            }
            const ColumnBlock& b = blocks[first + s];
            const auto row_x = [&](int i) { return b.x + (long long)i * b.ld; };
            e.x = b.x; e.v = b.v; e.pbest = b.pbest; e.gbest = b.gbest;
            e.n = b.n; e.d0 = b.d0;
            e.vec = vec ? 1 : 0;
            c.x = b.x; c.gbest = b.gbest; c.n = b.n; c.reserved = 0;
            const unsigned tile = (unsigned)block * 4u;
            unsigned long long grid = 0, copy_grid = 0;
            if (!plan_order(h, h->K, tiles_per_row(h->K, b.n, vec, tile, row_x), tile, &e.ord, &grid) ||
                !plan_copy_order(h, tiles_per_row(h->K, b.n, true, kCopyTile, row_x), &c.ord,
                                 &copy_grid))
                return hip_fail(h, hipErrorInvalidConfiguration);
            e.first_wg = tab.first_wg[s] = (unsigned)update_wg;
            c.first_wg = ctab.first_wg[s] = (unsigned)copy_wg;
            update_wg += grid;
            copy_wg += copy_grid;
            if (update_wg >= (1ull << 31) || copy_wg >= (1ull << 31))
                return hip_fail(h, hipErrorInvalidConfiguration);
        }
        tables.push_back(tab);
        copy_tables.push_back(ctab);
        update_totals.push_back((unsigned)update_wg);
        copy_totals.push_back((unsigned)copy_wg);
    }
    for (size_t t = 0; t < copy_tables.size(); ++t) {
        hipLaunchKernelGGL(select_gbest_segments_kernel, dim3(copy_totals[t]), dim3(kCopyBlock), 0,
                           stream, h->K, loss, pbest_loss, h->sel, copy_tables[t],
                           (const float*)gbest_loss, t == 0 ? 1 : 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(h, e);
    }
    h->last_stream = stream;
    h->have_selection = true;
    const unsigned lds = occupancy_cap_lds(h, block);
    for (size_t t = 0; t < tables.size(); ++t) {
        float* const store_loss = t == 0 ? gbest_loss : nullptr;
#define PSO_PS_LAUNCH(B)                                                                      \
    hipLaunchKernelGGL(update_segments_kernel<B>, dim3(update_totals[t]), dim3(B), lds, stream, \
                       tables[t], h->K, (const Selection*)h->sel, m, store_loss)
        switch (block) {
            case 64: PSO_PS_LAUNCH(64); break;
            case 128: PSO_PS_LAUNCH(128); break;
            case 256: PSO_PS_LAUNCH(256); break;
            case 512: PSO_PS_LAUNCH(512); break;
            case 1024: PSO_PS_LAUNCH(1024); break;
            default: return PSO_PS_EINVAL;
        }
#undef PSO_PS_LAUNCH
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(h, e);
    }
    return PSO_PS_OK;
}

// The stage on K separate rows; gbest_loss as in sync_flat.
int sync_rows(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows, float* const* pbest_rows,
              float* pbest_loss, const float* loss, float* gbest, float* gbest_loss,
              const MoveParams& m, hipStream_t stream) {
    if (!h || !x_rows || !v_rows || !pbest_rows || !pbest_loss || !loss || !gbest)
        return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4) || !aligned_to(gbest_loss, 4))
        return PSO_PS_EALIGN;
    for (int i = 0; i < h->K; ++i) {
        const int rc = check_arrays(x_rows[i], v_rows[i], pbest_rows[i], gbest);
        if (rc != PSO_PS_OK) return rc;
    }
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const long long n = (long long)h->D;
    if (single_launch_chosen(h)) {   // implies K <= kTableRows
        TableRows rows;
        for (int i = 0; i < kTableRows; ++i) {
            rows.tab.x[i] = (i < h->K) ? x_rows[i] : nullptr;
            rows.tab.v[i] = (i < h->K) ? v_rows[i] : nullptr;
            rows.tab.pbest[i] = (i < h->K) ? pbest_rows[i] : nullptr;
        }
        const unsigned long long phase = (reinterpret_cast<uintptr_t>(x_rows[0]) >> 2) & (kStageTile - 1u);
        const unsigned long long grid = (phase + (unsigned long long)n + kStageTile - 1u) / kStageTile;
        if (grid >= (1ull << 31)) return hip_fail(h, hipErrorInvalidConfiguration);
        const int waves = h->K < kStageWaves ? h->K : kStageWaves;
        hipLaunchKernelGGL(whole_stage_rows_kernel, dim3((unsigned)grid), dim3(64u * (unsigned)waves), 0,
                           stream, rows, gbest, n, h->K, loss, pbest_loss, h->sel, m, gbest_loss,
                           h->tickets);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(h, e);
        h->last_stream = stream;
        h->have_selection = true;
        return PSO_PS_OK;
    }
    // gbest copies first (each launch carries up to kTableRows row pointers and
    // copies only if g is among them), then the updates.
    for (int row0 = 0; row0 < h->K; row0 += kTableRows) {
        TableSource src;
        src.row0 = row0;
        src.rows = (h->K - row0 < kTableRows) ? h->K - row0 : kTableRows;
        for (int i = 0; i < kTableRows; ++i) src.x[i] = (i < src.rows) ? x_rows[row0 + i] : nullptr;
        const int rc = enqueue_select_gbest(h, pbest_loss, loss, src, src.rows,
                                            [&](int i) { return x_rows[row0 + i]; }, gbest, n,
                                            gbest_loss, row0 == 0, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    for (int row0 = 0; row0 < h->K; row0 += kTableRows) {
        RowTable tab;
        const int rows = (h->K - row0 < kTableRows) ? h->K - row0 : kTableRows;
        for (int i = 0; i < kTableRows; ++i) {
            tab.x[i] = (i < rows) ? x_rows[row0 + i] : nullptr;
            tab.v[i] = (i < rows) ? v_rows[row0 + i] : nullptr;
            tab.pbest[i] = (i < rows) ? pbest_rows[row0 + i] : nullptr;
        }
        const int rc = enqueue_update_rows(h, tab, gbest, row0, rows, m,
                                           row0 == 0 ? gbest_loss : nullptr, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    return PSO_PS_OK;
}

// The stage for callers that must not allocate: looks up, once per device, the
// address that the file-scope array `scratch` has on that GPU.
constexpr int kMaxDevices = 64;
struct StaticDevice {
    bool ready = false;
    Selection* ptr = nullptr;  // device address of `scratch` on this GPU
    bool eight_xcds = false;
};
StaticDevice g_static_device[kMaxDevices];
std::mutex g_static_mutex;

// Device address of the static scratch on `device` (which must be current).
hipError_t static_scratch(int device, StaticDevice* out) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticDevice& d = g_static_device[device];
    if (!d.ready) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        int compute_units = 0;
        e = hipDeviceGetAttribute(&compute_units, hipDeviceAttributeMultiprocessorCount, device);
        if (e != hipSuccess) return e;
        d.ptr = static_cast<Selection*>(ptr);
        d.eight_xcds = compute_units == 256;
        d.ready = true;
    }
    *out = d;
    return hipSuccess;
}

}  // namespace

extern "C" {

int pso_ps_create(pso_ps_ctx** out, int K, int64_t D, int64_t ld, int n_seg,
                  const int64_t* seg_sizes, int device) {
    if (!out) return PSO_PS_EINVAL;
    *out = nullptr;
    if (K < 1 || D < 1 || ld < D || n_seg < 0 || device < 0) return PSO_PS_EINVAL;
    if (n_seg > 0 && !seg_sizes) return PSO_PS_EINVAL;
    if ((uint64_t)D > (1ull << 33)) return PSO_PS_EINVAL;
    int64_t total = 0;
    for (int s = 0; s < n_seg; ++s) {
        if (seg_sizes[s] < 0 || seg_sizes[s] > D) return PSO_PS_EINVAL;
        total += seg_sizes[s];
        if (total > D) return PSO_PS_EINVAL;
    }
    if (n_seg > 0 && total != D) return PSO_PS_EINVAL;

    pso_ps_ctx* h = new (std::nothrow) pso_ps_ctx();
    if (!h) return PSO_PS_ENOMEM;
    h->K = K; h->D = D; h->ld = ld; h->device = device;
    try {
        if (n_seg > 0) {
            h->seg_sizes.assign(seg_sizes, seg_sizes + n_seg);
            const size_t launches = ((size_t)n_seg + kTableSegs - 1) / kTableSegs;
            h->seg_blocks.reserve((size_t)n_seg);
            h->seg_tables.reserve(launches);
            h->seg_copy_tables.reserve(launches);
            h->seg_update_wgs.reserve(launches);
            h->seg_copy_wgs.reserve(launches);
        }
    } catch (...) {
        delete h;
        return PSO_PS_ENOMEM;
    }
    h->mask_words = (K + 63) / 64;
    h->sel_bytes = sizeof(Selection) + (size_t)(h->mask_words - 1) * sizeof(uint64_t);
    h->sel = nullptr; h->last_stream = nullptr; h->have_selection = false;
    h->block_threads = 0; h->super_tiles = 0; h->chunk_tiles = 0; h->wgs_per_cu = 0;
    h->force_generic = false; h->fused_rows = 0; h->chunk_origin = 0; h->best_first = true; h->eight_xcds = true; h->last_hip_error = 0;
    h->single_launch = -1; h->tickets = nullptr;

    DeviceScope scope(device);
    hipError_t e = scope.err;
    int compute_units = 0;
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&compute_units, hipDeviceAttributeMultiprocessorCount, device);
    h->eight_xcds = compute_units == 256;
    if (e == hipSuccess) e = hipMalloc((void**)&h->sel, h->sel_bytes);
    if (e == hipSuccess) e = hipMemset(h->sel, 0, h->sel_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&h->tickets, kTicketBytes);
    if (e == hipSuccess) e = hipMemset(h->tickets, 0, kTicketBytes);
    if (e != hipSuccess) {
        if (h->tickets) (void)hipFree(h->tickets);
        if (h->sel) (void)hipFree(h->sel);
        delete h;
        (void)hipGetLastError();
        return PSO_PS_EHIP;
    }
    *out = h;
    return PSO_PS_OK;
}

int pso_ps_sync_begin(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                      const float* loss, float* gbest, float w, float c1, float c2,
                      uint64_t seed, uint64_t step, void* hip_stream) {
    return sync_flat(h, x, v, pbest, pbest_loss, loss, gbest, nullptr,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream, 1);
}

int pso_ps_sync_finish(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                       const float* loss, float* gbest, float w, float c1, float c2,
                       uint64_t seed, uint64_t step, void* hip_stream) {
    return sync_flat(h, x, v, pbest, pbest_loss, loss, gbest, nullptr,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream, 2);
}

int pso_ps_sync(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                const float* loss, float* gbest, float w, float c1, float c2,
                uint64_t seed, uint64_t step, void* hip_stream) {
    return sync_flat(h, x, v, pbest, pbest_loss, loss, gbest, nullptr,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_history(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                        const float* loss, float* gbest, float* gbest_loss, float w, float c1,
                        float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!gbest_loss) return PSO_PS_EINVAL;
    return sync_flat(h, x, v, pbest, pbest_loss, loss, gbest, gbest_loss,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_static(int device, int K, int64_t D, int64_t ld, float* x, float* v, float* pbest,
                       float* pbest_loss, const float* loss, float* gbest, float w, float c1,
                       float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (device < 0 || device >= kMaxDevices || K < 1 || D < 1 || ld < D) return PSO_PS_EINVAL;
    if ((uint64_t)D > (1ull << 33)) return PSO_PS_EINVAL;
    if (K > kStaticMaxK) return PSO_PS_ELIMIT;
    DeviceScope scope(device);
    if (scope.err != hipSuccess) return PSO_PS_EHIP;
    StaticDevice dev;
    if (static_scratch(device, &dev) != hipSuccess) {
        (void)hipGetLastError();
        return PSO_PS_EHIP;
    }
    // A handle on the stack: default launch shape, the static scratch, no
    // segment lists (empty vectors own no memory).
    pso_ps_ctx h;
    h.K = K; h.D = D; h.ld = ld; h.device = device;
    h.sel = dev.ptr; h.mask_words = (K + 63) / 64;
    h.sel_bytes = sizeof(Selection) + (size_t)(h.mask_words - 1) * sizeof(uint64_t);
    h.last_stream = nullptr; h.have_selection = false;
    h.block_threads = 0; h.super_tiles = 0; h.chunk_tiles = 0; h.wgs_per_cu = 0;
    h.force_generic = false; h.fused_rows = 0; h.chunk_origin = 0; h.best_first = true; h.eight_xcds = dev.eight_xcds; h.last_hip_error = 0;
    h.single_launch = -1;
    h.tickets = reinterpret_cast<unsigned*>(reinterpret_cast<unsigned char*>(dev.ptr) +
                                            kStaticSelectionBytes);
    return sync_flat(&h, x, v, pbest, pbest_loss, loss, gbest, nullptr,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_segments(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                         float* const* pbest_seg, float* pbest_loss, const float* loss,
                         float* const* gbest_seg, float w, float c1, float c2,
                         uint64_t seed, uint64_t step, void* hip_stream) {
    return sync_segments(h, x_seg, v_seg, pbest_seg, pbest_loss, loss, gbest_seg, nullptr,
                         make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_segments_history(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                                 float* const* pbest_seg, float* pbest_loss, const float* loss,
                                 float* const* gbest_seg, float* gbest_loss, float w, float c1,
                                 float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!gbest_loss) return PSO_PS_EINVAL;
    return sync_segments(h, x_seg, v_seg, pbest_seg, pbest_loss, loss, gbest_seg, gbest_loss,
                         make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_rows(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows,
                     float* const* pbest_rows, float* pbest_loss, const float* loss, float* gbest,
                     float w, float c1, float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    return sync_rows(h, x_rows, v_rows, pbest_rows, pbest_loss, loss, gbest, nullptr,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_sync_rows_history(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows,
                             float* const* pbest_rows, float* pbest_loss, const float* loss,
                             float* gbest, float* gbest_loss, float w, float c1, float c2,
                             uint64_t seed, uint64_t step, void* hip_stream) {
    if (!gbest_loss) return PSO_PS_EINVAL;
    return sync_rows(h, x_rows, v_rows, pbest_rows, pbest_loss, loss, gbest, gbest_loss,
                     make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
}

int pso_ps_average(pso_ps_ctx* h, float* x, float* mean, void* hip_stream) {
    if (!h || !x || !mean) return PSO_PS_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(mean, 4)) return PSO_PS_EALIGN;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    const long long n = (long long)h->D;
    const long long ld = (long long)h->ld;
    const long long blocks = (n + (long long)kMeanTile - 1) / (long long)kMeanTile;
    TileOrder mean_ord;
    unsigned long long mean_grid = 0;
    if (!plan_order(h, 1, (unsigned long long)blocks, kMeanTile, &mean_ord, &mean_grid))
        return hip_fail(h, hipErrorInvalidConfiguration);
    hipLaunchKernelGGL(mean_kernel, dim3((unsigned)mean_grid), dim3(kMeanBlock), 0, stream,
                       (const float*)x, mean, ld, n, h->K, mean_ord);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    // Tiles are aligned to each row's own address, so any 4-byte aligned row
    // can take the 128-bit stores.
    const bool vec = !h->force_generic;
    constexpr int BLOCK = 128;  // a write-only stream wants 128 threads: 64 cost 17 % here
    TileOrder ord;
    unsigned long long grid = 0;
    const unsigned long long tiles =
        tiles_per_row(h->K, n, vec, BLOCK * 4u, [&](int i) { return x + (long long)i * ld; });
    if (!plan_order(h, h->K, tiles, BLOCK * 4u, &ord, &grid))
        return hip_fail(h, hipErrorInvalidConfiguration);
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((broadcast_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, x, (const float*)mean, ld, n, h->K, ord);
    else
        hipLaunchKernelGGL((broadcast_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, x, (const float*)mean, ld, n, h->K, ord);
    e = hipGetLastError();
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

float pso_ps_inertia(int64_t t, int64_t t_max, float m_max, float m_min) {
    const double span = (double)m_max - (double)m_min;
    return (float)((double)m_max - ((double)t * span) / (double)t_max);
}

int pso_ps_schedule(int64_t t, int64_t iteration_size, int64_t epoch_size, int64_t step,
                    float m_max, float m_min, float c1, float c2,
                    int* is_stage, float* w, float* c1_eff, float* c2_eff) {
    if (!is_stage || !w || !c1_eff || !c2_eff) return PSO_PS_EINVAL;
    if (t < 1 || iteration_size < 1 || epoch_size < 1 || step < 1) return PSO_PS_EINVAL;
    if (epoch_size > INT64_MAX / iteration_size) return PSO_PS_EINVAL;
    const int64_t last = epoch_size * iteration_size;  // Max_t of Algorithm 1
    if (t > last) return PSO_PS_EINVAL;
    const float lambda = (float)((t - 1) / iteration_size + 1);
    *is_stage = (t < last && t % step == 0) ? 1 : 0;
    *w = pso_ps_inertia(t, last, m_max, m_min);
    *c1_eff = c1 / lambda;
    *c2_eff = c2 / lambda;
    return PSO_PS_OK;
}

int pso_ps_last_selection(pso_ps_ctx* h, int* g_out, uint64_t* improved_mask_out, int mask_words,
                          int* replaced_out) {
    if (!h || !h->have_selection) return PSO_PS_EINVAL;
    if (improved_mask_out && mask_words < h->mask_words) return PSO_PS_EINVAL;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    hipError_t e = hipStreamSynchronize(h->last_stream);
    if (e != hipSuccess) return hip_fail(h, e);
    std::vector<unsigned char> host;
    try {
        host.resize(h->sel_bytes);
    } catch (...) {
        return PSO_PS_ENOMEM;
    }
    e = hipMemcpy(host.data(), h->sel, h->sel_bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(h, e);
    const Selection* s = reinterpret_cast<const Selection*>(host.data());
    if (g_out) *g_out = s->g;
    if (replaced_out) *replaced_out = s->replaced;
    if (improved_mask_out)
        for (int j = 0; j < h->mask_words; ++j) improved_mask_out[j] = s->improved[j];
    return PSO_PS_OK;
}

int pso_ps_set_launch(pso_ps_ctx* h, int block_threads, int super_tiles, int chunk_tiles,
                      int wgs_per_cu, int force_generic) {
    if (!h) return PSO_PS_EINVAL;
    switch (block_threads) {
        case 0: case 64: case 128: case 256: case 512: case 1024: break;
        default: return PSO_PS_EINVAL;
    }
    if (super_tiles != 0 && (!is_pow2(super_tiles) || super_tiles > (1 << 20))) return PSO_PS_EINVAL;
    if (chunk_tiles != 0 && (!is_pow2(chunk_tiles) || chunk_tiles > (1 << 20))) return PSO_PS_EINVAL;
    if (wgs_per_cu < 0 || (wgs_per_cu > 0 && wgs_per_cu < 3)) return PSO_PS_EINVAL;
    h->block_threads = block_threads;
    h->super_tiles = super_tiles;
    h->chunk_tiles = chunk_tiles;
    h->wgs_per_cu = wgs_per_cu;
    h->force_generic = force_generic != 0;
    return PSO_PS_OK;
}

int pso_ps_set_variant(pso_ps_ctx* h, int fused_rows, int chunk_origin, int best_first) {
    if (!h || chunk_origin < 0 || chunk_origin > 2) return PSO_PS_EINVAL;
    h->best_first = best_first != 0;
    switch (fused_rows) {
        case 0: case 1: case 2: case 3: case 4: case 6: case 8: break;
        default: return PSO_PS_EINVAL;
    }
    h->fused_rows = fused_rows;
    h->chunk_origin = chunk_origin;
    return PSO_PS_OK;
}

int pso_ps_set_single_launch(pso_ps_ctx* h, int mode) {
    if (!h || mode < -1 || mode > 1) return PSO_PS_EINVAL;
    if (mode == 1 && !single_launch_possible(h)) return PSO_PS_ELIMIT;
    h->single_launch = mode;
    return PSO_PS_OK;
}

int pso_ps_last_hip_error(const pso_ps_ctx* h) { return h ? h->last_hip_error : 0; }

int pso_ps_destroy(pso_ps_ctx* h) {
    if (!h) return PSO_PS_OK;
    int rc = PSO_PS_OK;
    {
        DeviceScope scope(h->device);
        if (h->sel && hipFree(h->sel) != hipSuccess) rc = PSO_PS_EHIP;
        if (h->tickets && hipFree(h->tickets) != hipSuccess) rc = PSO_PS_EHIP;
    }
    delete h;
    return rc;
}

#ifndef PSO_PS_SOURCE_HASH
#define PSO_PS_SOURCE_HASH "unstamped"
#endif
const char* pso_ps_source_hash(void) {
    // The marker lets a tool find the stamp in the file without loading it.
    static const char stamp[] = "pso_ps_source_hash=" PSO_PS_SOURCE_HASH;
    return stamp + sizeof("pso_ps_source_hash=") - 1;
}

const char* pso_ps_strerror(int code) {
    switch (code) {
        case PSO_PS_OK: return "ok";
        case PSO_PS_EINVAL: return "invalid argument";
        case PSO_PS_EALIGN: return "array not 4-byte aligned";
        case PSO_PS_EHIP: return "HIP runtime call failed";
        case PSO_PS_ENOMEM: return "host allocation failed";
        case PSO_PS_ELIMIT:
            return "more particles than the fixed scratch of the allocation-free entry point or the "
                   "single-launch stage holds";
        default: return "unknown status code";
    }
}

}  // extern "C"
