// PSO-PS synchronization step for gfx950 (MI355X): HIP kernels and the C ABI
// declared in include/pso_ps.h.
//
// Two kernels per stage:
//   select_gbest_kernel  g = argmin loss (Algorithm 3), improved_i = loss_i <
//                        pbest_loss_i with the pbest_loss update (Algorithm 1),
//                        and the copy gbest = x_g (Algorithm 3's return value).
//   update_kernel        one streaming pass over [K, D]: conditional pbest
//                        copy, Eq. (6) velocity and Eq. (7) position update.
// The same two steps exist for K separate row arrays (update_rows_kernel, the
// gbest copy with a TableSource) and for ragged per-tensor segments, 32 per
// launch (select_gbest_segments_kernel, update_segments_kernel).  Parameter
// averaging, the synchronization the method replaces, is mean_kernel +
// broadcast_kernel.
//
// The update pass is bound by HBM traffic, not by arithmetic: per particle
// parameter it must read x and v, write x and v, and either read pbest (not
// improved) or write it (improved; its old value is not needed because
// pbest - x is then exactly zero): 20 bytes.  gbest costs 12 bytes per column
// (read x_g, write gbest, first read of gbest by the update pass); the other
// K-1 reads of a gbest tile are served by the caches.
//
// Mapping of the update pass: one workgroup = one row (particle) x one tile of
// BLOCK*4 consecutive floats, one 128-bit access per thread and array, i.e. the
// access pattern of a plain streaming copy.  What makes it reach copy-like
// bandwidth on this chip:
//   * tiles are aligned to the ADDRESS of the row (not to column 0), so every
//     wavefront touches whole 128-byte lines even when the row stride is not a
//     multiple of the tile (D = 25,557,032 gives rows 160 bytes off a 4 KiB
//     boundary); the ragged head and tail of a row are handled element-wise;
//   * x, v, pbest use non-temporal accesses (each byte is touched once); gbest
//     uses ordinary cached loads so that it stays resident;
//   * the workgroup order is XCD-aware: workgroup b runs on XCD b % 8, each XCD
//     is given chunks of consecutive tiles and walks a "super-chunk" of its
//     tiles for row 0, 1, .., K-1 before moving on, so that a gbest tile is
//     re-read from the XCD's own L2 and the DRAM pages of few rows are open at
//     a time;
//   * the Philox rounds are placed between the loads and their first use;
//   * each launch reserves LDS it never touches, which caps a compute unit at
//     about 20 resident wavefronts of the 32 it could hold: HBM serves fewer,
//     steadier request streams better than the full house.
// Because gbest is copied out by the first kernel, the in-place update of row g
// cannot race with anything.
//
// Compile with -ffp-contract=off: the only fused operations are the two
// explicit fmaf of the velocity update.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
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
// keeps its own workgroup order; its workgroups are first_update_wg .. (a
// multiple of 8, so that wg & 7 is still the XCD) in the update launch and
// first_copy_wg .. in the gbest copy launch.
constexpr int kTableSegs = 32;
struct SegEntry {
    float* x;
    float* v;
    float* pbest;
    float* gbest;
    long long n;
    unsigned long long d0;
    TileOrder ord;
    unsigned first_update_wg;
    unsigned first_copy_wg;
    int vec;
    int reserved;
};
struct SegTable {
    // The first workgroups again, side by side: the lookup scans them with two
    // wide scalar loads instead of touching every entry.
    unsigned first_update_wg[kTableSegs];
    unsigned first_copy_wg[kTableSegs];
    SegEntry seg[kTableSegs];
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
__device__ __forceinline__ void move_single(const RowPtrs& r, const float* __restrict__ gbest,
                                            unsigned long long d0, long long col, unsigned i,
                                            bool improved, const MoveParams& m) {
    const unsigned long long d = d0 + (unsigned long long)col;
    const Words4 words = philox4x32_10((uint32_t)(d >> 1), i, m.step_lo, m.step_hi, m.key0, m.key1);
    float xv = r.x[col];
    float vv = r.v[col];
    const float pv = improved ? xv : r.pbest[col];
    if (improved) r.pbest[col] = xv;
    const bool odd = d & 1ull;
    move_element(xv, vv, pv, gbest[col], odd ? words.s2 : words.s0, odd ? words.s3 : words.s1, m);
    r.x[col] = xv;
    r.v[col] = vv;
}

// Columns c .. c+3 of row i with 128-bit accesses (the addresses are 16-byte
// aligned in x, v and pbest, and d0 + c is even).  improved (uniform over the
// workgroup): Algorithm 1 replaced this particle's personal best by its
// position, so pbest is written instead of read.
__device__ __forceinline__ void move_quad(const RowPtrs& r, const float* __restrict__ gbest,
                                          unsigned long long d0, long long c, unsigned i,
                                          bool improved, const MoveParams& m) {
    float* xp = r.x + c;
    float* vp = r.v + c;
    float* pp = r.pbest + c;
    f32x4 x_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xp));
    f32x4 v_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(vp));
    f32x4 p_old = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!improved) p_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(pp));
    f32x4 gb = *reinterpret_cast<const f32x4_a4*>(gbest + c);
    __builtin_amdgcn_sched_barrier(0);  // all four loads are issued before anything below

    // The random words need nothing from memory: compute them while the loads
    // are in flight.  The empty asm ties the loaded values to the last random
    // words, which keeps the compiler from moving any use of them (and the
    // wait that goes with it) in front of the Philox rounds.
    const uint32_t pair = (uint32_t)((d0 + (unsigned long long)c) >> 1);
    const Words4 ra = philox4x32_10(pair, i, m.step_lo, m.step_hi, m.key0, m.key1);
    const Words4 rb = philox4x32_10(pair + 1u, i, m.step_lo, m.step_hi, m.key0, m.key1);
    asm volatile("" : "+v"(x_old), "+v"(v_old), "+v"(p_old), "+v"(gb) : "v"(ra.s0), "v"(rb.s0));

    const f32x4 pv = improved ? x_old : p_old;
    float xs[4] = {x_old.x, x_old.y, x_old.z, x_old.w};
    float vs[4] = {v_old.x, v_old.y, v_old.z, v_old.w};
    move_element(xs[0], vs[0], pv.x, gb.x, ra.s0, ra.s1, m);
    move_element(xs[1], vs[1], pv.y, gb.y, ra.s2, ra.s3, m);
    move_element(xs[2], vs[2], pv.z, gb.z, rb.s0, rb.s1, m);
    move_element(xs[3], vs[3], pv.w, gb.w, rb.s2, rb.s3, m);
    __builtin_nontemporal_store(f32x4{xs[0], xs[1], xs[2], xs[3]}, reinterpret_cast<f32x4*>(xp));
    __builtin_nontemporal_store(f32x4{vs[0], vs[1], vs[2], vs[3]}, reinterpret_cast<f32x4*>(vp));
    if (improved) __builtin_nontemporal_store(x_old, reinterpret_cast<f32x4*>(pp));
}

// One row x one tile.  VEC: x, v, pbest of the row are congruent modulo 16
// bytes and (d0 + element address of x) is even, so that an address-aligned
// group of four floats is two whole Philox pairs; tiles are then aligned to the
// address of the row.  Otherwise tiles start at column 0 and everything is
// element-wise.
template <int BLOCK, bool VEC>
__device__ __forceinline__ void update_tile(const RowPtrs& r, const float* __restrict__ gbest,
                                            long long n, unsigned long long d0, unsigned i,
                                            unsigned tile, bool improved, const MoveParams& m) {
    constexpr unsigned TILE = BLOCK * 4;
    long long phase = 0;
    if (VEC) phase = (long long)((reinterpret_cast<uintptr_t>(r.x) >> 2) & (TILE - 1u));
    const long long c = (long long)tile * TILE - phase + 4 * (long long)threadIdx.x;
    if (c + 4 <= 0 || c >= n) return;
    if (VEC && c >= 0 && c + 4 <= n) {
        move_quad(r, gbest, d0, c, i, improved, m);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long long col = c + e;
            if (col >= 0 && col < n) move_single(r, gbest, d0, col, i, improved, m);
        }
    }
}

// Update pass over stacked [K, ld] arrays.  gbest_loss (may be null) is the
// caller's historical-gBest loss: the selection kernel only reads it, and the
// value that belongs to this stage is stored here, after that kernel is done.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_kernel(ColumnBlock b, int K,
                                                       const Selection* __restrict__ sel,
                                                       MoveParams m, TileOrder ord,
                                                       float* gbest_loss) {
    if (gbest_loss && blockIdx.x == 0 && threadIdx.x == 0) *gbest_loss = sel->gbest_loss;
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)K, blockIdx.x, &i, &tile)) return;
    const long long row = (long long)i * b.ld;
    const RowPtrs r{b.x + row, b.v + row, b.pbest + row};
    update_tile<BLOCK, VEC>(r, b.gbest, b.n, b.d0, i, tile, is_improved(sel, (int)i), m);
}

// Update pass over `rows` separate particle arrays, particles row0 .. row0+rows-1.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_rows_kernel(RowTable tab, const float* gbest,
                                                            long long n, int row0, int rows,
                                                            const Selection* __restrict__ sel,
                                                            MoveParams m, TileOrder ord) {
    unsigned i, tile;
    if (!decode_tile_order(ord, (unsigned)rows, blockIdx.x, &i, &tile)) return;
    const RowPtrs r{tab.x[i], tab.v[i], tab.pbest[i]};
    const unsigned particle = (unsigned)row0 + i;
    update_tile<BLOCK, VEC>(r, gbest, n, 0ull, particle, tile, is_improved(sel, (int)particle), m);
}

// The entry of the segment that workgroup `wg` belongs to (entries are sorted
// by their first workgroup).  The table is a kernel argument: the index is
// uniform, so the entry is fetched with scalar loads from the argument segment.
template <bool COPY>
__device__ __forceinline__ const SegEntry& segment_of(const SegTable& tab, unsigned wg) {
    int idx = 0;
#pragma unroll
    for (int s = 1; s < kTableSegs; ++s) {
        const unsigned first = COPY ? tab.first_copy_wg[s] : tab.first_update_wg[s];
        if (s < tab.count && wg >= first) idx = s;
    }
    return tab.seg[idx];
}

// Update pass over up to kTableSegs ragged segments in one launch.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void update_segments_kernel(SegTable tab, int K,
                                                                const Selection* __restrict__ sel,
                                                                MoveParams m) {
    const SegEntry& e = segment_of<false>(tab, blockIdx.x);
    unsigned i, tile;
    if (!decode_tile_order(e.ord, (unsigned)K, blockIdx.x - e.first_update_wg, &i, &tile)) return;
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
                                            int* g_out) {
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
                if (improved) pbest_loss[i] = l;
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

// Selection and gbest copy.  With do_select every wavefront finds g on its own;
// wavefront 0 of workgroup 0 also does the pBest test and publishes g, the
// improved mask and whether gbest is replaced.  Nobody but that wavefront
// touches pbest_loss or the scratch, and nobody in this launch reads what it
// writes, so there is no ordering problem.  Without do_select, g and the
// replace flag are read from the scratch (later segments / row groups).
//
// gbest_loss == null: gbest = x_g always (Algorithm 3).  Otherwise historical
// gBest: gbest = x_g only if this stage's lowest loss is strictly below
// *gbest_loss, which this kernel only reads.
//
// In row-pointer mode a launch carries some of the rows by value and copies
// only if g is one of them.
template <int BLOCK, class Source>
__global__ __launch_bounds__(BLOCK) void select_gbest_kernel(int K, const float* __restrict__ loss,
                                                             float* pbest_loss, Selection* sel,
                                                             Source source,
                                                             float* __restrict__ gbest, long long n,
                                                             const float* gbest_loss,
                                                             int do_select) {
    int g;
    bool replace;
    if (do_select) {
        const bool publisher = blockIdx.x == 0 && threadIdx.x < 64;
        float best;
        wave_argmin(K, loss, pbest_loss, sel, publisher, &best, &g);
        const float kept = gbest_loss ? *gbest_loss : 0.0f;
        replace = gbest_loss ? (best < kept) : true;
        if (publisher && (threadIdx.x & 63) == 0) {
            sel->g = g;
            sel->replaced = replace ? 1 : 0;
            sel->gbest_loss = replace ? best : kept;
        }
    } else {
        g = sel->g;
        replace = sel->replaced != 0;
    }
    if (!replace) return;
    const float* src = source.row(g);
    if (!src) return;
    const long long c = ((long long)blockIdx.x * BLOCK + threadIdx.x) * 4;
    if (c >= n) return;
    if (c + 4 <= n) {
        *reinterpret_cast<f32x4_a4*>(gbest + c) = *reinterpret_cast<const f32x4_a4*>(src + c);
    } else {
        for (long long e = c; e < n; ++e) gbest[e] = src[e];
    }
}

// Selection (if do_select) and the gbest copies of up to kTableSegs segments.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void select_gbest_segments_kernel(
    int K, const float* __restrict__ loss, float* pbest_loss, Selection* sel, SegTable tab,
    int do_select) {
    int g;
    if (do_select) {
        const bool publisher = blockIdx.x == 0 && threadIdx.x < 64;
        float best;
        wave_argmin(K, loss, pbest_loss, sel, publisher, &best, &g);
        if (publisher && (threadIdx.x & 63) == 0) {
            sel->g = g;
            sel->replaced = 1;
            sel->gbest_loss = best;
        }
    } else {
        g = sel->g;
    }
    const SegEntry& e = segment_of<true>(tab, blockIdx.x);
    const long long c = ((long long)(blockIdx.x - e.first_copy_wg) * BLOCK + threadIdx.x) * 4;
    if (c >= e.n) return;
    const float* src = e.x + (long long)g * e.n;
    if (c + 4 <= e.n) {
        *reinterpret_cast<f32x4_a4*>(e.gbest + c) = *reinterpret_cast<const f32x4_a4*>(src + c);
    } else {
        for (long long k = c; k < e.n; ++k) e.gbest[k] = src[k];
    }
}

// Parameter averaging (Section II-B, step 5) on the stacked layout, first half:
// one thread owns four columns, sums the K rows in order and divides by K.
// Reading K rows at one column is tolerant of the rows' different alignments.
// Column tiles are dealt to the XCDs in chunks like those of the update pass
// (`ord` is an order for a single row of column tiles).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void mean_kernel(const float* __restrict__ x,
                                                     float* __restrict__ mean, long long ld,
                                                     long long n, int K, TileOrder ord) {
    unsigned row, tile;
    if (!decode_tile_order(ord, 1u, blockIdx.x, &row, &tile)) return;
    const long long c = ((long long)tile * BLOCK + threadIdx.x) * 4;
    if (c >= n) return;
    const float kf = (float)K;
    if (c + 4 <= n) {
        f32x4 sum = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(x + c));
        for (int k = 1; k < K; ++k)
            sum = sum + __builtin_nontemporal_load(
                            reinterpret_cast<const f32x4_a4*>(x + (long long)k * ld + c));
        *reinterpret_cast<f32x4_a4*>(mean + c) =
            f32x4{sum.x / kf, sum.y / kf, sum.z / kf, sum.w / kf};
    } else {
        for (long long e = c; e < n; ++e) {
            float sum = x[e];
            for (int k = 1; k < K; ++k) sum = sum + x[(long long)k * ld + e];
            mean[e] = sum / kf;
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
    bool eight_xcds;       // 256 compute units: the chip is driven as one device of 8 XCDs
    int last_hip_error;
};

namespace {

// Defaults from a sweep on MI355X with K = 32, D = 25.6 M (tile = 2 KiB):
constexpr int kDefaultBlock = 128;
constexpr unsigned kDefaultSuperBytes = 2u << 20;    // gbest footprint per XCD, in its 4 MiB L2
constexpr unsigned kDefaultChunkBytes = 256u << 10;  // consecutive addresses handed to one XCD
constexpr int kCopyBlock = 256;                      // select_gbest_kernel, average_kernel
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

// Can one row take the 128-bit path?  x, v, pbest congruent modulo 16 bytes and
// (element address of x + flat index of its first column) even.
bool row_vector_ok(const float* x, const float* v, const float* pbest, unsigned long long d0) {
    const uintptr_t ax = reinterpret_cast<uintptr_t>(x);
    const uintptr_t av = reinterpret_cast<uintptr_t>(v);
    const uintptr_t ap = reinterpret_cast<uintptr_t>(pbest);
    if (((ax ^ av) & 15u) || ((ax ^ ap) & 15u)) return false;
    return (((ax >> 2) + d0) & 1ull) == 0;
}

bool block_vector_ok(const pso_ps_ctx* h, const ColumnBlock& b) {
    if (h->force_generic) return false;
    if (h->K > 1 && (b.ld & 1)) return false;
    return row_vector_ok(b.x, b.v, b.pbest, b.d0);
}

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

// Tiles per row: with the vector path tiles are aligned to each row's address.
template <class RowX>
unsigned long long tiles_per_row(int rows, long long n, bool vec, unsigned tile, RowX row_x) {
    unsigned long long max_phase = 0;
    if (vec) {
        for (int i = 0; i < rows; ++i) {
            const unsigned long long a = (reinterpret_cast<uintptr_t>(row_x(i)) >> 2) & (tile - 1u);
            if (a > max_phase) max_phase = a;
        }
    }
    return (max_phase + (unsigned long long)n + tile - 1) / tile;
}

template <int BLOCK>
hipError_t launch_update(const pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, bool vec,
                         float* gbest_loss, hipStream_t stream) {
    TileOrder ord;
    unsigned long long grid = 0;
    const unsigned long long tiles = tiles_per_row(
        h->K, b.n, vec, BLOCK * 4u, [&](int i) { return b.x + (long long)i * b.ld; });
    if (!plan_order(h, h->K, tiles, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((update_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, (const Selection*)h->sel, m, ord, gbest_loss);
    else
        hipLaunchKernelGGL((update_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, b, h->K, (const Selection*)h->sel, m, ord, gbest_loss);
    return hipGetLastError();
}

template <int BLOCK>
hipError_t launch_update_rows(const pso_ps_ctx* h, const RowTable& tab, const float* gbest,
                              int row0, int rows, const MoveParams& m, bool vec,
                              hipStream_t stream) {
    TileOrder ord;
    unsigned long long grid = 0;
    const long long n = (long long)h->D;
    const unsigned long long tiles =
        tiles_per_row(rows, n, vec, BLOCK * 4u, [&](int i) { return tab.x[i]; });
    if (!plan_order(h, rows, tiles, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    const unsigned lds = occupancy_cap_lds(h, BLOCK);
    if (vec)
        hipLaunchKernelGGL((update_rows_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, tab, gbest, n, row0, rows, (const Selection*)h->sel, m, ord);
    else
        hipLaunchKernelGGL((update_rows_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), lds,
                           stream, tab, gbest, n, row0, rows, (const Selection*)h->sel, m, ord);
    return hipGetLastError();
}

#define PSO_PS_DISPATCH_BLOCK(h, e, CALL)                              \
    switch ((h)->block_threads ? (h)->block_threads : kDefaultBlock) { \
        case 64: e = CALL(64); break;                                  \
        case 128: e = CALL(128); break;                                \
        case 256: e = CALL(256); break;                                \
        case 512: e = CALL(512); break;                                \
        case 1024: e = CALL(1024); break;                              \
        default: return PSO_PS_EINVAL;                                 \
    }

// Enqueue the update pass over one dense block (already validated).
int enqueue_update(pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, float* gbest_loss,
                   hipStream_t stream) {
    if (b.n == 0) return PSO_PS_OK;
    const bool vec = block_vector_ok(h, b);
    hipError_t e;
#define CALL(B) launch_update<B>(h, b, m, vec, gbest_loss, stream)
    PSO_PS_DISPATCH_BLOCK(h, e, CALL)
#undef CALL
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

int enqueue_update_rows(pso_ps_ctx* h, const RowTable& tab, const float* gbest, int row0, int rows,
                        const MoveParams& m, hipStream_t stream) {
    bool vec = !h->force_generic;
    for (int i = 0; i < rows && vec; ++i) vec = row_vector_ok(tab.x[i], tab.v[i], tab.pbest[i], 0);
    hipError_t e;
#define CALL(B) launch_update_rows<B>(h, tab, gbest, row0, rows, m, vec, stream)
    PSO_PS_DISPATCH_BLOCK(h, e, CALL)
#undef CALL
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

// Enqueue selection (if do_select) and the gbest copy from `source`.
template <class Source>
int enqueue_select_gbest(pso_ps_ctx* h, float* pbest_loss, const float* loss, const Source& source,
                         float* gbest, long long n, const float* gbest_loss, bool do_select,
                         hipStream_t stream) {
    if (n == 0 && !do_select) return PSO_PS_OK;
    long long blocks = (n + 4LL * kCopyBlock - 1) / (4LL * kCopyBlock);
    if (blocks < 1) blocks = 1;  // selection still has to run
    if (blocks > 0x7fffffffLL) return hip_fail(h, hipErrorInvalidConfiguration);
    hipLaunchKernelGGL((select_gbest_kernel<kCopyBlock, Source>), dim3((unsigned)blocks),
                       dim3(kCopyBlock), 0, stream, h->K, loss, pbest_loss, h->sel, source, gbest,
                       n, gbest_loss, do_select ? 1 : 0);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    if (do_select) h->have_selection = true;
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

// Whole flat stage; gbest_loss == null: best of this stage, else historical gBest.
int sync_flat(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss, const float* loss,
              float* gbest, float* gbest_loss, const MoveParams& m, hipStream_t stream) {
    if (!h || !pbest_loss || !loss) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4) || !aligned_to(gbest_loss, 4))
        return PSO_PS_EALIGN;
    ColumnBlock b{x, v, pbest, gbest, (long long)h->ld, (long long)h->D, 0ull};
    int rc = check_block(b);
    if (rc != PSO_PS_OK) return rc;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    rc = enqueue_select_gbest(h, pbest_loss, loss, StackedSource{x, b.ld}, gbest, b.n, gbest_loss,
                              true, stream);
    if (rc != PSO_PS_OK) return rc;
    return enqueue_update(h, b, m, gbest_loss, stream);
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
    h->force_generic = false; h->eight_xcds = true; h->last_hip_error = 0;

    DeviceScope scope(device);
    hipError_t e = scope.err;
    int compute_units = 0;
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&compute_units, hipDeviceAttributeMultiprocessorCount, device);
    h->eight_xcds = compute_units == 256;
    if (e == hipSuccess) e = hipMalloc((void**)&h->sel, h->sel_bytes);
    if (e == hipSuccess) e = hipMemset(h->sel, 0, h->sel_bytes);
    if (e != hipSuccess) {
        if (h->sel) (void)hipFree(h->sel);
        delete h;
        (void)hipGetLastError();
        return PSO_PS_EHIP;
    }
    *out = h;
    return PSO_PS_OK;
}

int pso_ps_select(pso_ps_ctx* h, const float* x, float* pbest_loss, const float* loss,
                  float* gbest, void* hip_stream) {
    if (!h || !x || !pbest_loss || !loss || !gbest) return PSO_PS_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(pbest_loss, 4) || !aligned_to(loss, 4) ||
        !aligned_to(gbest, 4))
        return PSO_PS_EALIGN;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    return enqueue_select_gbest(h, pbest_loss, loss, StackedSource{x, (long long)h->ld}, gbest,
                                (long long)h->D, nullptr, true, (hipStream_t)hip_stream);
}

int pso_ps_update(pso_ps_ctx* h, float* x, float* v, float* pbest, const float* gbest,
                  float w, float c1, float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !h->have_selection) return PSO_PS_EINVAL;
    ColumnBlock b{x, v, pbest, const_cast<float*>(gbest), (long long)h->ld, (long long)h->D, 0ull};
    const int rc = check_block(b);
    if (rc != PSO_PS_OK) return rc;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const int rc2 = enqueue_update(h, b, make_params(w, c1, c2, seed, step), nullptr,
                                   (hipStream_t)hip_stream);
    if (rc2 == PSO_PS_OK) h->last_stream = (hipStream_t)hip_stream;
    return rc2;
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

int pso_ps_sync_segments(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                         float* const* pbest_seg, float* pbest_loss, const float* loss,
                         float* const* gbest_seg, float w, float c1, float c2,
                         uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !x_seg || !v_seg || !pbest_seg || !gbest_seg || !pbest_loss || !loss)
        return PSO_PS_EINVAL;
    if (h->seg_sizes.empty()) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4)) return PSO_PS_EALIGN;
    const int n_seg = (int)h->seg_sizes.size();
    // Validate every segment before anything is enqueued.  The work lists were
    // reserved at create: no allocation happens here.
    std::vector<ColumnBlock>& blocks = h->seg_blocks;
    std::vector<SegTable>& tables = h->seg_tables;
    std::vector<unsigned>& update_totals = h->seg_update_wgs;
    std::vector<unsigned>& copy_totals = h->seg_copy_wgs;
    blocks.clear(); tables.clear(); update_totals.clear(); copy_totals.clear();
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
    const hipStream_t stream = (hipStream_t)hip_stream;
    const MoveParams m = make_params(w, c1, c2, seed, step);
    const int block = h->block_threads ? h->block_threads : kDefaultBlock;
    // Up to kTableSegs segments per launch; the selection rides on the first
    // gbest-copy launch.  All copies are enqueued before the first update.
    for (size_t first = 0; first < blocks.size(); first += kTableSegs) {
        SegTable tab;
        tab.count = (int)((blocks.size() - first < (size_t)kTableSegs) ? blocks.size() - first
                                                                      : (size_t)kTableSegs);
        unsigned long long update_wg = 0, copy_wg = 0;
        for (int s = 0; s < kTableSegs; ++s) {
            SegEntry& e = tab.seg[s];
            if (s >= tab.count) {
                e = tab.seg[tab.count - 1];  // never selected: segment_of stops at count
                tab.first_update_wg[s] = 0xffffffffu;
                tab.first_copy_wg[s] = 0xffffffffu;
                continue;
            }
            const ColumnBlock& b = blocks[first + s];
            e.x = b.x; e.v = b.v; e.pbest = b.pbest; e.gbest = b.gbest;
            e.n = b.n; e.d0 = b.d0; e.reserved = 0;
            e.vec = block_vector_ok(h, b) ? 1 : 0;
            const unsigned tile = (unsigned)block * 4u;
            const unsigned long long tiles = tiles_per_row(
                h->K, b.n, e.vec != 0, tile, [&](int i) { return b.x + (long long)i * b.ld; });
            unsigned long long grid = 0;
            if (!plan_order(h, h->K, tiles, tile, &e.ord, &grid))
                return hip_fail(h, hipErrorInvalidConfiguration);
            e.first_update_wg = (unsigned)update_wg;
            e.first_copy_wg = (unsigned)copy_wg;
            tab.first_update_wg[s] = e.first_update_wg;
            tab.first_copy_wg[s] = e.first_copy_wg;
            update_wg += grid;
            copy_wg += (unsigned long long)((b.n + 4LL * kCopyBlock - 1) / (4LL * kCopyBlock));
            if (update_wg >= (1ull << 31) || copy_wg >= (1ull << 31))
                return hip_fail(h, hipErrorInvalidConfiguration);
        }
        tables.push_back(tab);
        update_totals.push_back((unsigned)update_wg);
        copy_totals.push_back((unsigned)copy_wg);
    }
    for (size_t t = 0; t < tables.size(); ++t) {
        hipLaunchKernelGGL(select_gbest_segments_kernel<kCopyBlock>, dim3(copy_totals[t]),
                           dim3(kCopyBlock), 0, stream, h->K, loss, pbest_loss, h->sel, tables[t],
                           t == 0 ? 1 : 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(h, e);
    }
    h->last_stream = stream;
    h->have_selection = true;
    const unsigned seg_lds = occupancy_cap_lds(h, block);
    for (size_t t = 0; t < tables.size(); ++t) {
        switch (block) {
            case 64: hipLaunchKernelGGL(update_segments_kernel<64>, dim3(update_totals[t]), dim3(64), seg_lds, stream, tables[t], h->K, (const Selection*)h->sel, m); break;
            case 128: hipLaunchKernelGGL(update_segments_kernel<128>, dim3(update_totals[t]), dim3(128), seg_lds, stream, tables[t], h->K, (const Selection*)h->sel, m); break;
            case 256: hipLaunchKernelGGL(update_segments_kernel<256>, dim3(update_totals[t]), dim3(256), seg_lds, stream, tables[t], h->K, (const Selection*)h->sel, m); break;
            case 512: hipLaunchKernelGGL(update_segments_kernel<512>, dim3(update_totals[t]), dim3(512), seg_lds, stream, tables[t], h->K, (const Selection*)h->sel, m); break;
            case 1024: hipLaunchKernelGGL(update_segments_kernel<1024>, dim3(update_totals[t]), dim3(1024), seg_lds, stream, tables[t], h->K, (const Selection*)h->sel, m); break;
            default: return PSO_PS_EINVAL;
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(h, e);
    }
    return PSO_PS_OK;
}

int pso_ps_sync_rows(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows,
                     float* const* pbest_rows, float* pbest_loss, const float* loss, float* gbest,
                     float w, float c1, float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !x_rows || !v_rows || !pbest_rows || !pbest_loss || !loss || !gbest)
        return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4)) return PSO_PS_EALIGN;
    for (int i = 0; i < h->K; ++i) {
        const int rc = check_arrays(x_rows[i], v_rows[i], pbest_rows[i], gbest);
        if (rc != PSO_PS_OK) return rc;
    }
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    const long long n = (long long)h->D;
    // gbest copies first (each launch carries up to kTableRows row pointers and
    // copies only if g is among them), then the updates.
    for (int row0 = 0; row0 < h->K; row0 += kTableRows) {
        TableSource src;
        src.row0 = row0;
        src.rows = (h->K - row0 < kTableRows) ? h->K - row0 : kTableRows;
        for (int i = 0; i < kTableRows; ++i) src.x[i] = (i < src.rows) ? x_rows[row0 + i] : nullptr;
        const int rc = enqueue_select_gbest(h, pbest_loss, loss, src, gbest, n, nullptr, row0 == 0,
                                            stream);
        if (rc != PSO_PS_OK) return rc;
    }
    const MoveParams m = make_params(w, c1, c2, seed, step);
    for (int row0 = 0; row0 < h->K; row0 += kTableRows) {
        RowTable tab;
        const int rows = (h->K - row0 < kTableRows) ? h->K - row0 : kTableRows;
        for (int i = 0; i < kTableRows; ++i) {
            tab.x[i] = (i < rows) ? x_rows[row0 + i] : nullptr;
            tab.v[i] = (i < rows) ? v_rows[row0 + i] : nullptr;
            tab.pbest[i] = (i < rows) ? pbest_rows[row0 + i] : nullptr;
        }
        const int rc = enqueue_update_rows(h, tab, gbest, row0, rows, m, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    return PSO_PS_OK;
}

int pso_ps_average(pso_ps_ctx* h, float* x, float* mean, void* hip_stream) {
    if (!h || !x || !mean) return PSO_PS_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(mean, 4)) return PSO_PS_EALIGN;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    const long long n = (long long)h->D;
    const long long ld = (long long)h->ld;
    const long long blocks = (n + 4LL * kCopyBlock - 1) / (4LL * kCopyBlock);
    TileOrder mean_ord;
    unsigned long long mean_grid = 0;
    if (!plan_order(h, 1, (unsigned long long)blocks, kCopyBlock * 4u, &mean_ord, &mean_grid))
        return hip_fail(h, hipErrorInvalidConfiguration);
    hipLaunchKernelGGL(mean_kernel<kCopyBlock>, dim3((unsigned)mean_grid), dim3(kCopyBlock), 0,
                       stream, (const float*)x, mean, ld, n, h->K, mean_ord);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    // Tiles are aligned to each row's own address, so any 4-byte aligned row
    // can take the 128-bit stores.
    const bool vec = !h->force_generic;
    constexpr int BLOCK = kDefaultBlock;
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

int pso_ps_last_hip_error(const pso_ps_ctx* h) { return h ? h->last_hip_error : 0; }

int pso_ps_destroy(pso_ps_ctx* h) {
    if (!h) return PSO_PS_OK;
    int rc = PSO_PS_OK;
    {
        DeviceScope scope(h->device);
        if (h->sel && hipFree(h->sel) != hipSuccess) rc = PSO_PS_EHIP;
    }
    delete h;
    return rc;
}

const char* pso_ps_strerror(int code) {
    switch (code) {
        case PSO_PS_OK: return "ok";
        case PSO_PS_EINVAL: return "invalid argument";
        case PSO_PS_EALIGN: return "array not 4-byte aligned";
        case PSO_PS_EHIP: return "HIP runtime call failed";
        case PSO_PS_ENOMEM: return "host allocation failed";
        default: return "unknown status code";
    }
}

}  // extern "C"
