// PSO-PS synchronization step for gfx950 (MI355X): HIP kernels and the C ABI
// declared in include/pso_ps.h.
//
// Two kernels per stage:
//   select_gbest_kernel  g = argmin loss (Algorithm 3), improved_i = loss_i <
//                        pbest_loss_i with the pbest_loss update (Algorithm 1),
//                        and the copy gbest = x_g (Algorithm 3's return value).
//   update_kernel        one streaming pass over [K, D]: conditional pbest
//                        copy, Eq. (6) velocity and Eq. (7) position update.
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
//   * the Philox rounds are placed between the loads and their first use.
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

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
// Same, but only promised to be 4-byte aligned (the hardware takes unaligned
// multi-dword global accesses; the compiler picks the instruction).
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// Device scratch owned by a handle.
struct Selection {
    int g;                 // index of the global best particle
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

struct MoveParams {
    float w, c1, c2;            // inertia (paper's m), effective accelerations
    uint32_t key0, key1;        // seed halves  -> Philox key
    uint32_t step_lo, step_hi;  // step halves  -> Philox counter words 2, 3
};

// Workgroup order of the update pass.  Workgroup b belongs to XCD b & 7 and is
// the (b >> 3)-th of that XCD.  An XCD owns the tile chunks m with m % 8 == xcd
// (a chunk is 2^chunk_log2 consecutive tiles), listed as u = 0 .. per_xcd-1.  The
// list is cut into super-chunks of 2^super_log2 entries (the last one may be
// shorter); within a super-chunk the order is row-major: all its tiles for row
// 0, then for row 1, ...
struct TileOrder {
    unsigned tiles;       // tiles per row (address-aligned tiles, first/last partial)
    unsigned per_xcd;     // list length per XCD (multiple of the chunk size)
    unsigned super_log2;
    unsigned chunk_log2;
    unsigned full;        // number of full super-chunks
    unsigned last;        // entries in the last, shorter super-chunk (0 if none)
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
// generic path.  `col` is the column inside the block, `row` the row offset.
__device__ __forceinline__ void move_single(const ColumnBlock& b, long long row, long long col, int i,
                                            bool improved, const MoveParams& m) {
    const unsigned long long d = b.d0 + (unsigned long long)col;
    const Words4 r = philox4x32_10((uint32_t)(d >> 1), (uint32_t)i, m.step_lo, m.step_hi,
                                   m.key0, m.key1);
    const long long at = row + col;
    float xv = b.x[at];
    float vv = b.v[at];
    const float pv = improved ? xv : b.pbest[at];
    if (improved) b.pbest[at] = xv;
    const bool odd = d & 1ull;
    move_element(xv, vv, pv, b.gbest[col], odd ? r.s2 : r.s0, odd ? r.s3 : r.s1, m);
    b.x[at] = xv;
    b.v[at] = vv;
}

// Columns c .. c+3 of row i with 128-bit accesses (the addresses are 16-byte
// aligned in x, v and pbest, and d0 + c is even).  improved (uniform over the
// workgroup): Algorithm 1 replaced this particle's personal best by its
// position, so pbest is written instead of read.
__device__ __forceinline__ void move_quad(const ColumnBlock& b, long long row, long long c,
                                          unsigned i, bool improved, const MoveParams& m) {
    float* xp = b.x + row + c;
    float* vp = b.v + row + c;
    float* pp = b.pbest + row + c;
    f32x4 x_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xp));
    f32x4 v_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(vp));
    f32x4 p_old = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!improved) p_old = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(pp));
    f32x4 gb = *reinterpret_cast<const f32x4_a4*>(b.gbest + c);
    __builtin_amdgcn_sched_barrier(0);  // all four loads are issued before anything below

    // The random words need nothing from memory: compute them while the loads
    // are in flight.  The empty asm ties the loaded values to the last random
    // words, which keeps the compiler from moving any use of them (and the
    // wait that goes with it) in front of the Philox rounds.
    const uint32_t pair = (uint32_t)((b.d0 + (unsigned long long)c) >> 1);
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

// Update pass.  VEC: x, v, pbest are congruent modulo 16 bytes, rows are an even
// number of elements apart and (d0 + element address of x) is even, so that an
// address-aligned group of four floats is two whole Philox pairs.  Otherwise
// (VEC = false) tiles start at column 0 and everything is element-wise.
template <int BLOCK, bool VEC>
__global__ __launch_bounds__(BLOCK) void update_kernel(ColumnBlock b, int K,
                                                       const Selection* __restrict__ sel,
                                                       MoveParams m, TileOrder ord) {
    constexpr unsigned TILE = BLOCK * 4;
    // -- which (row, tile) is this workgroup? ---------------------------------
    const unsigned xcd = blockIdx.x & 7u;
    const unsigned j = blockIdx.x >> 3;
    const unsigned super = 1u << ord.super_log2;
    const unsigned full_span = (ord.full << ord.super_log2) * (unsigned)K;
    unsigned i, u;
    if (j < full_span) {
        const unsigned q = j >> ord.super_log2;        // (super-chunk, row) pair
        const unsigned sc = q / (unsigned)K;
        i = q - sc * (unsigned)K;
        u = (sc << ord.super_log2) + (j & (super - 1u));
    } else {
        const unsigned r = j - full_span;
        i = r / ord.last;
        u = (ord.full << ord.super_log2) + (r - i * ord.last);
    }
    const unsigned chunk_mask = (1u << ord.chunk_log2) - 1u;
    const unsigned t = ((((u >> ord.chunk_log2) << 3) + xcd) << ord.chunk_log2) + (u & chunk_mask);
    if (t >= ord.tiles || i >= (unsigned)K) return;

    // -- which columns? tiles are aligned to the address of the row -----------
    const long long row = (long long)i * b.ld;
    long long phase = 0;
    if (VEC) phase = (long long)((reinterpret_cast<uintptr_t>(b.x + row) >> 2) & (TILE - 1u));
    const long long c = (long long)t * TILE - phase + 4 * (long long)threadIdx.x;
    if (c + 4 <= 0 || c >= b.n) return;
    const bool improved = is_improved(sel, (int)i);

    if (VEC && c >= 0 && c + 4 <= b.n) {
        move_quad(b, row, c, i, improved, m);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long long col = c + e;
            if (col >= 0 && col < b.n) move_single(b, row, col, (int)i, improved, m);
        }
    }
}

// Selection and gbest copy.  With do_select every wavefront finds g on its own
// from the K losses (lexicographic minimum of (loss, index), NaN read as +inf:
// the first argmin of Algorithm 3); wavefront 0 of workgroup 0 also applies the
// strict "<" test of Algorithm 1 against pbest_loss and publishes g and the
// improved mask.  Nobody but that wavefront touches pbest_loss, and nobody
// reads what it writes, so there is no ordering problem inside the launch.
// Without do_select g is read from the handle's scratch.  Then gbest = x_g.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void select_gbest_kernel(int K, const float* __restrict__ loss,
                                                             float* pbest_loss, Selection* sel,
                                                             const float* __restrict__ x,
                                                             float* __restrict__ gbest,
                                                             long long ld, long long n,
                                                             int do_select) {
    int g;
    if (do_select) {
        const int lane = threadIdx.x & 63;
        const bool publisher = blockIdx.x == 0 && threadIdx.x < 64;
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
        g = best_i;
        if (publisher && lane == 0) sel->g = g;
    } else {
        g = sel->g;
    }
    const long long c = ((long long)blockIdx.x * BLOCK + threadIdx.x) * 4;
    if (c >= n) return;
    const float* src = x + (long long)g * ld + c;
    if (c + 4 <= n) {
        *reinterpret_cast<f32x4_a4*>(gbest + c) = *reinterpret_cast<const f32x4_a4*>(src);
    } else {
        for (long long e = 0; c + e < n; ++e) gbest[c + e] = src[e];
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
bool aligned_to(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

unsigned ceil_log2(unsigned long long t) {
    unsigned l = 0;
    while ((1ull << l) < t) ++l;
    return l;
}

}  // namespace

struct pso_ps_ctx {
    int K;
    int64_t D;
    int64_t ld;
    std::vector<int64_t> seg_sizes;  // empty: one flat block
    int device;
    Selection* sel;        // device
    size_t sel_bytes;
    int mask_words;
    hipStream_t last_stream;
    bool have_selection;
    int block_threads;     // 0 = default
    int super_tiles;       // 0 = default; else a power of two
    int chunk_tiles;       // 0 = default; else a power of two <= super_tiles
    bool force_generic;
    int last_hip_error;
};

namespace {

// Defaults from a sweep on MI355X with K = 32, D = 25.6 M (tile = 2 KiB):
constexpr int kDefaultBlock = 128;
constexpr unsigned kDefaultSuperBytes = 2u << 20;    // gbest footprint per XCD, in its 4 MiB L2
constexpr unsigned kDefaultChunkBytes = 256u << 10;  // consecutive addresses handed to one XCD

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

int check_block(const ColumnBlock& b) {
    if (!b.x || !b.v || !b.pbest || !b.gbest) return PSO_PS_EINVAL;
    if (!aligned_to(b.x, 4) || !aligned_to(b.v, 4) || !aligned_to(b.pbest, 4) ||
        !aligned_to(b.gbest, 4))
        return PSO_PS_EALIGN;
    if (b.n < 0 || b.ld < b.n) return PSO_PS_EINVAL;
    // Philox counter word 0 holds the pair index: flat indices must stay below 2^33.
    if (b.d0 + (unsigned long long)b.n > (1ull << 33)) return PSO_PS_EINVAL;
    return PSO_PS_OK;
}

// Can this block take the 128-bit path?  See update_kernel.
bool vector_path_ok(const pso_ps_ctx* h, const ColumnBlock& b) {
    if (h->force_generic) return false;
    const uintptr_t ax = reinterpret_cast<uintptr_t>(b.x);
    const uintptr_t av = reinterpret_cast<uintptr_t>(b.v);
    const uintptr_t ap = reinterpret_cast<uintptr_t>(b.pbest);
    if (((ax ^ av) & 15u) || ((ax ^ ap) & 15u)) return false;
    if (h->K > 1 && (b.ld & 1)) return false;
    return (((ax >> 2) + b.d0) & 1ull) == 0;
}

// Tiles per row and the workgroup order for one block of columns.
// Returns false if the launch would not fit the grid limits.
bool plan_order(const pso_ps_ctx* h, const ColumnBlock& b, bool vec, unsigned tile,
                TileOrder* ord, unsigned long long* grid) {
    unsigned long long max_phase = 0;
    if (vec) {
        for (int i = 0; i < h->K; ++i) {
            const unsigned long long a =
                (reinterpret_cast<uintptr_t>(b.x + (long long)i * b.ld) >> 2) & (tile - 1u);
            if (a > max_phase) max_phase = a;
        }
    }
    const unsigned long long tiles = (max_phase + (unsigned long long)b.n + tile - 1) / tile;
    // Large blocks: XCD-aware super-chunks.  Small ones: plain row-major order,
    // which is the special case "one super-chunk, chunks of one tile".
    unsigned long long super = h->super_tiles ? (unsigned long long)h->super_tiles
                                              : kDefaultSuperBytes / (tile * 4u);
    unsigned long long chunk = h->chunk_tiles ? (unsigned long long)h->chunk_tiles
                                              : kDefaultChunkBytes / (tile * 4u);
    if (chunk > super) chunk = super;
    if (tiles < 16ull * super) chunk = 1;           // keep all eight XCDs evenly loaded
    const unsigned long long per_xcd = (tiles + 8 * chunk - 1) / (8 * chunk) * chunk;
    if (!h->super_tiles && tiles < 16ull * super) super = 1ull << ceil_log2(per_xcd);
    if (tiles >= (1ull << 31) || per_xcd * 8ull * (unsigned long long)h->K >= (1ull << 31))
        return false;
    ord->tiles = (unsigned)tiles;
    ord->per_xcd = (unsigned)per_xcd;
    ord->super_log2 = ceil_log2(super);
    ord->chunk_log2 = ceil_log2(chunk);
    ord->full = (unsigned)(per_xcd >> ord->super_log2);
    ord->last = (unsigned)(per_xcd - ((unsigned long long)ord->full << ord->super_log2));
    *grid = per_xcd * 8ull * (unsigned long long)h->K;
    return true;
}

template <int BLOCK>
hipError_t launch_update(const pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, bool vec,
                         hipStream_t stream) {
    TileOrder ord;
    unsigned long long grid = 0;
    if (!plan_order(h, b, vec, BLOCK * 4u, &ord, &grid)) return hipErrorInvalidConfiguration;
    if (vec)
        hipLaunchKernelGGL((update_kernel<BLOCK, true>), dim3((unsigned)grid), dim3(BLOCK), 0, stream,
                           b, h->K, (const Selection*)h->sel, m, ord);
    else
        hipLaunchKernelGGL((update_kernel<BLOCK, false>), dim3((unsigned)grid), dim3(BLOCK), 0, stream,
                           b, h->K, (const Selection*)h->sel, m, ord);
    return hipGetLastError();
}

// Enqueue the update pass over one dense block (already validated).
int enqueue_update(pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, hipStream_t stream) {
    if (b.n == 0) return PSO_PS_OK;
    const bool vec = vector_path_ok(h, b);
    hipError_t e;
    switch (h->block_threads ? h->block_threads : kDefaultBlock) {
        case 64: e = launch_update<64>(h, b, m, vec, stream); break;
        case 128: e = launch_update<128>(h, b, m, vec, stream); break;
        case 256: e = launch_update<256>(h, b, m, vec, stream); break;
        case 512: e = launch_update<512>(h, b, m, vec, stream); break;
        case 1024: e = launch_update<1024>(h, b, m, vec, stream); break;
        default: return PSO_PS_EINVAL;
    }
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

// Enqueue selection (if do_select) and the gbest copy of one dense block.
int enqueue_select_gbest(pso_ps_ctx* h, float* pbest_loss, const float* loss, const ColumnBlock& b,
                         bool do_select, hipStream_t stream) {
    constexpr int BLOCK = 256;
    if (b.n == 0 && !do_select) return PSO_PS_OK;
    long long blocks = (b.n + 4LL * BLOCK - 1) / (4LL * BLOCK);
    if (blocks < 1) blocks = 1;  // selection still has to run
    if (blocks > 0x7fffffffLL) return hip_fail(h, hipErrorInvalidConfiguration);
    hipLaunchKernelGGL(select_gbest_kernel<BLOCK>, dim3((unsigned)blocks), dim3(BLOCK), 0, stream,
                       h->K, loss, pbest_loss, h->sel, (const float*)b.x, b.gbest,
                       b.ld, b.n, do_select ? 1 : 0);
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
        if (n_seg > 0) h->seg_sizes.assign(seg_sizes, seg_sizes + n_seg);
    } catch (...) {
        delete h;
        return PSO_PS_ENOMEM;
    }
    h->mask_words = (K + 63) / 64;
    h->sel_bytes = sizeof(Selection) + (size_t)(h->mask_words - 1) * sizeof(uint64_t);
    h->sel = nullptr; h->last_stream = nullptr; h->have_selection = false;
    h->block_threads = 0; h->super_tiles = 0; h->chunk_tiles = 0;
    h->force_generic = false; h->last_hip_error = 0;

    DeviceScope scope(device);
    hipError_t e = scope.err;
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
    ColumnBlock b{const_cast<float*>(x), nullptr, nullptr, gbest, (long long)h->ld, (long long)h->D, 0ull};
    return enqueue_select_gbest(h, pbest_loss, loss, b, true, (hipStream_t)hip_stream);
}

int pso_ps_update(pso_ps_ctx* h, float* x, float* v, float* pbest, const float* gbest,
                  float w, float c1, float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !h->have_selection) return PSO_PS_EINVAL;
    ColumnBlock b{x, v, pbest, const_cast<float*>(gbest), (long long)h->ld, (long long)h->D, 0ull};
    const int rc = check_block(b);
    if (rc != PSO_PS_OK) return rc;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const int rc2 = enqueue_update(h, b, make_params(w, c1, c2, seed, step), (hipStream_t)hip_stream);
    if (rc2 == PSO_PS_OK) h->last_stream = (hipStream_t)hip_stream;
    return rc2;
}

int pso_ps_sync(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                const float* loss, float* gbest, float w, float c1, float c2,
                uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !pbest_loss || !loss) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4)) return PSO_PS_EALIGN;
    ColumnBlock b{x, v, pbest, gbest, (long long)h->ld, (long long)h->D, 0ull};
    int rc = check_block(b);
    if (rc != PSO_PS_OK) return rc;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    rc = enqueue_select_gbest(h, pbest_loss, loss, b, true, stream);
    if (rc != PSO_PS_OK) return rc;
    return enqueue_update(h, b, make_params(w, c1, c2, seed, step), stream);
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
    // Validate every segment before anything is enqueued.
    std::vector<ColumnBlock> blocks;
    try {
        blocks.reserve((size_t)n_seg);
    } catch (...) {
        return PSO_PS_ENOMEM;
    }
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
    // Selection rides on the first segment's gbest copy; every gbest copy is
    // enqueued before any update so that all of them see the positions as they
    // were (segments are separate arrays, so this is only for clarity).
    for (size_t s = 0; s < blocks.size(); ++s) {
        const int rc = enqueue_select_gbest(h, pbest_loss, loss, blocks[s], s == 0, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    const MoveParams m = make_params(w, c1, c2, seed, step);
    for (size_t s = 0; s < blocks.size(); ++s) {
        const int rc = enqueue_update(h, blocks[s], m, stream);
        if (rc != PSO_PS_OK) return rc;
    }
    return PSO_PS_OK;
}

int pso_ps_last_selection(pso_ps_ctx* h, int* g_out, uint64_t* improved_mask_out, int mask_words) {
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
    if (improved_mask_out)
        for (int j = 0; j < h->mask_words; ++j) improved_mask_out[j] = s->improved[j];
    return PSO_PS_OK;
}

int pso_ps_set_launch(pso_ps_ctx* h, int block_threads, int super_tiles, int chunk_tiles,
                      int force_generic) {
    if (!h) return PSO_PS_EINVAL;
    switch (block_threads) {
        case 0: case 64: case 128: case 256: case 512: case 1024: break;
        default: return PSO_PS_EINVAL;
    }
    if (super_tiles != 0 && (!is_pow2(super_tiles) || super_tiles > (1 << 20))) return PSO_PS_EINVAL;
    if (chunk_tiles != 0 && (!is_pow2(chunk_tiles) || chunk_tiles > (1 << 20))) return PSO_PS_EINVAL;
    h->block_threads = block_threads;
    h->super_tiles = super_tiles;
    h->chunk_tiles = chunk_tiles;
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
