// PSO-PS synchronization step for gfx950 (MI355X): HIP kernels and the C ABI
// declared in include/pso_ps.h.
//
// Two kernels per stage:
//   select_kernel  one wavefront: g = argmin loss (Algorithm 3), improved_i =
//                  loss_i < pbest_loss_i, pbest_loss update (Algorithm 1).
//   update kernels one streaming pass over [K, D]: gbest = x_g, conditional
//                  pbest copy, Eq. (6) velocity and Eq. (7) position update.
//
// The update pass is bound by HBM traffic, not by arithmetic: per particle
// parameter it must read x and v, write x and v, and either read pbest (not
// improved) or write it (improved; its old value is not needed because
// pbest - x is then exactly zero): 20 bytes, plus 4 bytes per column for gbest.
// Mapping: one thread owns four consecutive columns for ALL K rows.  It loads
// x_g for its columns once, keeps the four gbest values in registers across the
// row loop, and is the only thread that ever touches these columns, so the
// in-place update of row g cannot race with the read of gbest = x_g.  Row g's
// x is not read a second time.  All global accesses of a wavefront are
// contiguous (1 KiB per row and array with 128-bit accesses) and non-temporal:
// every byte is used exactly once.
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
typedef float f32x2 __attribute__((ext_vector_type(2)));

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

// 128-bit access when the address is 16-byte aligned, else two 64-bit ones
// (the address is always 8-byte aligned on this path).  `a16` is uniform.
__device__ __forceinline__ f32x4 load4(const float* p, bool a16) {
    if (a16) return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    const f32x2 lo = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(p));
    const f32x2 hi = __builtin_nontemporal_load(reinterpret_cast<const f32x2*>(p + 2));
    return f32x4{lo.x, lo.y, hi.x, hi.y};
}

__device__ __forceinline__ void store4(float* p, f32x4 t, bool a16) {
    if (a16) {
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
    } else {
        __builtin_nontemporal_store(f32x2{t.x, t.y}, reinterpret_cast<f32x2*>(p));
        __builtin_nontemporal_store(f32x2{t.z, t.w}, reinterpret_cast<f32x2*>(p + 2));
    }
}

__device__ __forceinline__ bool aligned16(const void* p) {
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// All K rows of the (at most two) columns that Philox call `pair` serves: flat
// indices 2*pair and 2*pair+1, where they fall inside the block.  Element-wise
// accesses only; used by the generic kernel and for the ragged last columns of
// the vector kernel.
__device__ void move_pair_all_rows(const ColumnBlock& b, int K, const Selection* __restrict__ sel,
                                   const MoveParams& m, unsigned long long pair, int g) {
    long long col[2];
    bool inside[2];
    float gb[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned long long d = 2ull * pair + (unsigned)j;
        inside[j] = d >= b.d0 && d - b.d0 < (unsigned long long)b.n;
        col[j] = inside[j] ? (long long)(d - b.d0) : 0;
        gb[j] = 0.0f;
        if (inside[j]) {
            gb[j] = b.x[(long long)g * b.ld + col[j]];
            b.gbest[col[j]] = gb[j];
        }
    }
    for (int i = 0; i < K; ++i) {
        const bool improved = is_improved(sel, i);
        const Words4 r = philox4x32_10((uint32_t)pair, (uint32_t)i, m.step_lo, m.step_hi,
                                       m.key0, m.key1);
        const long long row = (long long)i * b.ld;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (!inside[j]) continue;
            const long long at = row + col[j];
            float xv = (i == g) ? gb[j] : b.x[at];
            float vv = b.v[at];
            const float pv = improved ? xv : b.pbest[at];
            if (improved) b.pbest[at] = xv;
            move_element(xv, vv, pv, gb[j], j ? r.s2 : r.s0, j ? r.s3 : r.s1, m);
            b.x[at] = xv;
            b.v[at] = vv;
        }
    }
}

// Generic path: any alignment, any parity of d0, any stride.  One thread per
// Philox call (two columns).
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void update_generic_kernel(ColumnBlock b, int K,
                                                               const Selection* __restrict__ sel,
                                                               MoveParams m,
                                                               unsigned long long n_pairs) {
    const unsigned long long t = (unsigned long long)blockIdx.x * BLOCK + threadIdx.x;
    if (t >= n_pairs) return;
    move_pair_all_rows(b, K, sel, m, (b.d0 >> 1) + t, sel->g);
}

// Vector path.  Requires: d0 even; x, v, pbest row starts and gbest 8-byte
// aligned.  One thread owns columns [4q, 4q+4) of every row.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void update_vec4_kernel(ColumnBlock b, int K,
                                                            const Selection* __restrict__ sel,
                                                            MoveParams m) {
    const long long q = (long long)blockIdx.x * BLOCK + threadIdx.x;
    const long long c = q * 4;
    if (c >= b.n) return;
    const int g = sel->g;
    const unsigned long long pair0 = (b.d0 + (unsigned long long)c) >> 1;
    if (c + 4 > b.n) {  // ragged last columns of the block: 1..3 of them
        move_pair_all_rows(b, K, sel, m, pair0, g);
        if (c + 2 < b.n) move_pair_all_rows(b, K, sel, m, pair0 + 1, g);
        return;
    }

    // gbest = x_g before any move (Algorithm 3); kept in registers for all rows.
    const float* xg_row = b.x + (long long)g * b.ld;
    const f32x4 gb = load4(xg_row + c, aligned16(xg_row));
    store4(b.gbest + c, gb, aligned16(b.gbest));

    const uint32_t pa = (uint32_t)pair0;
    const uint32_t pb = pa + 1u;
    for (int i = 0; i < K; ++i) {
        const bool improved = is_improved(sel, i);
        float* xr = b.x + (long long)i * b.ld;
        float* vr = b.v + (long long)i * b.ld;
        float* pr = b.pbest + (long long)i * b.ld;
        const bool ax = aligned16(xr), av = aligned16(vr), ap = aligned16(pr);

        const f32x4 x_old = (i == g) ? gb : load4(xr + c, ax);
        const f32x4 v_old = load4(vr + c, av);
        // Algorithm 1: an improved particle's personal best becomes its current position.
        const f32x4 pv = improved ? x_old : load4(pr + c, ap);

        const Words4 ra = philox4x32_10(pa, (uint32_t)i, m.step_lo, m.step_hi, m.key0, m.key1);
        const Words4 rb = philox4x32_10(pb, (uint32_t)i, m.step_lo, m.step_hi, m.key0, m.key1);
        float xs[4] = {x_old.x, x_old.y, x_old.z, x_old.w};
        float vs[4] = {v_old.x, v_old.y, v_old.z, v_old.w};
        move_element(xs[0], vs[0], pv.x, gb.x, ra.s0, ra.s1, m);
        move_element(xs[1], vs[1], pv.y, gb.y, ra.s2, ra.s3, m);
        move_element(xs[2], vs[2], pv.z, gb.z, rb.s0, rb.s1, m);
        move_element(xs[3], vs[3], pv.w, gb.w, rb.s2, rb.s3, m);

        store4(xr + c, f32x4{xs[0], xs[1], xs[2], xs[3]}, ax);
        store4(vr + c, f32x4{vs[0], vs[1], vs[2], vs[3]}, av);
        if (improved) store4(pr + c, pv, ap);
    }
}

// Selection: one wavefront.  Lexicographic minimum of (loss, index) with NaN
// read as +inf gives the first argmin (Algorithm 3); the strict "<" against
// pbest_loss gives the improved flags (Algorithm 1).
__global__ __launch_bounds__(64) void select_kernel(int K, const float* __restrict__ loss,
                                                    float* __restrict__ pbest_loss,
                                                    Selection* __restrict__ sel) {
    const int lane = threadIdx.x;
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
            improved = l < pbest_loss[i];  // false if either is NaN
            if (improved) pbest_loss[i] = l;
        }
        const unsigned long long mask = __ballot(improved);
        if (lane == 0) sel->improved[base >> 6] = mask;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float other = __shfl_xor(best, off, 64);
        const int other_i = __shfl_xor(best_i, off, 64);
        if (other < best || (other == best && other_i < best_i)) { best = other; best_i = other_i; }
    }
    if (lane == 0) sel->g = best_i;
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
    int device;
    Selection* sel;        // device
    size_t sel_bytes;
    int mask_words;
    hipStream_t last_stream;
    bool have_selection;
    int block_threads;     // 0 = default
    bool force_generic;
    int last_hip_error;
};

namespace {

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

template <int BLOCK>
hipError_t launch_block(const pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, bool vec,
                        hipStream_t stream) {
    if (vec) {
        const long long quads = (b.n + 3) / 4;
        const long long blocks = (quads + BLOCK - 1) / BLOCK;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL(update_vec4_kernel<BLOCK>, dim3((unsigned)blocks), dim3(BLOCK), 0, stream,
                           b, h->K, (const Selection*)h->sel, m);
    } else {
        const unsigned long long first = b.d0 >> 1;
        const unsigned long long last = (b.d0 + (unsigned long long)b.n - 1) >> 1;
        const unsigned long long pairs = last - first + 1;
        const unsigned long long blocks = (pairs + BLOCK - 1) / BLOCK;
        if (blocks > 0x7fffffffULL) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL(update_generic_kernel<BLOCK>, dim3((unsigned)blocks), dim3(BLOCK), 0,
                           stream, b, h->K, (const Selection*)h->sel, m, pairs);
    }
    return hipGetLastError();
}

// Enqueue the update of one dense block.  Every shape assumption of the
// kernels is checked here.
int enqueue_block(pso_ps_ctx* h, const ColumnBlock& b, const MoveParams& m, hipStream_t stream) {
    if (b.n <= 0) return PSO_PS_OK;
    if (!b.x || !b.v || !b.pbest || !b.gbest) return PSO_PS_EINVAL;
    if (!aligned_to(b.x, 4) || !aligned_to(b.v, 4) || !aligned_to(b.pbest, 4) ||
        !aligned_to(b.gbest, 4))
        return PSO_PS_EALIGN;
    if (b.ld < b.n) return PSO_PS_EINVAL;
    // Philox counter word 0 holds the pair index: flat indices must stay below 2^33.
    if (b.d0 + (unsigned long long)b.n > (1ull << 33)) return PSO_PS_EINVAL;

    const bool rows_even = (h->K == 1) || (b.ld % 2 == 0);
    const bool vec = !h->force_generic && (b.d0 % 2 == 0) && rows_even && aligned_to(b.x, 8) &&
                     aligned_to(b.v, 8) && aligned_to(b.pbest, 8) && aligned_to(b.gbest, 8);
    int block = h->block_threads;
    if (block == 0) block = 256;
    hipError_t e;
    switch (block) {
        case 64: e = launch_block<64>(h, b, m, vec, stream); break;
        case 128: e = launch_block<128>(h, b, m, vec, stream); break;
        case 256: e = launch_block<256>(h, b, m, vec, stream); break;
        case 512: e = launch_block<512>(h, b, m, vec, stream); break;
        case 1024: e = launch_block<1024>(h, b, m, vec, stream); break;
        default: return PSO_PS_EINVAL;
    }
    return e == hipSuccess ? PSO_PS_OK : hip_fail(h, e);
}

MoveParams make_params(float w, float c1, float c2, uint64_t seed, uint64_t step) {
    MoveParams m;
    m.w = w; m.c1 = c1; m.c2 = c2;
    m.key0 = (uint32_t)seed; m.key1 = (uint32_t)(seed >> 32);
    m.step_lo = (uint32_t)step; m.step_hi = (uint32_t)(step >> 32);
    return m;
}

int do_select(pso_ps_ctx* h, float* pbest_loss, const float* loss, hipStream_t stream) {
    if (!pbest_loss || !loss) return PSO_PS_EINVAL;
    if (!aligned_to(pbest_loss, 4) || !aligned_to(loss, 4)) return PSO_PS_EALIGN;
    hipLaunchKernelGGL(select_kernel, dim3(1), dim3(64), 0, stream, h->K, loss, pbest_loss, h->sel);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(h, e);
    h->last_stream = stream;
    h->have_selection = true;
    return PSO_PS_OK;
}

int do_update_flat(pso_ps_ctx* h, float* x, float* v, float* pbest, float* gbest,
                   const MoveParams& m, hipStream_t stream) {
    if (!h->have_selection) return PSO_PS_EINVAL;
    ColumnBlock b{x, v, pbest, gbest, (long long)h->ld, (long long)h->D, 0ull};
    const int rc = enqueue_block(h, b, m, stream);
    if (rc == PSO_PS_OK) h->last_stream = stream;
    return rc;
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
        if (n_seg > 0) h->seg_sizes.assign(seg_sizes, seg_sizes + n_seg);
    } catch (...) {
        delete h;
        return PSO_PS_ENOMEM;
    }
    h->mask_words = (K + 63) / 64;
    h->sel_bytes = sizeof(Selection) + (size_t)(h->mask_words - 1) * sizeof(uint64_t);
    h->sel = nullptr; h->last_stream = nullptr; h->have_selection = false;
    h->block_threads = 0; h->force_generic = false; h->last_hip_error = 0;

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

int pso_ps_select(pso_ps_ctx* h, float* pbest_loss, const float* loss, void* hip_stream) {
    if (!h) return PSO_PS_EINVAL;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    return do_select(h, pbest_loss, loss, (hipStream_t)hip_stream);
}

int pso_ps_update(pso_ps_ctx* h, float* x, float* v, float* pbest, float* gbest,
                  float w, float c1, float c2, uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h) return PSO_PS_EINVAL;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    return do_update_flat(h, x, v, pbest, gbest, make_params(w, c1, c2, seed, step),
                          (hipStream_t)hip_stream);
}

int pso_ps_sync(pso_ps_ctx* h, float* x, float* v, float* pbest, float* pbest_loss,
                const float* loss, float* gbest, float w, float c1, float c2,
                uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !x || !v || !pbest || !gbest || !pbest_loss || !loss) return PSO_PS_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(v, 4) || !aligned_to(pbest, 4) || !aligned_to(gbest, 4) ||
        !aligned_to(pbest_loss, 4) || !aligned_to(loss, 4))
        return PSO_PS_EALIGN;
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    const int rc = do_select(h, pbest_loss, loss, stream);
    if (rc != PSO_PS_OK) return rc;
    return do_update_flat(h, x, v, pbest, gbest, make_params(w, c1, c2, seed, step), stream);
}

int pso_ps_sync_segments(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                         float* const* pbest_seg, float* pbest_loss, const float* loss,
                         float* const* gbest_seg, float w, float c1, float c2,
                         uint64_t seed, uint64_t step, void* hip_stream) {
    if (!h || !x_seg || !v_seg || !pbest_seg || !gbest_seg || !pbest_loss || !loss)
        return PSO_PS_EINVAL;
    if (h->seg_sizes.empty()) return PSO_PS_EINVAL;
    const int n_seg = (int)h->seg_sizes.size();
    // Validate every segment before anything is enqueued.
    for (int s = 0; s < n_seg; ++s) {
        if (h->seg_sizes[s] == 0) continue;
        if (!x_seg[s] || !v_seg[s] || !pbest_seg[s] || !gbest_seg[s]) return PSO_PS_EINVAL;
        if (!aligned_to(x_seg[s], 4) || !aligned_to(v_seg[s], 4) || !aligned_to(pbest_seg[s], 4) ||
            !aligned_to(gbest_seg[s], 4))
            return PSO_PS_EALIGN;
    }
    DeviceScope scope(h->device);
    if (scope.err != hipSuccess) return hip_fail(h, scope.err);
    const hipStream_t stream = (hipStream_t)hip_stream;
    int rc = do_select(h, pbest_loss, loss, stream);
    if (rc != PSO_PS_OK) return rc;
    const MoveParams m = make_params(w, c1, c2, seed, step);
    unsigned long long start = 0;
    for (int s = 0; s < n_seg; ++s) {
        const long long n = (long long)h->seg_sizes[s];
        if (n > 0) {
            ColumnBlock b{x_seg[s], v_seg[s], pbest_seg[s], gbest_seg[s], n, n, start};
            rc = enqueue_block(h, b, m, stream);
            if (rc != PSO_PS_OK) return rc;
        }
        start += (unsigned long long)n;
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

int pso_ps_set_launch(pso_ps_ctx* h, int block_threads, int force_generic) {
    if (!h) return PSO_PS_EINVAL;
    switch (block_threads) {
        case 0: case 64: case 128: case 256: case 512: case 1024: break;
        default: return PSO_PS_EINVAL;
    }
    h->block_threads = block_threads;
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
