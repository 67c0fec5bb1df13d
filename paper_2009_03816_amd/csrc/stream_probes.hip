// Arithmetic-free streams over the arrays of a swarm, for gfx950 (MI355X):
// what the memory system gives to the access mix of the PSO-PS update pass
// (Eq. (6), (7): read x, v, pbest, write x, v) and to simpler mixes, under the
// launch shapes the update kernel can choose from.  Measurement code: the
// benchmark loads this library to print ceilings next to the kernels' rates;
// nothing of the synchronization stage is computed here and the library of the
// stage never calls it.  C ABI in include/pso_ps_probes.h.
//
// Every kernel is one workgroup = R consecutive rows x one tile of BLOCK * 4 *
// QUADS consecutive floats, 128-bit accesses, tiles aligned to the address of
// each row (so the arrays must be 16-byte aligned with a row stride that is a
// multiple of four floats).  The in-place mix writes back the values it read,
// so the arrays are left as they were.

#include <hip/hip_runtime.h>

#include <cstdint>

#include "pso_ps_probes.h"
#include "tile_order.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct StreamArgs {
    float* x;
    float* v;
    float* p;
    long long ld;
    long long n;
    int rows;          // K
    int rows_per_wg;   // R: a workgroup walks R consecutive rows of its tile
    int chunked;       // 1: XCD-aware order (TileOrder), 0: plain row-major
    int absolute;      // chunked only: chunk borders at absolute addresses, not counted from the row start
    TileOrder ord;
};

template <bool NT>
__device__ __forceinline__ f32x4 ld(const float* p) {
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return *reinterpret_cast<const f32x4*>(p);
}
template <bool NT>
__device__ __forceinline__ void st(float* p, f32x4 q) {
    if (NT) __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(p));
    else *reinterpret_cast<f32x4*>(p) = q;
}

// MIX 0: read x, v, p.  MIX 1: copy x -> v.  MIX 2: read x, v, p, write x, v.
template <int BLOCK, int QUADS, int MIX, bool NTL, bool NTS>
__global__ __launch_bounds__(BLOCK) void stream_kernel(StreamArgs a, float* sink) {
    constexpr unsigned TILE = BLOCK * 4 * QUADS;
    const unsigned groups = (unsigned)((a.rows + a.rows_per_wg - 1) / a.rows_per_wg);
    unsigned grp, tile;
    if (a.chunked) {
        if (!decode_tile_order(a.ord, groups, blockIdx.x, &grp, &tile)) return;
    } else {
        grp = blockIdx.x / a.ord.tiles;
        tile = blockIdx.x - grp * a.ord.tiles;
        if (grp >= groups) return;
    }
    for (int r = 0; r < a.rows_per_wg; ++r) {
        const long long i = (long long)grp * a.rows_per_wg + r;
        if (i >= a.rows) return;
        float* x = a.x + i * a.ld;
        float* v = a.v + i * a.ld;
        float* p = a.p + i * a.ld;
        const long long phase = (long long)((reinterpret_cast<uintptr_t>(x) >> 2) & (TILE - 1u));
        long long t = tile;
        if (a.absolute) {
            // `tile` counts from the last multiple of eight chunks (absolute 2: of
            // one chunk) at or below the row's first tile; tiles before the row's
            // first one do not exist
            const unsigned long long cycle = (a.absolute == 2 ? 1ull : 8ull) << a.ord.chunk_log2;
            t -= (long long)((reinterpret_cast<uintptr_t>(x) / (TILE * 4u)) % cycle);
            if (t < 0) continue;
        }
        const long long c0 = t * TILE - phase + 4 * (long long)threadIdx.x;
        f32x4 xq[QUADS], vq[QUADS], pq[QUADS];
        bool ok[QUADS];
#pragma unroll
        for (int u = 0; u < QUADS; ++u) {
            const long long c = c0 + (long long)u * BLOCK * 4;
            ok[u] = c >= 0 && c + 4 <= a.n;   // the ragged ends of a row are skipped: a probe
            if (!ok[u]) continue;
            xq[u] = ld<NTL>(x + c);
            if (MIX != 1) { vq[u] = ld<NTL>(v + c); pq[u] = ld<NTL>(p + c); }
        }
#pragma unroll
        for (int u = 0; u < QUADS; ++u) {
            const long long c = c0 + (long long)u * BLOCK * 4;
            if (!ok[u]) continue;
            if (MIX == 0) {
                const f32x4 s = xq[u] + vq[u] + pq[u];
                if (s.x == 1.2345e30f && s.y == 6.789e-30f) *sink = s.z;   // keeps the loads alive
            } else if (MIX == 1) {
                st<NTS>(v + c, xq[u]);
            } else {
                // written back unchanged; the compare keeps the pbest load alive
                if (pq[u].x == 1.2345e30f && pq[u].y == 6.789e-30f) *sink = pq[u].z;
                st<NTS>(x + c, xq[u]);
                st<NTS>(v + c, vq[u]);
            }
        }
    }
}

template <int BLOCK, int QUADS, int MIX>
hipError_t launch_nt(int ntl, int nts, dim3 grid, unsigned lds, hipStream_t s, const StreamArgs& a,
                     float* sink) {
    if (ntl && nts) hipLaunchKernelGGL((stream_kernel<BLOCK, QUADS, MIX, true, true>), grid, dim3(BLOCK), lds, s, a, sink);
    else if (ntl) hipLaunchKernelGGL((stream_kernel<BLOCK, QUADS, MIX, true, false>), grid, dim3(BLOCK), lds, s, a, sink);
    else if (nts) hipLaunchKernelGGL((stream_kernel<BLOCK, QUADS, MIX, false, true>), grid, dim3(BLOCK), lds, s, a, sink);
    else hipLaunchKernelGGL((stream_kernel<BLOCK, QUADS, MIX, false, false>), grid, dim3(BLOCK), lds, s, a, sink);
    return hipGetLastError();
}

template <int BLOCK, int QUADS>
hipError_t launch_mix(int mix, int ntl, int nts, dim3 grid, unsigned lds, hipStream_t s,
                      const StreamArgs& a, float* sink) {
    switch (mix) {
        case 0: return launch_nt<BLOCK, QUADS, 0>(ntl, nts, grid, lds, s, a, sink);
        case 1: return launch_nt<BLOCK, QUADS, 1>(ntl, nts, grid, lds, s, a, sink);
        case 2: return launch_nt<BLOCK, QUADS, 2>(ntl, nts, grid, lds, s, a, sink);
        default: return hipErrorInvalidValue;
    }
}

// The in-place mix (read x, v, pbest; write x, v back) with the cache-policy
// bits of the accesses chosen freely: 64 threads, one 128-bit access per thread
// and array, XCD-aware order.  Raw buffer loads and stores carry the bits as
// an immediate (sc0 = 1, nt = 2, sc1 = 16 and their sums); the buffer spans one
// row, so an access outside it would be dropped by the hardware.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int LOADS, int STORES>
__global__ __launch_bounds__(64) void policy_kernel(StreamArgs a, float* sink) {
    constexpr unsigned TILE = 256;
    unsigned row, tile;
    if (!decode_tile_order(a.ord, (unsigned)a.rows, blockIdx.x, &row, &tile)) return;
    float* x = a.x + (long long)row * a.ld;
    float* v = a.v + (long long)row * a.ld;
    float* p = a.p + (long long)row * a.ld;
    const long long phase = (long long)((reinterpret_cast<uintptr_t>(x) >> 2) & (TILE - 1u));
    const long long c = (long long)tile * TILE - phase + 4 * (long long)threadIdx.x;
    if (c < 0 || c + 4 > a.n) return;   // the ragged ends of a row are skipped: a probe
    const unsigned bytes = (unsigned)(a.n * 4);
    const unsigned off = (unsigned)(c * 4);
    constexpr int kRsrcFlags = 0x00020000;   // raw 32-bit data, no swizzle
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(x, 0, bytes, kRsrcFlags);
    __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(v, 0, bytes, kRsrcFlags);
    __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(p, 0, bytes, kRsrcFlags);
    const u32x4 xq = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, LOADS);
    const u32x4 vq = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, LOADS);
    const u32x4 pq = __builtin_amdgcn_raw_buffer_load_b128(rp, off, 0, LOADS);
    if (pq.x == 0x7f123456u && pq.y == 0x7f654321u) *sink = (float)pq.z;   // keeps the load alive
    __builtin_amdgcn_raw_buffer_store_b128(xq, rx, off, 0, STORES);
    __builtin_amdgcn_raw_buffer_store_b128(vq, rv, off, 0, STORES);
}

typedef void (*PolicyKernel)(StreamArgs, float*);
template <int LOADS>
PolicyKernel policy_for_stores(int stores) {
    switch (stores) {
        case 0: return policy_kernel<LOADS, 0>;
        case 1: return policy_kernel<LOADS, 1>;
        case 2: return policy_kernel<LOADS, 2>;
        case 3: return policy_kernel<LOADS, 3>;
        case 16: return policy_kernel<LOADS, 16>;
        case 17: return policy_kernel<LOADS, 17>;
        case 18: return policy_kernel<LOADS, 18>;
        case 19: return policy_kernel<LOADS, 19>;
        default: return nullptr;
    }
}
PolicyKernel policy_for(int loads, int stores) {
    switch (loads) {
        case 0: return policy_for_stores<0>(stores);
        case 1: return policy_for_stores<1>(stores);
        case 2: return policy_for_stores<2>(stores);
        case 3: return policy_for_stores<3>(stores);
        case 16: return policy_for_stores<16>(stores);
        case 17: return policy_for_stores<17>(stores);
        case 18: return policy_for_stores<18>(stores);
        case 19: return policy_for_stores<19>(stores);
        default: return nullptr;
    }
}

}  // namespace

extern "C" int pso_ps_probe_stream(int mix, float* x, float* v, float* pbest, float* sink, int K,
                                   int64_t D, int64_t ld, int block_threads, int quads,
                                   int rows_per_wg, int chunked, int super_tiles, int chunk_tiles,
                                   int wgs_per_cu, int nt_loads, int nt_stores, int absolute_chunks,
                                   void* hip_stream) {
    if (!x || !v || !pbest || !sink || K < 1 || D < 4 || ld < D || rows_per_wg < 1) return -1;
    if (mix < 0 || mix > 2 || (quads != 1 && quads != 2)) return -1;
    if (absolute_chunks < 0 || absolute_chunks > 2) return -1;
    if (block_threads != 64 && block_threads != 128 && block_threads != 256) return -1;
    if (super_tiles < 1 || chunk_tiles < 1 || (super_tiles & (super_tiles - 1)) ||
        (chunk_tiles & (chunk_tiles - 1)))
        return -1;
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(pbest)) & 15u)
        return -2;
    if (K > 1 && (ld & 3)) return -2;
    StreamArgs a{x, v, pbest, (long long)ld, (long long)D, K, rows_per_wg, chunked ? 1 : 0,
                 chunked ? absolute_chunks : 0, {}};
    const unsigned tile = (unsigned)block_threads * 4u * (unsigned)quads;
    unsigned long long max_phase = 0;
    for (int i = 0; i < K; ++i) {
        const unsigned long long ph = (reinterpret_cast<uintptr_t>(x + (long long)i * ld) >> 2) & (tile - 1u);
        if (ph > max_phase) max_phase = ph;
    }
    unsigned long long tiles = (max_phase + (unsigned long long)D + tile - 1) / tile;
    if (a.absolute) {  // room for the row that starts furthest into its cycle of eight chunks
        unsigned long long chunk = 1;
        while (chunk < (unsigned long long)(chunk_tiles < super_tiles ? chunk_tiles : super_tiles)) chunk <<= 1;
        tiles += 8ull * chunk - 1;
    }
    const int groups = (K + rows_per_wg - 1) / rows_per_wg;
    unsigned long long grid = 0;
    if (!plan_tile_order(groups, tiles, (unsigned long long)super_tiles, (unsigned long long)chunk_tiles,
                         &a.ord, &grid))
        return -1;
    if (!chunked) grid = tiles * (unsigned long long)groups;
    if (grid >= (1ull << 31)) return -1;
    unsigned lds = 0;   // untouched LDS reservation: caps the workgroups per compute unit
    if (wgs_per_cu >= 3 && wgs_per_cu < 64) {
        lds = (160u * 1024u / (unsigned)wgs_per_cu) & ~511u;
        if (lds > 64u * 1024u) lds = 64u * 1024u;
    }
    const hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
#define PROBE(B, Q) launch_mix<B, Q>(mix, nt_loads, nt_stores, dim3((unsigned)grid), lds, s, a, sink)
    if (block_threads == 64) e = quads == 1 ? PROBE(64, 1) : PROBE(64, 2);
    else if (block_threads == 128) e = quads == 1 ? PROBE(128, 1) : PROBE(128, 2);
    else e = quads == 1 ? PROBE(256, 1) : PROBE(256, 2);
#undef PROBE
    return e == hipSuccess ? 0 : -3;
}

extern "C" int pso_ps_probe_policy(float* x, float* v, float* pbest, float* sink, int K, int64_t D,
                                   int64_t ld, int super_tiles, int chunk_tiles, int wgs_per_cu,
                                   int load_policy, int store_policy, void* hip_stream) {
    if (!x || !v || !pbest || !sink || K < 1 || D < 4 || ld < D) return -1;
    if ((uint64_t)D * 4u >= (1ull << 32)) return -1;   // a row must fit one buffer descriptor
    if (super_tiles < 1 || chunk_tiles < 1 || (super_tiles & (super_tiles - 1)) ||
        (chunk_tiles & (chunk_tiles - 1)))
        return -1;
    const PolicyKernel kernel = policy_for(load_policy, store_policy);
    if (!kernel) return -1;
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(pbest)) & 15u)
        return -2;
    if (K > 1 && (ld & 3)) return -2;
    StreamArgs a{x, v, pbest, (long long)ld, (long long)D, K, 1, 1, 0, {}};
    unsigned long long max_phase = 0;
    for (int i = 0; i < K; ++i) {
        const unsigned long long ph = (reinterpret_cast<uintptr_t>(x + (long long)i * ld) >> 2) & 255u;
        if (ph > max_phase) max_phase = ph;
    }
    const unsigned long long tiles = (max_phase + (unsigned long long)D + 255u) / 256u;
    unsigned long long grid = 0;
    if (!plan_tile_order(K, tiles, (unsigned long long)super_tiles, (unsigned long long)chunk_tiles,
                         &a.ord, &grid) || grid >= (1ull << 31))
        return -1;
    unsigned lds = 0;
    if (wgs_per_cu >= 3 && wgs_per_cu < 64) {
        lds = (160u * 1024u / (unsigned)wgs_per_cu) & ~511u;
        if (lds > 64u * 1024u) lds = 64u * 1024u;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(64), lds, (hipStream_t)hip_stream, a, sink);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}
