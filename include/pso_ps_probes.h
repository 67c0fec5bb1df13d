/* pso_ps_probes.h - C ABI of the stream probes: arithmetic-free kernels that
 * measure what one AMD GPU's memory system gives to the access mix of the
 * PSO-PS update pass (Eq. (6), (7) of the paper read x, v and pbest of every
 * particle and write x and v back) and to simpler mixes, under the launch
 * shapes the update kernel can choose from.  Measurement only: the benchmark
 * prints these rates as ceilings next to the kernels' own; the library of the
 * synchronization stage never calls this one.
 */
#ifndef PSO_PS_PROBES_H
#define PSO_PS_PROBES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueue one stream over the K rows of D floats (row stride ld) of the device
 * arrays x, v, pbest on hip_stream and return without waiting.
 *   mix          0: read x, v, pbest (3 K D floats read)
 *                1: copy x -> v (K D read, K D written; v is overwritten)
 *                2: read x, v, pbest and write x, v back unchanged (the update
 *                   pass's mix, 3 reads + 2 writes; the arrays keep their values)
 *   sink         device, 1 float; never written in practice (keeps loads alive)
 *   block_threads 64, 128 or 256; quads 1 or 2: 128-bit accesses per thread and
 *                array; a tile is block_threads * 4 * quads floats of one row
 *   rows_per_wg  R >= 1: one workgroup walks R consecutive rows of its tile
 *   chunked      0: workgroup b takes tile b % tiles of row b / tiles;
 *                1: the XCD-aware order of the update pass with super_tiles and
 *                   chunk_tiles (powers of two; used only if chunked)
 *   wgs_per_cu   cap on resident workgroups per compute unit (3..63), by an LDS
 *                reservation that is never touched; other values: no cap
 *   nt_loads, nt_stores  != 0: non-temporal accesses
 *   absolute_chunks  chunked only.  0: the runs of chunk_tiles tiles handed to an
 *                XCD are counted from each row's first tile.  1: they start at
 *                absolute multiples of their size in memory and go to XCD
 *                (address / run size) mod 8, so the same columns of different
 *                rows go to different XCDs.  2: they start at absolute
 *                multiples of their size, but the first run of every row goes
 *                to XCD 0, so the columns of an XCD shift by less than one run
 *                from row to row
 * The arrays must be 16-byte aligned and ld a multiple of 4 (K > 1); the first
 * and last partial 16 bytes of a row are skipped.
 * Returns 0, -1 (bad argument), -2 (alignment) or -3 (launch failed). */
int pso_ps_probe_stream(int mix, float* x, float* v, float* pbest, float* sink, int K,
                        int64_t D, int64_t ld, int block_threads, int quads, int rows_per_wg,
                        int chunked, int super_tiles, int chunk_tiles, int wgs_per_cu,
                        int nt_loads, int nt_stores, int absolute_chunks, void* hip_stream);

/* The in-place mix of pso_ps_probe_stream (mix 2) in its default shape (64
 * threads, one 128-bit access per thread and array, XCD-aware order) with the
 * cache-policy bits of the loads and of the stores chosen freely: 0 none,
 * 1 sc0, 2 nt (what "non-temporal" compiles to), 16 sc1, and the sums 3, 17, 18,
 * 19.  A row must be shorter than 4 GiB.  Same alignment rules and return
 * codes. */
int pso_ps_probe_policy(float* x, float* v, float* pbest, float* sink, int K, int64_t D,
                        int64_t ld, int super_tiles, int chunk_tiles, int wgs_per_cu,
                        int load_policy, int store_policy, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PSO_PS_PROBES_H */
