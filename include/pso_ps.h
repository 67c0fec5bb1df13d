/* pso_ps.h - C ABI of the PSO-PS synchronization step on one AMD GPU.
 *
 * One synchronization stage of "PSO-PS: Parameter Synchronization with
 * Particle Swarm Optimization for Distributed Training of Deep Neural
 * Networks" (Ye, Han, Sun, Lv): the branch of Algorithm 1 taken every `step`
 * iterations.  K workers' weight vectors (the particles, Table I) are stacked
 * as rows of [K, ld] float arrays in device memory, with their training losses
 * (the fitness, Table I).  A stage
 *   1. picks the global best g = argmin_i loss_i              (Algorithm 3),
 *   2. copies gbest = x_g as it is before anybody moves        (Algorithm 3),
 *   3. for each particle with loss_i < pbest_loss_i sets pbest_i = x_i and
 *      pbest_loss_i = loss_i                          (Algorithm 1, pBest test),
 *   4. moves every particle, for every coordinate d,
 *        v_id <- w v_id + c1 r1 (pbest_id - x_id) + c2 r2 (gbest_d - x_id)
 *        x_id <- x_id + v_id                                   (Eq. (6), (7)),
 *      r1, r2 uniform in [0,1) (Table II), independent per (i, d).
 *
 * Naming: x = positions = the paper's weights w_i; v = velocities; `w` here is
 * the inertia weight, the paper's m (Eq. (5) gives its schedule; the caller
 * evaluates it and passes the value); c1, c2 are the effective acceleration
 * coefficients, i.e. already divided by the damping lambda of Eq. (6).
 *
 * Conventions fixed by this interface (the paper leaves them open):
 *   - ties in the argmin go to the lowest index; a NaN loss never wins the
 *     argmin and never improves a personal best; if no loss is below +inf, g = 0;
 *   - gbest is the best of this stage only (no history across stages);
 *   - step 4 uses the personal best after step 3;
 *   - r1, r2 are produced by Philox4x32-10 (Salmon et al., SC'11) with
 *       counter = (lo32(d >> 1), i, lo32(step), hi32(step)), key = (lo32(seed), hi32(seed)),
 *       r1 = (word[2(d&1)] >> 8) * 2^-24, r2 = (word[2(d&1)+1] >> 8) * 2^-24,
 *     where d is the flat coordinate index (for segments: in concatenation
 *     order).  The result therefore depends only on the arguments, never on
 *     row stride, segmentation, launch shape or stream;
 *   - arithmetic is IEEE binary32, round to nearest even, evaluated as
 *       acc = w*v; acc = fma(c1*r1, pbest - x, acc); acc = fma(c2*r2, gbest - x, acc);
 *       v = acc; x = x + acc.
 *
 * Memory: every array argument is DEVICE memory owned by the caller, float32,
 * 4-byte aligned (otherwise PSO_PS_EALIGN).  Any such arrays, row strides and
 * segment starts take the same 128-bit path (accesses are aligned to each
 * row's own address in x; v and pbest are fastest when they are congruent to
 * x modulo 16 bytes); results never depend on alignment.  x, v, pbest,
 * pbest_loss are updated in place; gbest is written; loss is read.  The
 * arrays must not overlap each other.  Padding columns D..ld-1 are neither
 * read nor written.
 *
 * Execution: the calls enqueue work on `hip_stream` (a hipStream_t passed as
 * void*, NULL = the default stream) and return without waiting; nothing is
 * allocated or copied to the host per call.  The handle owns a few KiB of
 * device scratch (g, the improved mask, the ticket counters of the
 * single-launch stage).  Calls on one handle must be
 * issued from one host thread at a time and on one stream at a time (work of
 * two stages on different streams would share the scratch).
 *
 * Errors: every function returns PSO_PS_OK (0) or a negative code; nothing
 * throws or aborts.  On error no work has been enqueued, except that a failed
 * multi-segment call may have enqueued some segments.
 */
#ifndef PSO_PS_H
#define PSO_PS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSO_PS_OK       0
#define PSO_PS_EINVAL  (-1)  /* null pointer, K < 1, D < 1, ld < D, bad segment table, bad handle state */
#define PSO_PS_EALIGN  (-2)  /* an array is not 4-byte aligned */
#define PSO_PS_EHIP    (-3)  /* a HIP runtime call failed; see pso_ps_last_hip_error */
#define PSO_PS_ENOMEM  (-4)  /* host allocation failed */
#define PSO_PS_ELIMIT  (-5)  /* K beyond PSO_PS_STATIC_MAX_K (pso_ps_sync_static) or
                                beyond PSO_PS_SINGLE_LAUNCH_MAX_K (pso_ps_set_single_launch) */

#define PSO_PS_STATIC_MAX_K 4096  /* largest swarm pso_ps_sync_static accepts */
#define PSO_PS_SINGLE_LAUNCH_MAX_K 64  /* largest swarm the single-launch stage takes */
/* K * D up to which pso_ps_sync and pso_ps_sync_history choose the
 * single-launch stage by themselves (for K <= 16) */
#define PSO_PS_SINGLE_LAUNCH_MAX_PARAMS 1000000

typedef struct pso_ps_ctx pso_ps_ctx;

/* Create a handle for a swarm of K particles (Table I: population = number of
 * workers) with D parameters each, on HIP device `device`.
 *   ld        row stride of the flat [K, ld] arrays in elements, >= D.
 *   n_seg, seg_sizes (host)  optional ragged structure (Algorithm 2 clones the
 *             network "including the structure"): n_seg per-layer sizes, each
 *             >= 0, summing to D.  n_seg = 0 / NULL means one flat block.
 * The handle is written to *out.  Allocates the device scratch. */
int pso_ps_create(pso_ps_ctx** out, int K, int64_t D, int64_t ld,
                  int n_seg, const int64_t* seg_sizes, int device);

/* One whole synchronization stage (steps 1-4 above) on flat arrays.
 *   x, v, pbest   device [K, ld], in/out      pbest_loss  device [K], in/out
 *   loss          device [K], in              gbest       device [D], out
 *   w, c1, c2     inertia (paper's m) and effective accelerations
 *   seed, step    select the random numbers; the same pair reproduces them
 * Equivalent to pso_ps_sync_begin followed by pso_ps_sync_finish. */
int pso_ps_sync(pso_ps_ctx* h, float* x, float* v, float* pbest,
                float* pbest_loss, const float* loss, float* gbest,
                float w, float c1, float c2, uint64_t seed, uint64_t step,
                void* hip_stream);

/* The same stage on the ragged layout given at create: x_seg, v_seg,
 * pbest_seg, gbest_seg are HOST arrays of n_seg device pointers; segment s is
 * a dense [K, seg_sizes[s]] array (gbest_seg[s]: [seg_sizes[s]]).  Pointers of
 * empty segments are ignored.  Bitwise the same result as the flat call on
 * the concatenated columns. */
int pso_ps_sync_segments(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                         float* const* pbest_seg, float* pbest_loss, const float* loss,
                         float* const* gbest_seg, float w, float c1, float c2,
                         uint64_t seed, uint64_t step, void* hip_stream);

/* The stage with the historical global best, the reading of the standard PSO
 * framework (Section II-C, step 3: gBest "from the history of all particles"):
 * gbest (device [D]) and gbest_loss (device, 1 float) are in/out and persist
 * across stages; they are replaced by x_g and loss_g only if loss_g is
 * strictly below *gbest_loss (a NaN never replaces).  Start with
 * *gbest_loss = +inf.  Everything else as pso_ps_sync; in a stage that keeps
 * the old gbest, this stage's best particle is pulled towards it too. */
int pso_ps_sync_history(pso_ps_ctx* h, float* x, float* v, float* pbest,
                        float* pbest_loss, const float* loss, float* gbest,
                        float* gbest_loss, float w, float c1, float c2,
                        uint64_t seed, uint64_t step, void* hip_stream);

/* pso_ps_sync_segments with the historical global best (see
 * pso_ps_sync_history): gbest_seg[s] (device [seg_sizes[s]]) and gbest_loss
 * (device, 1 float) are in/out and persist across stages. */
int pso_ps_sync_segments_history(pso_ps_ctx* h, float* const* x_seg, float* const* v_seg,
                                 float* const* pbest_seg, float* pbest_loss, const float* loss,
                                 float* const* gbest_seg, float* gbest_loss, float w, float c1,
                                 float c2, uint64_t seed, uint64_t step, void* hip_stream);

/* The stage on K separate per-worker arrays instead of one stacked buffer: the
 * single-GPU stand-in for Algorithm 3's gather and Algorithm 1's "distribute
 * new weights", with no packing copy.  x_rows, v_rows, pbest_rows are HOST
 * arrays of K device pointers, row i holding D floats; ld of the handle is
 * ignored.  Bitwise the same result as pso_ps_sync on the stacked rows. */
int pso_ps_sync_rows(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows,
                     float* const* pbest_rows, float* pbest_loss, const float* loss,
                     float* gbest, float w, float c1, float c2,
                     uint64_t seed, uint64_t step, void* hip_stream);

/* pso_ps_sync_rows with the historical global best (see pso_ps_sync_history):
 * gbest (device [D]) and gbest_loss (device, 1 float) are in/out and persist. */
int pso_ps_sync_rows_history(pso_ps_ctx* h, float* const* x_rows, float* const* v_rows,
                             float* const* pbest_rows, float* pbest_loss, const float* loss,
                             float* gbest, float* gbest_loss, float w, float c1, float c2,
                             uint64_t seed, uint64_t step, void* hip_stream);

/* pso_ps_sync for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  No
 * handle: the few bytes of selection scratch that pso_ps_create would allocate
 * live in a fixed device array inside the library (about 5 KiB: the selection
 * record for up to PSO_PS_STATIC_MAX_K particles and the ticket counters of
 * the single-launch stage; held by every GPU the library runs on until the
 * process ends), so this call and
 * everything under it allocate and free nothing, on the host or the device.
 *   device        HIP device (0 .. 63) that holds the arrays
 *   K, D, ld      as for pso_ps_create; K <= PSO_PS_STATIC_MAX_K, else
 *                 PSO_PS_ELIMIT and nothing is enqueued
 *   the rest      as for pso_ps_sync; same bits as pso_ps_sync
 * All calls on one GPU share that GPU's array: calls whose work overlaps on
 * one GPU (two streams, two threads) race on it and must be serialized by the
 * caller; back-to-back calls on one stream are fine.  The array keeps the last
 * call's contents; every call rewrites all of it that it reads, and leaves the
 * ticket counters at zero, as it found them.  The stage takes one launch or
 * two as pso_ps_sync does by default (see pso_ps_set_single_launch).  The
 * first call on a device looks up the array's address on that GPU
 * (hipGetSymbolAddress, once per device and process): a caller that captures
 * into a HIP graph makes its first call on the device before the capture. */
int pso_ps_sync_static(int device, int K, int64_t D, int64_t ld, float* x, float* v,
                       float* pbest, float* pbest_loss, const float* loss, float* gbest,
                       float w, float c1, float c2, uint64_t seed, uint64_t step,
                       void* hip_stream);

/* Parameter averaging (Section II-B, step 5), the synchronization PSO-PS
 * replaces, on the same stacked layout: mean[d] = (x[0][d] + ... + x[K-1][d]) / K,
 * summed in that order in binary32, written to `mean` (device [D]) and to
 * every row of x (device [K, ld], in/out). */
int pso_ps_average(pso_ps_ctx* h, float* x, float* mean, void* hip_stream);

/* Eq. (5): inertia after t of t_max iterations, falling linearly from m_max to
 * m_min; evaluated in double, rounded to float once.  Host function. */
float pso_ps_inertia(int64_t t, int64_t t_max, float m_max, float m_min);

/* Host-side scalars of iteration t (1-based, as Algorithm 1 counts) of a run
 * of epoch_size epochs with iteration_size iterations each and a stage every
 * `step` iterations: *is_stage = (t % step == 0 and t < Max_t), Max_t =
 * epoch_size * iteration_size; *w = Eq. (5) with t_max = Max_t; *c1_eff =
 * c1 / lambda, *c2_eff = c2 / lambda with lambda = the number (1 .. epoch_size)
 * of the epoch t falls in.  Table II: m_max 0.9, m_min 0.3, c1 0.2, c2 0.9.
 * PSO_PS_EINVAL for t outside 1 .. Max_t or a non-positive size. */
int pso_ps_schedule(int64_t t, int64_t iteration_size, int64_t epoch_size, int64_t step,
                    float m_max, float m_min, float c1, float c2,
                    int* is_stage, float* w, float* c1_eff, float* c2_eff);

/* pso_ps_sync in two calls, split where its two kernel launches meet, for
 * callers that want to time or interleave the halves.  Both take exactly the
 * arguments of pso_ps_sync and must be given the same values, on the same
 * stream, begin first; together they are pso_ps_sync bit for bit.
 *   pso_ps_sync_begin   steps 1 and 2 and the test of step 3 (g, gbest, the
 *                       improved flags; they stay in the handle's scratch),
 *                       and step 4 for the best particle itself, whose
 *                       position before the move is what gbest receives;
 *   pso_ps_sync_finish  pbest_loss_i = loss_i for the improved particles and
 *                       step 4 for the other K-1 particles.
 * (With the copy-based split of pso_ps_set_variant, begin is the selection and
 * the copy gbest = x_g, and finish moves all K particles.)
 * pso_ps_sync_finish without a begin before it on this handle: PSO_PS_EINVAL. */
int pso_ps_sync_begin(pso_ps_ctx* h, float* x, float* v, float* pbest,
                      float* pbest_loss, const float* loss, float* gbest,
                      float w, float c1, float c2, uint64_t seed, uint64_t step,
                      void* hip_stream);
int pso_ps_sync_finish(pso_ps_ctx* h, float* x, float* v, float* pbest,
                       float* pbest_loss, const float* loss, float* gbest,
                       float w, float c1, float c2, uint64_t seed, uint64_t step,
                       void* hip_stream);

/* Read back the last selection: waits for the stream of the last call on this
 * handle, then writes g to *g_out, the improved flags, bit i of word i/64, to
 * improved_mask_out[0..mask_words-1] (host; mask_words >= (K+63)/64), and to
 * *replaced_out whether gbest was (re)written (always 1 without history).
 * Any output may be NULL.  For tests and logging, not for the hot path. */
int pso_ps_last_selection(pso_ps_ctx* h, int* g_out, uint64_t* improved_mask_out,
                          int mask_words, int* replaced_out);

/* Launch shape of the update kernel, for measurement and tests; results are
 * bitwise independent of all of it.  0 selects the library default.
 *   block_threads  threads per workgroup: 64, 128, 256, 512 or 1024; a tile is
 *                  block_threads*4 consecutive floats of one row
 *   super_tiles    tiles (power of two) that one XCD walks for every row before
 *                  it moves on; bounds the gbest footprint in that XCD's L2
 *   chunk_tiles    longest run of consecutive tiles (power of two <=
 *                  super_tiles) handed to one XCD at a time; what is left of a
 *                  row after whole rounds of such runs is dealt in shorter ones
 *   wgs_per_cu     cap on the update workgroups resident on one compute unit
 *                  (>= 3; 64 and above mean no cap), enforced by reserving LDS
 *                  that the kernel never touches; the default keeps about 20
 *                  wavefronts per compute unit
 *   force_generic  != 0: element-wise path instead of the 128-bit one
 * The gbest copy of a stage has a fixed shape of its own (256 threads, 16 KiB
 * per workgroup) and follows only the chunk and super-chunk sizes, in bytes.
 * All of this concerns the stage in two launches; the single-launch stage that
 * small swarms take (pso_ps_set_single_launch) has one fixed shape. */
int pso_ps_set_launch(pso_ps_ctx* h, int block_threads, int super_tiles, int chunk_tiles,
                      int wgs_per_cu, int force_generic);

/* Which kernels the flat stage uses on this handle, for measurement; results
 * are bitwise the same in every combination.
 *   best_first != 0 (default)  pso_ps_sync, pso_ps_sync_static: the first launch
 *                   does the selection and moves the best particle, writing
 *                   gbest from the values it loads anyway; the second moves
 *                   the other K-1 particles, one workgroup per (particle,
 *                   tile), gbest re-read through the caches.
 *   best_first = 0  the copy-based split: selection + copy gbest = x_g, then
 *                   all K particles.  pso_ps_sync_history always uses it (a
 *                   stage that keeps the old gbest has no best particle to
 *                   move first), and so do the ragged and row-pointer calls.
 *   fused_rows = P  in {1, 2, 3, 4, 6, 8} (0: off, default): a one-wavefront
 *                   selection launch, then a single pass in which one
 *                   workgroup owns a tile of columns for all K particles, keeps
 *                   its piece of gbest on chip and has the loads of P
 *                   particles in flight (block_threads 64, 128 or 256).  Moves
 *                   the fewest bytes and is slower; see the kernel's comment.
 *   chunk_origin    where the runs of chunk_tiles consecutive tiles that an XCD
 *                   is handed start in the copy-based split's update pass:
 *                   0 counted from each row's first tile; 1 at absolute
 *                   multiples of the run size in memory, run j of memory going
 *                   to XCD j mod 8; 2 at absolute multiples of the run size,
 *                   the first run of every row going to XCD 0.
 * The ragged and row-pointer entry points ignore all three, and so does the
 * single-launch stage, except that fused_rows > 0 takes precedence over it. */
int pso_ps_set_variant(pso_ps_ctx* h, int fused_rows, int chunk_origin, int best_first);

/* Whether pso_ps_sync, pso_ps_sync_history, the ragged and the row-pointer
 * calls run the stage (Algorithm 3, Algorithm 1's pBest update, Eq. (6), (7))
 * as ONE kernel launch: a workgroup owns 256 columns of all K particles, one
 * wavefront per particle (with K > 16 a wavefront takes several); the
 * workgroup that finishes its reads of the losses last (found by ticket
 * counters in the handle's scratch) updates pbest_loss.  A stage of a small
 * swarm is bound by its two dependent launches; a large one is faster in two
 * launches, whose access order suits HBM.  Results are bitwise the same.
 *   mode -1 (default)  single launch where it measured faster: K <= 16 (one
 *                      wavefront per particle) and K * D <=
 *                      PSO_PS_SINGLE_LAUNCH_MAX_PARAMS
 *   mode 0             never
 *   mode 1             always; PSO_PS_ELIMIT if K > PSO_PS_SINGLE_LAUNCH_MAX_K
 * The row-pointer calls follow the same setting, and so do the ragged calls
 * when the handle has at most 32 non-empty segments (a workgroup then owns 256
 * columns of one segment); pso_ps_sync_static follows the default.
 * pso_ps_sync_begin / pso_ps_sync_finish and the single-pass variant of
 * pso_ps_set_variant always take two launches. */
int pso_ps_set_single_launch(pso_ps_ctx* h, int mode);

/* hipError_t (as int) of the last failed HIP call on this handle, 0 if none. */
int pso_ps_last_hip_error(const pso_ps_ctx* h);

/* Free the scratch and the handle.  The caller must have synchronized the
 * streams it used with this handle.  NULL is accepted. */
int pso_ps_destroy(pso_ps_ctx* h);

/* Hash of the source files this library was compiled from (stamped in by the
 * build; "unstamped" if it was compiled some other way).  The Python binding
 * refuses, or rebuilds, a library whose stamp differs from the sources next
 * to it.  Host function; the string is static. */
const char* pso_ps_source_hash(void);

/* Static, human-readable text for a status code. */
const char* pso_ps_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PSO_PS_H */
