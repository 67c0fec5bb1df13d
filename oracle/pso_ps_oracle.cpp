// CPU oracle for the PSO-PS synchronization step.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is the plain, slow, single-threaded
// statement of what one synchronization stage computes, written from the
// paper (Ye, Han, Sun, Lv, "PSO-PS: Parameter Synchronization with Particle
// Swarm Optimization for Distributed Training of Deep Neural Networks").  The
// GPU library is checked against it; the GPU library never calls it, and the
// two share no code, headers, tables or helpers.  Only tests, the smoke check
// and the benchmark's CPU-baseline leg may load it.
//
// Notation.  The paper writes the network weights of worker i as w_i (the
// particle position p_i, Table I) and the inertia weight as m.  Here the
// positions are `x`, the velocities `v`, the inertia `w` (= the paper's m),
// the fitness of particle i is `loss[i]` (Table I: fitness = training loss).
//
// What one stage does (the synchronization branch of Algorithm 1, with
// Algorithm 3 for the global best and Eq. (6), (7) for the move):
//   1. g = argmin_i loss_i                       (Algorithm 3; Table I, gBest)
//   2. gbest = x_g, taken before any particle moves          (Algorithm 3)
//   3. for every particle i: if loss_i < pbest_loss_i then pbest_i = x_i and
//      pbest_loss_i = loss_i                   (Algorithm 1, the pBest test)
//   4. for every particle i and coordinate d:
//        v_id = w v_id + c1 r1 (pbest_id - x_id) + c2 r2 (gbest_d - x_id)
//        x_id = x_id + v_id                                  (Eq. (6), (7))
//      with r1, r2 uniform in [0,1) (Table II: random(0,1)), independent per
//      (particle, coordinate).  The damping lambda of Eq. (6) divides c1 and
//      c2; the caller passes c1/lambda and c2/lambda.
//
// Readings where the paper is silent (each also listed in the design notes):
//   * ties in the argmin go to the lowest index; a NaN loss never wins and
//     never improves a personal best; if no loss is finite g = 0;
//   * the personal-best test is the strict "<" the algorithm prints;
//   * gbest is the best of the current stage only (Algorithm 3 returns the
//     just-gathered parameters of the argmin worker), no history;
//   * the velocity uses the personal best after step 3, so an improved
//     particle has pbest - x == 0 exactly;
//   * the best particle moves like every other one (its gbest - x is 0);
//   * r1, r2 come from the counter-based generator Philox4x32-10 (Salmon,
//     Moraes, Dror, Shaw, SC'11) so that the result does not depend on the
//     order in which particles or coordinates are processed:
//        pair index p = d >> 1, lane j = d & 1   (d = flat coordinate index)
//        out[0..3] = Philox4x32-10(counter = (lo32(p), i, lo32(step), hi32(step)),
//                                  key     = (lo32(seed), hi32(seed)))
//        r1 = (out[2j]   >> 8) * 2^-24,  r2 = (out[2j+1] >> 8) * 2^-24
//   * arithmetic is IEEE binary32, round to nearest even, in this order:
//        dp = pbest - x;  dg = gbest - x;  a1 = c1*r1;  a2 = c2*r2;
//        acc = w*v;  acc = fma(a1, dp, acc);  acc = fma(a2, dg, acc);
//        v = acc;  x = x + acc.
//
// Variants and companions (each pinned by its own CPU tests):
//   * historical gBest (the standard-PSO reading, "gBest from the history of
//     all particles"): gbest and gbest_loss persist across stages and are
//     replaced only when this stage's minimum loss is strictly lower;
//   * the scalar schedule around a stage: Eq. (5) for the inertia, the damping
//     lambda of Eq. (6) read as the current epoch number, Algorithm 1's
//     "t % step == 0" cadence with Max_t = epoch_size * iteration_size;
//   * parameter averaging (Section II-B, step 5: new weights = (1/n) sum of
//     the workers' weights, redistributed to all workers), the method PSO-PS
//     replaces, on the same stacked layout.
//
// Pins (tests marked "not gpu"): identity and fixed-point special cases of
// Eq. (6), (7); first-argmin and strict-"<" properties; exact-zero
// consequences for the best and the improved particles; a K=2, D=8 swarm
// worked in exact rational arithmetic; an independent big-integer Philox and
// AMD's open-source rocRAND Philox engine run on the host; moments of r1, r2;
// a float64 closed form with an error bound; order independence.
// The paper prints no worked numerical example of this step, so no output
// value is pinned against a printed number.
//
// Build: g++ -O2 -ffp-contract=off -shared -fPIC (no fast-math).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace {

// ---- Philox4x32-10, from its published definition --------------------------
// One round maps (c0,c1,c2,c3) under round key (k0,k1) to
//   ( hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0) )
// where hi/lo are the halves of the 64-bit product.  Ten rounds; between
// rounds the key advances by the Weyl constants W0, W1 (mod 2^32).
const uint32_t PHILOX_M0 = 0xD2511F53u;
const uint32_t PHILOX_M1 = 0xCD9E8D57u;
const uint32_t PHILOX_W0 = 0x9E3779B9u;  // floor(2^32 * (sqrt(5)-1)/2)
const uint32_t PHILOX_W1 = 0xBB67AE85u;  // floor(2^32 * (sqrt(3)-1))

void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod0 = (uint64_t)PHILOX_M0 * (uint64_t)c0;
        const uint64_t prod1 = (uint64_t)PHILOX_M1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)prod1;
        const uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += PHILOX_W0;
        k1 += PHILOX_W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// 24 high bits of a word as a binary32 in [0, 1 - 2^-24]; both steps exact.
float unit_interval(uint32_t word) {
    return (float)(word >> 8) * 0x1.0p-24f;
}

// r1, r2 of Eq. (6) for particle i and flat coordinate d at (seed, step).
void draw_r(uint64_t seed, uint64_t step, uint32_t i, uint64_t d, float* r1, float* r2) {
    const uint64_t p = d >> 1;
    const unsigned j = (unsigned)(d & 1u);
    const uint32_t ctr[4] = {(uint32_t)p, i, (uint32_t)step, (uint32_t)(step >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    *r1 = unit_interval(out[2 * j]);
    *r2 = unit_interval(out[2 * j + 1]);
}

// Algorithm 3: index of the minimum training loss, first occurrence.
int argmin_loss(int K, const float* loss) {
    int g = 0;
    float best = std::numeric_limits<float>::infinity();
    for (int i = 0; i < K; ++i) {
        const float key = std::isnan(loss[i]) ? std::numeric_limits<float>::infinity() : loss[i];
        if (key < best) { best = key; g = i; }
    }
    return g;
}

// Steps 2-4 above for one dense block of n consecutive coordinates whose first
// coordinate has flat index d0.  Rows are `ld` elements apart.
void move_block(int K, int64_t n, int64_t ld, uint64_t d0, int g, bool replace_gbest,
                const uint8_t* improved, float* x, float* v, float* pbest, float* gbest,
                float w, float c1, float c2, uint64_t seed, uint64_t step) {
    // gbest = x_g, before any position changes (Algorithm 3).
    if (replace_gbest)
        for (int64_t d = 0; d < n; ++d) gbest[d] = x[(int64_t)g * ld + d];
    // pBest_i = w_i for the particles that improved (Algorithm 1).
    for (int i = 0; i < K; ++i) {
        if (!improved[i]) continue;
        for (int64_t d = 0; d < n; ++d) pbest[(int64_t)i * ld + d] = x[(int64_t)i * ld + d];
    }
    // Eq. (6), (7).
    for (int i = 0; i < K; ++i) {
        float* xi = x + (int64_t)i * ld;
        float* vi = v + (int64_t)i * ld;
        const float* pi = pbest + (int64_t)i * ld;
        for (int64_t d = 0; d < n; ++d) {
            float r1, r2;
            draw_r(seed, step, (uint32_t)i, d0 + (uint64_t)d, &r1, &r2);
            const float dp = pi[d] - xi[d];
            const float dg = gbest[d] - xi[d];
            const float a1 = c1 * r1;
            const float a2 = c2 * r2;
            float acc = w * vi[d];
            acc = std::fmaf(a1, dp, acc);
            acc = std::fmaf(a2, dg, acc);
            vi[d] = acc;
            xi[d] = xi[d] + acc;
        }
    }
}

}  // namespace

extern "C" {

// Raw generator, exported so that tests can pin it on its own.
void pso_ps_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    philox4x32_10(ctr, key, out);
}

// r1, r2 for (seed, step, particle i, flat coordinate d).
void pso_ps_oracle_draw_r(uint64_t seed, uint64_t step, uint32_t i, uint64_t d,
                          float* r1, float* r2) {
    draw_r(seed, step, i, d, r1, r2);
}

// Algorithm 3 on its own.
int pso_ps_oracle_argmin(int K, const float* loss) { return argmin_loss(K, loss); }

// One synchronization stage over n_seg dense blocks (n_seg = 1 and
// seg_sizes[0] = D for a flat swarm).  Block s holds coordinates
// [start_s, start_s + seg_sizes[s]) of every particle as a row-major
// [K, seg_ld[s]] array; start_0 = d0 and start_{s+1} = start_s + seg_sizes[s].
// d0 lets a caller run a window of a larger swarm: the random numbers are
// those of flat coordinates d0, d0+1, ...  All arrays are host memory, updated
// in place.  g_out (1 int) and improved_out (K bytes) may be null.
// Returns 0, or -1 for an invalid argument.
//
// gbest_loss (1 float, in/out) may be null: then gbest is the best of this
// stage only (Algorithm 3).  Otherwise gbest is an input as well, and it and
// *gbest_loss are replaced only if the minimum loss of this stage is strictly
// below *gbest_loss (historical gBest); replaced_out (1 int) reports which.
int pso_ps_oracle_sync(int K, int n_seg, const int64_t* seg_sizes, const int64_t* seg_ld,
                       uint64_t d0,
                       float* const* x_seg, float* const* v_seg, float* const* pbest_seg,
                       float* pbest_loss, const float* loss, float* const* gbest_seg,
                       float* gbest_loss,
                       float w, float c1, float c2, uint64_t seed, uint64_t step,
                       int* g_out, uint8_t* improved_out, int* replaced_out) {
    if (K < 1 || n_seg < 1 || !seg_sizes || !seg_ld || !x_seg || !v_seg || !pbest_seg ||
        !pbest_loss || !loss || !gbest_seg)
        return -1;
    for (int s = 0; s < n_seg; ++s)
        if (seg_sizes[s] < 0 || seg_ld[s] < seg_sizes[s]) return -1;

    const int g = argmin_loss(K, loss);
    bool replace = true;
    if (gbest_loss) {
        replace = loss[g] < *gbest_loss;  // false for NaN on either side
        if (replace) *gbest_loss = loss[g];
    }

    uint8_t* improved = new uint8_t[K];
    for (int i = 0; i < K; ++i) {
        improved[i] = (loss[i] < pbest_loss[i]) ? 1 : 0;  // false when either is NaN
        if (improved[i]) pbest_loss[i] = loss[i];
    }

    uint64_t start = d0;
    for (int s = 0; s < n_seg; ++s) {
        if (seg_sizes[s] > 0)
            move_block(K, seg_sizes[s], seg_ld[s], start, g, replace, improved, x_seg[s], v_seg[s],
                       pbest_seg[s], gbest_seg[s], w, c1, c2, seed, step);
        start += (uint64_t)seg_sizes[s];
    }

    if (g_out) *g_out = g;
    if (improved_out) std::memcpy(improved_out, improved, (size_t)K);
    if (replaced_out) *replaced_out = replace ? 1 : 0;
    delete[] improved;
    return 0;
}

// Eq. (5): inertia after t of t_max iterations, falling linearly from m_max to
// m_min.  Evaluated in double and rounded to float once.
float pso_ps_oracle_inertia(int64_t t, int64_t t_max, float m_max, float m_min) {
    const double m = (double)m_max - (double)t * ((double)m_max - (double)m_min) / (double)t_max;
    return (float)m;
}

// Scalars of iteration t (1-based, as Algorithm 1 counts) for a run of
// epoch_size epochs of iteration_size iterations with a stage every `step`
// iterations: whether t is a stage (t % step == 0 and t < Max_t), the inertia
// of Eq. (5) with t_max = Max_t = epoch_size * iteration_size, and c1, c2
// divided by lambda = the number of the epoch that t falls in (1 .. epoch_size;
// the reading of "range 1 to epoch_size ... as the epoch number increases the
// random variable factor decays").  Returns 0, or -1 for an invalid argument.
int pso_ps_oracle_schedule(int64_t t, int64_t iteration_size, int64_t epoch_size, int64_t step,
                           float m_max, float m_min, float c1, float c2,
                           int* is_stage, float* w, float* c1_eff, float* c2_eff) {
    if (t < 1 || iteration_size < 1 || epoch_size < 1 || step < 1) return -1;
    const int64_t max_t = epoch_size * iteration_size;
    if (t > max_t) return -1;
    const int64_t epoch = (t - 1) / iteration_size + 1;
    const float lambda = (float)epoch;
    *is_stage = (t % step == 0 && t < max_t) ? 1 : 0;
    *w = pso_ps_oracle_inertia(t, max_t, m_max, m_min);
    *c1_eff = c1 / lambda;
    *c2_eff = c2 / lambda;
    return 0;
}

// Parameter averaging, step 5: mean[d] = (x[0][d] + x[1][d] + ... + x[K-1][d]) / K,
// summed in that order in binary32, and every row is overwritten by the mean.
int pso_ps_oracle_average(int K, int64_t n, int64_t ld, float* x, float* mean) {
    if (K < 1 || n < 0 || ld < n || !x || !mean) return -1;
    for (int64_t d = 0; d < n; ++d) {
        float sum = x[d];
        for (int k = 1; k < K; ++k) sum = sum + x[(int64_t)k * ld + d];
        mean[d] = sum / (float)K;
    }
    for (int k = 0; k < K; ++k)
        for (int64_t d = 0; d < n; ++d) x[(int64_t)k * ld + d] = mean[d];
    return 0;
}

}  // extern "C"
