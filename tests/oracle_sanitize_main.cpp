// Small driver that runs the oracle under AddressSanitizer / UBSan on the CPU:
// ragged and odd-sized segments, strided rows, windows, history, averaging.
// Built by tests/test_oracle_sanitized.py together with oracle/pso_ps_oracle.cpp.
#include <cstdint>
#include <cstdio>
#include <vector>

extern "C" int pso_ps_oracle_sync(int K, int n_seg, const int64_t* seg_sizes, const int64_t* seg_ld,
                                  uint64_t d0, float* const* x_seg, float* const* v_seg,
                                  float* const* pbest_seg, float* pbest_loss, const float* loss,
                                  float* const* gbest_seg, float* gbest_loss, float w, float c1,
                                  float c2, uint64_t seed, uint64_t step, int* g_out,
                                  uint8_t* improved_out, int* replaced_out);
extern "C" int pso_ps_oracle_average(int K, int64_t n, int64_t ld, float* x, float* mean);

int main() {
    const int K = 5;
    const std::vector<int64_t> sizes = {7, 0, 64, 1, 131};
    const std::vector<int64_t> lds = {9, 3, 64, 1, 140};   // some rows padded
    std::vector<std::vector<float>> x, v, p, g;
    std::vector<float*> xp, vp, pp, gp;
    for (size_t s = 0; s < sizes.size(); ++s) {
        x.emplace_back((size_t)(K * lds[s]), 0.25f);
        v.emplace_back((size_t)(K * lds[s]), -0.125f);
        p.emplace_back((size_t)(K * lds[s]), 0.5f);
        g.emplace_back((size_t)sizes[s], 0.0f);
    }
    for (size_t s = 0; s < sizes.size(); ++s) {
        xp.push_back(x[s].data()); vp.push_back(v[s].data());
        pp.push_back(p[s].data()); gp.push_back(g[s].data());
    }
    std::vector<float> pbest_loss(K, 1.0f), loss = {0.5f, 2.0f, 0.25f, 1.0f, 0.75f};
    float gbest_loss = 0.3f;
    int gi = -1, replaced = -1;
    std::vector<uint8_t> improved(K);
    for (uint64_t step = 0; step < 3; ++step) {
        if (pso_ps_oracle_sync(K, (int)sizes.size(), sizes.data(), lds.data(), 12345, xp.data(),
                               vp.data(), pp.data(), pbest_loss.data(), loss.data(), gp.data(),
                               step == 1 ? &gbest_loss : nullptr, 0.7f, 1.5f, 1.5f, 99, step, &gi,
                               improved.data(), &replaced) != 0)
            return 1;
    }
    std::vector<float> mean(131);
    if (pso_ps_oracle_average(K, 131, 140, x[4].data(), mean.data()) != 0) return 2;
    std::printf("sanitized oracle run ok (g=%d)\n", gi);
    return gi == 2 ? 0 : 3;
}
