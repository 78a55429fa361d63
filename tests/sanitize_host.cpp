// Host-only driver run under AddressSanitizer + UBSan by tests/test_sanitizers.py: exercises the
// CPU oracle and the library's host segment-table code on ragged inputs.  Exit code 0 = clean.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "adagc.h"

extern "C" {
typedef struct {
    double lr, beta1, beta2, eps, weight_decay, lambda_rel, ema_beta, lambda_abs;
    int64_t t_start;
    int32_t optimizer, grad_dtype, clip_mode, reserved;
    double z_thres;
} oracle_step_hyper;
int oracle_adagc_step(int64_t n_tensors, const int64_t* numel, float* const* theta, const void* const* grad,
                      float* const* m, float* const* v, uint16_t* const* theta_bf16, float* gamma,
                      const oracle_step_hyper* hp, int64_t step, double* out_norm, double* out_coef,
                      uint8_t* out_clipped);
double oracle_l2_norm(const void* g, int64_t numel, int grad_dtype);
uint16_t oracle_float_to_bf16_rne(float f);
}

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main()
{
    // ---- segment table on a ragged list, with exact-size output arrays
    const int64_t sizes[] = {1, 2, 3, 15, 16, 17, 31, 32, 33, 1000, 1, 64};
    const int64_t n = sizeof(sizes) / sizeof(sizes[0]);
    std::vector<adagc_tensor_desc> descs(n);
    for (int64_t i = 0; i < n; ++i) descs[i] = adagc_tensor_desc{sizes[i], 0, 0};
    for (int64_t chunk : {1, 7, 16, 16384}) {
        std::vector<int64_t> begin(n + 1);
        int64_t total = 0;
        CHECK(adagc_build_segment_table(descs.data(), n, chunk, begin.data(), nullptr, nullptr, 0, &total) == ADAGC_OK);
        std::vector<uint32_t> tensor(total), index(total);
        CHECK(adagc_build_segment_table(descs.data(), n, chunk, begin.data(), tensor.data(), index.data(), total, &total) ==
              ADAGC_OK);
        int64_t covered = 0;
        for (int64_t c = 0; c < total; ++c) {
            const int64_t first = (int64_t)index[c] * chunk, numel = sizes[tensor[c]];
            CHECK(first < numel);
            covered += (numel - first < chunk) ? numel - first : chunk;
        }
        int64_t sum = 0;
        for (int64_t s : sizes) sum += s;
        CHECK(covered == sum && begin[n] == total);
        CHECK(adagc_build_segment_table(descs.data(), n, chunk, begin.data(), tensor.data(), index.data(), total - 1,
                                        &total) == ADAGC_ERR_INVALID_ARG);
    }
    descs[3].numel = 0;
    int64_t total = 0;
    std::vector<int64_t> begin(n + 1);
    CHECK(adagc_build_segment_table(descs.data(), n, 16, begin.data(), nullptr, nullptr, 0, &total) == ADAGC_ERR_INVALID_ARG);

    // ---- visiting order: a permutation for every (parts, run)
    for (int64_t nc : {1, 7, 8, 9, 63, 64, 65, 1000, 4099})
        for (int32_t parts : {1, 2, 3, 4, 8, 16, 5000})
            for (int32_t run : {1, 2, 8, 13}) {
                std::vector<uint32_t> order((size_t)nc, 0xFFFFFFFFu);
                CHECK(adagc_build_visiting_order(nc, parts, run, order.data()) == ADAGC_OK);
                std::vector<char> seen((size_t)nc, 0);
                for (uint32_t c : order) {
                    CHECK(c < (uint32_t)nc && !seen[c]);
                    seen[c] = 1;
                }
            }
    CHECK(adagc_build_visiting_order(0, 2, 8, nullptr) == ADAGC_ERR_INVALID_ARG);

    // ---- oracle: several steps through warm-up, AdaGC, the global modes, AdamW and Lion, fp32 and bf16
    for (int optimizer = 0; optimizer < 2; ++optimizer)
        for (int dtype = 0; dtype < 2; ++dtype)
            for (int mode = 0; mode < 6; ++mode) {
                std::vector<std::vector<float>> theta, m, v, gf;
                std::vector<std::vector<uint16_t>> gb, copy;
                std::vector<float*> p_theta, p_m, p_v;
                std::vector<const void*> p_g;
                std::vector<uint16_t*> p_copy;
                std::vector<int64_t> numel(sizes, sizes + n);
                uint32_t lcg = 12345u + optimizer * 7 + dtype * 3 + mode;
                auto rnd = [&lcg]() { lcg = lcg * 1664525u + 1013904223u; return ((lcg >> 8) / 8388608.0f) - 1.0f; };
                for (int64_t i = 0; i < n; ++i) {
                    theta.emplace_back(sizes[i]); m.emplace_back(sizes[i], 0.f); v.emplace_back(sizes[i], 0.f);
                    gf.emplace_back(sizes[i]); gb.emplace_back(sizes[i]); copy.emplace_back(sizes[i]);
                    for (auto& x : theta.back()) x = 0.02f * rnd();
                }
                for (int64_t i = 0; i < n; ++i) {
                    p_theta.push_back(theta[i].data()); p_m.push_back(m[i].data()); p_v.push_back(v[i].data());
                    p_copy.push_back(copy[i].data());
                    p_g.push_back(dtype ? (const void*)gb[i].data() : (const void*)gf[i].data());
                }
                std::vector<float> gamma(n, 0.f);
                std::vector<double> norm(n), coef(n);
                std::vector<uint8_t> clipped(n);
                oracle_step_hyper hp = {3e-4, 0.9, 0.95, 1e-8, 0.1, 1.04, 0.99, 0.05, 2, optimizer, dtype, mode, 0, 2.0};
                for (int64_t step = 1; step <= 6; ++step) {
                    const float scale = (step == 4) ? 30.f : 1.f;
                    for (int64_t i = 0; i < n; ++i)
                        for (int64_t j = 0; j < sizes[i]; ++j) {
                            gf[i][j] = 0.01f * scale * rnd();
                            gb[i][j] = oracle_float_to_bf16_rne(gf[i][j]);
                        }
                    CHECK(oracle_adagc_step(n, numel.data(), p_theta.data(), p_g.data(), p_m.data(),
                                            optimizer ? nullptr : p_v.data(), p_copy.data(), gamma.data(), &hp, step,
                                            norm.data(), coef.data(), clipped.data()) == 0);
                    for (int64_t i = 0; i < n; ++i) CHECK(std::isfinite(norm[i]) && coef[i] >= 0.0 && coef[i] <= 1.0);
                }
                CHECK(oracle_adagc_step(n, numel.data(), p_theta.data(), p_g.data(), p_m.data(), p_v.data(), nullptr,
                                        gamma.data(), &hp, 0, nullptr, nullptr, nullptr) == -1);
            }
    std::puts("sanitize_host: ok");
    return 0;
}
