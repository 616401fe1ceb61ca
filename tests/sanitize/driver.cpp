// Sanitizer build of the CPU code: the oracle (C) and the host side of the library (plan
// construction, queries, argument checks) compiled with -fsanitize=address,undefined and
// driven through their C interfaces on small seeded inputs.  Any out-of-bounds access,
// use after free, leak, signed overflow or misaligned access aborts the run; a handful of
// invariants the paper fixes are checked on the way (Eq. 11's count, sent + residual = v).
// Test infrastructure: built and run by tests/test_sanitizers.py only.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/rsdgc.h"

extern "C" {
int64_t rsdgc_oracle_k(int64_t G, int p, double rho);
int64_t rsdgc_oracle_compress_layer(const float *g, float *r, int64_t R, int64_t C, int p, double alpha,
                                    double rho, uint32_t *idx, float *val, uint32_t *centres,
                                    int64_t *k_out, float *tau_out, float *nsi_out, float *v_out);
int64_t rsdgc_oracle_compress_layer_momentum(const float *g, float *u, float *r, float m, int64_t R,
                                             int64_t C, int p, double alpha, double rho, uint32_t *idx,
                                             float *val, uint32_t *centres, int64_t *k_out,
                                             float *tau_out, float *nsi_out, float *v_out);
int64_t rsdgc_oracle_compress_layer_blocks(const float *g, float *r, int64_t R, int64_t C, int p,
                                           double alpha, double rho, uint32_t *blocks, float *val,
                                           float *tau_out, float *nsi_out, float *v_out);
int64_t rsdgc_oracle_compress_layer_blocks_momentum(const float *g, float *u, float *r, float m, int64_t R,
                                                    int64_t C, int p, double alpha, double rho,
                                                    uint32_t *blocks, float *val, float *tau_out,
                                                    float *nsi_out, float *v_out);
void rsdgc_oracle_decompress(const uint32_t *idx, const float *val, int64_t n, float *dense, int64_t G,
                             int accumulate);
void rsdgc_oracle_decompress_blocks(const uint32_t *blocks, const float *val, int64_t k, int64_t R,
                                    int64_t C, int p, float *dense, int accumulate);
int rsdgc_oracle_apply(float *w, int64_t G, int32_t n_msgs, const uint32_t *const *idx,
                       const float *const *val, const int64_t *n, float eta);
int rsdgc_oracle_dynamic_ratios(const float *w_all, const int64_t *off, int32_t L, double rho,
                                double *ratio_out);
// rsdgc_plan.cpp releases profiling events through this entry point of the HIP side; no events
// exist here
int rsdgc_profile_end(rsdgc_plan_t *, double *, int32_t *) { return RSDGC_OK; }
}

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                        \
        }                                                                        \
    } while (0)

static uint32_t rng_state = 12345u;
static float rnd() {   // small LCG: values in [-1, 1)
    rng_state = rng_state * 1664525u + 1013904223u;
    return static_cast<float>(static_cast<int32_t>(rng_state >> 8) % 20001 - 10000) * 1e-4f;
}

static void oracle_cases() {
    const int shapes[][2] = {{1, 1}, {1, 37}, {5, 2}, {9, 9}, {16, 33}, {40, 70}, {2, 300}};
    const int ps[] = {1, 3, 5, 7};
    const double rhos[] = {0.0, 0.013, 0.3, 1.0};
    for (const auto &sh : shapes)
        for (int p : ps)
            for (double rho : rhos) {
                const int64_t R = sh[0], C = sh[1], G = R * C;
                std::vector<float> g(G), r(G), u(G), r0;
                for (auto &x : g) x = rnd();
                for (auto &x : r) x = 0.5f * rnd();
                for (auto &x : u) x = 0.25f * rnd();
                r0 = r;
                const int64_t k = rsdgc_oracle_k(G, p, rho);
                CHECK(k >= 0 && k <= G && std::fabs(static_cast<double>(k) - std::ceil(double(G) / (p * p) * rho)) < 1.5);
                const int64_t cap = std::min<int64_t>(k * p * p, G);
                std::vector<uint32_t> idx(std::max<int64_t>(cap, 1)), centres(std::max<int64_t>(k, 1));
                std::vector<float> val(std::max<int64_t>(cap, 1)), nsi(G), v(G);
                int64_t k_out = -1;
                float tau = 0.f;
                const int64_t n = rsdgc_oracle_compress_layer(g.data(), r.data(), R, C, p, 0.5, rho, idx.data(),
                                                              val.data(), centres.data(), &k_out, &tau,
                                                              nsi.data(), v.data());
                CHECK(n >= 0 && n <= cap && k_out == k && (k == 0 || n >= k));
                std::vector<float> dense(G, 7.f);
                rsdgc_oracle_decompress(idx.data(), val.data(), n, dense.data(), G, 0);
                for (int64_t i = 0; i < G; ++i) {      // sent + residual = v, bit for bit
                    const float s = dense[i] + r[i];
                    CHECK(std::memcmp(&s, &v[i], 4) == 0 || (s == 0.f && v[i] == 0.f));
                }
                const std::vector<uint32_t> idx0(idx.begin(), idx.begin() + n);
                const std::vector<float> val0(val.begin(), val.begin() + n);
                // momentum form and block form on the same input
                std::vector<float> r2 = r0, u2 = u;
                CHECK(rsdgc_oracle_compress_layer_momentum(g.data(), u2.data(), r2.data(), 0.9f, R, C, p, 0.25, rho,
                                                           idx.data(), val.data(), centres.data(), &k_out, &tau,
                                                           nsi.data(), v.data()) >= 0);
                const int64_t BR = (R + p - 1) / p, BC = (C + p - 1) / p;
                const int64_t kb = std::min<int64_t>(k, BR * BC);
                std::vector<uint32_t> blocks(std::max<int64_t>(kb, 1));
                std::vector<float> bval(std::max<int64_t>(kb * p * p, 1)), bnsi(BR * BC);
                std::vector<float> r3 = r0;
                CHECK(rsdgc_oracle_compress_layer_blocks(g.data(), r3.data(), R, C, p, 0.5, rho, blocks.data(),
                                                         bval.data(), &tau, bnsi.data(), v.data()) == kb);
                rsdgc_oracle_decompress_blocks(blocks.data(), bval.data(), kb, R, C, p, dense.data(), 0);
                std::vector<float> r4 = r0, u4 = u;
                CHECK(rsdgc_oracle_compress_layer_blocks_momentum(g.data(), u4.data(), r4.data(), 0.9f, R, C, p, 0.5,
                                                                  rho, blocks.data(), bval.data(), &tau,
                                                                  bnsi.data(), v.data()) == kb);
                // receiving side: the plain call's message from two nodes
                std::vector<float> w(G, 1.f);
                const uint32_t *ip[2] = {idx0.data(), idx0.data()};
                const float *vp[2] = {val0.data(), val0.data()};
                const int64_t nn[2] = {n, n};
                CHECK(rsdgc_oracle_apply(w.data(), G, 2, ip, vp, nn, 0.1f) == 0);
                for (int64_t j = 0; j < n; ++j) {
                    const float want = 1.f - 0.1f * (val0[j] + val0[j]);
                    CHECK(std::fabs(w[idx0[j]] - want) <= 1e-6f * (1.f + std::fabs(want)));
                }
            }
    // dynamic ratios over three layers
    std::vector<float> wall(60);
    for (auto &x : wall) x = rnd();
    const int64_t off[4] = {0, 10, 35, 60};
    double ratio[3];
    CHECK(rsdgc_oracle_dynamic_ratios(wall.data(), off, 3, 0.2, ratio) == 0);
    const double kept = ratio[0] * 10 + ratio[1] * 25 + ratio[2] * 25;
    CHECK(std::fabs(kept - 12.0) < 1e-9);
}

static void plan_cases() {
    const rsdgc_shape_t shapes[] = {{64, 27}, {512, 4608}, {1, 777}, {4096, 45}, {300, 1000}};
    const double ratios[] = {0.5, 0.02, 0.1, 0.0, 0.06};
    const int32_t pp[] = {3, 3, 1, 5, 7};
    for (int blocks = 0; blocks < 2; ++blocks) {
        rsdgc_plan_t *plan = nullptr;
        const int rc = blocks ? rsdgc_plan_blocks(shapes, 5, 3, pp, 0.5, ratios, &plan)
                              : rsdgc_plan(shapes, 5, 3, pp, 0.5, ratios, &plan);
        CHECK(rc == RSDGC_OK && plan != nullptr);
        CHECK(rsdgc_n_layers(plan) == 5 && rsdgc_layer_k(plan, 3) == 0);
        CHECK(rsdgc_workspace_bytes(plan) % 256 == 0 && rsdgc_total_elems(plan) % 64 == 0);
        int64_t out = 0;
        for (int l = 0; l < 5; ++l) {
            CHECK(rsdgc_out_offset(plan, l) == out);
            const int64_t G = shapes[l].rows * shapes[l].cols, k = rsdgc_layer_k(plan, l);
            out += blocks ? k * pp[l] * pp[l] : std::min<int64_t>(k * pp[l] * pp[l], G);
        }
        CHECK(rsdgc_out_capacity(plan) == out);
        const double more[] = {1.0, 0.3, 1.0, 0.2, 0.001};
        CHECK(rsdgc_plan_set_ratios(plan, more) == RSDGC_OK);
        CHECK(rsdgc_plan_set_work_feed(plan, RSDGC_FEED_ON) == RSDGC_OK);
        if (!blocks) CHECK(rsdgc_plan_set_path(plan, RSDGC_PATH_FULL_MAP) == RSDGC_OK);
        CHECK(rsdgc_plan_forget_workspace(plan) == RSDGC_OK);
        CHECK(rsdgc_layer_k(plan, 5) == -1 && rsdgc_layer_offset(plan, -1) == -1);
        rsdgc_plan_destroy(plan);
    }
    rsdgc_plan_t *plan = nullptr;
    const rsdgc_shape_t bad[] = {{0, 5}};
    const double one[] = {0.1};
    CHECK(rsdgc_plan(bad, 1, 3, nullptr, 0.5, one, &plan) == RSDGC_EINVAL && plan == nullptr);
    CHECK(rsdgc_plan(shapes, 1, 4, nullptr, 0.5, one, &plan) == RSDGC_EINVAL);
    CHECK(rsdgc_plan(shapes, 1, 3, nullptr, 1.5, one, &plan) == RSDGC_EINVAL);
    rsdgc_plan_destroy(nullptr);
}

int main() {
    oracle_cases();
    plan_cases();
    std::puts("sanitized run ok");
    return 0;
}
