// Driver for the sanitizer build of the library's host-only code (host optimizer, strategy search).  Built and run by tests/test_host_sanitizers.py with
// -fsanitize=address,undefined; exits 0 when every call returned what it should and the sanitizers
// stayed silent.  Buffers are allocated at their exact sizes so that any out-of-bounds access of the
// vector paths (ragged tails, unaligned starts, slices cut between threads) is caught.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/autohete.h"

static uint64_t rng_state = 0x1234567;
static uint32_t rnd()
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}

#define REQUIRE(x) do { if (!(x)) { std::printf("FAILED: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main()
{
    autohete_hparams hp = {1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 1.0f, 8.0f};
    for (int dtype = 0; dtype < 2; ++dtype) {
        for (int scalar = 0; scalar < 2; ++scalar) {
            autohete_host_force_scalar(scalar);
            const size_t sizes[] = {1, 2, 7, 8, 9, 15, 16, 17, 31, 33, 1000, 4097, 70001};
            std::vector<std::vector<uint16_t>> g, q;
            std::vector<std::vector<float>> p, m, v;
            std::vector<autohete_chunk> ch;
            for (size_t n : sizes) {
                g.emplace_back(n); q.emplace_back(n); p.emplace_back(n); m.emplace_back(n); v.emplace_back(n);
                for (size_t i = 0; i < n; ++i) {
                    g.back()[i] = (uint16_t)(dtype == AH_BF16 ? 0x3A00 + (rnd() & 0xFF) + ((rnd() & 1) << 15)
                                                              : 0x2000 + (rnd() & 0x3FF) + ((rnd() & 1) << 15));
                    p.back()[i] = 0.02f * ((int)(rnd() % 2001) - 1000) / 1000.0f;
                    m.back()[i] = 1e-4f * ((int)(rnd() % 2001) - 1000) / 1000.0f;
                    v.back()[i] = 1e-6f * (rnd() % 1000) / 1000.0f;
                }
            }
            for (size_t c = 0; c < g.size(); ++c)
                ch.push_back({g[c].data(), q[c].data(), p[c].data(), m[c].data(), v[c].data(), (uint64_t)g[c].size()});
            for (int threads : {1, 2, 5, 16}) {
                double s = 0;
                uint32_t f = 7;
                REQUIRE(autohete_host_grad_sumsq(ch.data(), ch.size(), dtype, 8.0f, threads, &s, &f) == AH_OK);
                REQUIRE(f == 0 && std::isfinite(s) && s > 0);
                REQUIRE(autohete_host_adamw_step(ch.data(), ch.size(), dtype, 3, &hp, s, f, threads) == AH_OK);
                for (auto &vec : p)
                    for (float x : vec) REQUIRE(std::isfinite(x));
            }
            /* gradient and parameter sharing one buffer, as in the pinned staging of the hybrid placement */
            autohete_chunk alias = {g[12].data(), g[12].data(), p[12].data(), m[12].data(), v[12].data(), (uint64_t)g[12].size()};
            REQUIRE(autohete_host_adamw_step(&alias, 1, dtype, 4, &hp, 1.0, 0, 3) == AH_OK);
        }
    }
    autohete_cost_model cm = {6, 100, 10, 50, 5, 5, 6000, 5000, 1, 2, 3, 1, 4, 0.2};
    autohete_strategy best;
    REQUIRE(autohete_strategy_search(&cm, &best) == AH_OK && best.feasible == 1);
    cm.gpu_capacity_bytes = 1;
    REQUIRE(autohete_strategy_search(&cm, &best) == AH_EINFEASIBLE);
    std::printf("sanitizer driver: ok\n");
    return 0;
}
