// Driver for tests/test_host_sanitizers.py: exercises the host-only parts of the library (layout,
// placement plan, chunk-size search, loss scaler, and the worker pool with the host-core Adam) so
// that AddressSanitizer / UndefinedBehaviorSanitizer / ThreadSanitizer builds of them can be run on
// the CPU.  Results are compared with the scalar oracle where there is one.  Never built for the GPU.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

#include "psx_internal.h"
using namespace psx;

extern "C" {   // the oracle's C interface (oracle/psx_oracle.c)
typedef struct { double lr, beta1, beta2, eps, weight_decay, loss_scale; uint64_t step; uint32_t adamw_mode, reserved; } orc_adam_hyper;
typedef struct { float step_size, c2, inv_scale, beta1, beta2, omb1, omb2, eps, wd, decay; } orc_adam_scalars;
typedef struct { uint32_t chunk, reserved; uint64_t offset, numel; } orc_slot;
void orc_adam_prepare(const orc_adam_hyper *, orc_adam_scalars *);
void orc_adam_chunk(const uint16_t *, uint16_t *, float *, float *, float *, uint64_t, const orc_adam_hyper *);
void orc_recast_chunk(uint16_t *, const float *, uint64_t);
int orc_chunk_layout(const uint64_t *, uint64_t, uint64_t, int, orc_slot *, uint64_t *, uint64_t, uint64_t *);
}

#define CHECK(cond, ...) do { if (!(cond)) { printf(__VA_ARGS__); printf("\n"); return 1; } } while (0)

static int host_calls(std::mt19937_64 &rng, int iters) {
    for (int it = 0; it < iters; it++) {
        const size_t n = rng() % 12;
        const uint64_t C = 1 + rng() % 40;
        std::vector<uint64_t> numel(n);
        for (auto &x : numel) x = rng() % (3 * C);
        size_t nch = 0;
        CHECK(psx_chunk_layout(numel.data(), n, C, 0, nullptr, nullptr, 0, &nch) == PSX_OK, "layout sizing failed");
        std::vector<psx_slot> slots(n + 1);
        std::vector<uint64_t> used(nch);
        CHECK(psx_chunk_layout(numel.data(), n, C, 0, slots.data(), used.data(), nch, &nch) == PSX_OK, "layout failed");
        std::vector<orc_slot> o_slots(n + 1);
        std::vector<uint64_t> o_used(nch);
        uint64_t o_nch = 0;
        CHECK(orc_chunk_layout(numel.data(), n, C, 0, o_slots.data(), o_used.data(), nch, &o_nch) == 0 && o_nch == nch, "oracle layout disagrees on the chunk count");
        for (size_t i = 0; i < n; i++)
            CHECK(slots[i].chunk == o_slots[i].chunk && slots[i].offset == o_slots[i].offset && slots[i].numel == o_slots[i].numel, "slot %zu differs", i);
        CHECK(memcmp(used.data(), o_used.data(), nch * sizeof(uint64_t)) == 0, "used[] differs");
        // an output array that is one entry short must be refused, not overrun
        if (nch > 1) {
            std::vector<uint64_t> small(nch - 1);
            CHECK(psx_chunk_layout(numel.data(), n, C, 0, nullptr, small.data(), nch - 1, &nch) == PSX_ECAP, "short used[] accepted");
        }
        std::vector<uint8_t> loc(nch);
        uint64_t he = 0;
        CHECK(psx_plan_residency(used.data(), nch, C, (rng() % (nch + 2)) * 12 * C, loc.data(), &he) == PSX_OK, "plan failed");
        uint64_t best = 0; double util = 0; size_t bn = 0;
        const int rc = psx_chunk_size_search(numel.data(), n, 1 + rng() % 5, 50, 1 + rng() % 7, rng() % 2, 0, &best, &util, &bn);
        CHECK(rc == PSX_OK || rc == PSX_ETOOLARGE, "search rc %d", rc);
    }
    psx_scaler s{65536.0f, 3, 0, 0, 1};
    for (int i = 0; i < 1000; i++) CHECK(psx_loss_scale_update(&s, (rng() % 7) == 0) == PSX_OK, "scaler");
    CHECK(psx_loss_scale_update(nullptr, 0) == PSX_EINVAL && psx_last_error()[0] != 0, "NULL scaler accepted");
    return 0;
}

static int cpu_adam_against_oracle(std::mt19937_64 &rng) {
    if (!cpu_adam_supported()) { printf("host has no AVX2 + F16C: host-core Adam not exercised\n"); return 0; }
    std::normal_distribution<float> nd(0.f, 1.f);
    int it = 0;
    for (int threads = 1; threads <= 7; threads++) {
        for (int cycle = 0; cycle < 3; cycle++) {                 // create / destroy cycles
            CpuPool *pool = cpu_pool_create(threads);
            CHECK(cpu_pool_size(pool) == threads, "pool size");
            for (int rep = 0; rep < 6; rep++, it++) {             // back-to-back parallel() calls on one pool
                const size_t n = rep == 0 ? 1 : (rep == 1 ? 15 + threads : 1 + rng() % 30000);   // mostly not multiples of 16
                const int dm = it % 3;
                std::vector<uint16_t> g(n), h1(n), h2(n), r1(n), r2(n);
                std::vector<float> p(n), m(n), v(n);
                for (size_t i = 0; i < n; i++) {
                    g[i] = (uint16_t)(rng() & 0xFFFF);
                    if ((g[i] & 0x7C00) == 0x7C00) g[i] &= 0x3FFF;
                    p[i] = nd(rng) * 0.02f; m[i] = nd(rng) * 1e-3f; v[i] = std::fabs(nd(rng)) * 1e-6f;
                }
                auto p2 = p, m2 = m, v2 = v;
                orc_adam_hyper oh{1e-3, 0.9, 0.999, 1e-8, dm ? 0.01 : 0.0, 1024.0, (uint64_t)(1 + it), (uint32_t)(dm == 2), 0};
                orc_adam_scalars os;
                orc_adam_prepare(&oh, &os);
                AdamScalars s{os.step_size, os.c2, os.inv_scale, os.beta1, os.beta2, os.omb1, os.omb2, os.eps, os.wd, os.decay, (uint32_t)dm};
                cpu_adam_tile(pool, g.data(), h1.data(), p.data(), m.data(), v.data(), n, s, it & 1);
                orc_adam_chunk(g.data(), h2.data(), p2.data(), m2.data(), v2.data(), n, &oh);
                CHECK(!memcmp(p.data(), p2.data(), n * 4) && !memcmp(m.data(), m2.data(), n * 4) && !memcmp(v.data(), v2.data(), n * 4) &&
                      !memcmp(h1.data(), h2.data(), n * 2), "host-core Adam differs from the oracle: threads %d n %zu decay mode %d", threads, n, dm);
                cpu_recast_tile(pool, r1.data(), p.data(), n);
                orc_recast_chunk(r2.data(), p2.data(), n);
                CHECK(!memcmp(r1.data(), r2.data(), n * 2), "host-core re-cast differs from the oracle: threads %d n %zu", threads, n);
            }
            cpu_pool_destroy(pool);
        }
    }
    // two pools alive at once, driven from two threads (one context each is the rule; pools must not share state)
    int bad = 0;
    auto drive = [&](int seed) {
        std::mt19937_64 r(seed);
        CpuPool *pool = cpu_pool_create(3);
        for (int rep = 0; rep < 20; rep++) {
            const size_t n = 1 + r() % 5000;
            std::vector<float> p(n, 0.25f);
            std::vector<uint16_t> a(n), b(n);
            cpu_recast_tile(pool, a.data(), p.data(), n);
            orc_recast_chunk(b.data(), p.data(), n);
            if (memcmp(a.data(), b.data(), n * 2)) __atomic_fetch_add(&bad, 1, __ATOMIC_RELAXED);
        }
        cpu_pool_destroy(pool);
    };
    std::thread t1(drive, 1), t2(drive, 2);
    t1.join(); t2.join();
    CHECK(bad == 0, "two pools at once disturbed each other");
    return 0;
}

int main(int argc, char **argv) {
    std::mt19937_64 rng(5);
    const int iters = argc > 1 ? atoi(argv[1]) : 20000;
    if (host_calls(rng, iters)) return 1;
    if (cpu_adam_against_oracle(rng)) return 1;
    printf("host sanitizer driver ok\n");
    return 0;
}
