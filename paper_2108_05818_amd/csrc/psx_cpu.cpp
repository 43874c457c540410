// Adam on the host cores for host-resident chunks (Sec. "Device-aware Operator
// Placement": the element-wise, memory-bound ADAM operators may run on either
// device; running them where the optimizer states live keeps the fp32 states
// off the host link, only fp16 gradients and fp16 parameters cross it).
//
// The arithmetic is the one printed in include/psx.h, in the same order, with
// AVX2 + F16C (or AVX-512 where the host has it): every vector instruction used here is IEEE-correct per lane
// (mul, add, sub, div, sqrt; no fused multiply-add is ever issued), fp16->fp32
// is exact and fp32->fp16 rounds to nearest even, so the results equal the GPU
// kernel's bit for bit.  MXCSR is set to round-to-nearest with denormals kept
// in every worker.
#include <immintrin.h>

#include <condition_variable>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "psx_internal.h"

namespace psx {

bool cpu_adam_supported() {
    return __builtin_cpu_supports("avx2") && __builtin_cpu_supports("f16c");
}

// ------------------------------------------------------------------ worker pool

struct CpuPool {
    std::vector<std::thread> workers;
    std::mutex mu;
    std::condition_variable cv_work, cv_done;
    std::function<void(int)> job;      // called with the worker index
    uint64_t generation = 0;
    int pending = 0;
    bool stop = false;

    explicit CpuPool(int n) {
        for (int i = 0; i < n; i++) workers.emplace_back([this, i] { run(i); });
    }
    ~CpuPool() {
        {
            std::lock_guard<std::mutex> lk(mu);
            stop = true;
        }
        cv_work.notify_all();
        for (auto &t : workers) t.join();
    }
    void run(int idx) {
        _mm_setcsr(0x1F80);            // round to nearest, all exceptions masked, no FTZ, no DAZ
        uint64_t seen = 0;
        for (;;) {
            std::function<void(int)> f;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv_work.wait(lk, [&] { return stop || generation != seen; });
                if (stop) return;
                seen = generation;
                f = job;
            }
            f(idx);
            {
                std::lock_guard<std::mutex> lk(mu);
                if (--pending == 0) cv_done.notify_all();
            }
        }
    }
    // Runs f(worker) on every worker and returns when all are done.
    void parallel(const std::function<void(int)> &f) {
        std::unique_lock<std::mutex> lk(mu);
        job = f;
        pending = (int)workers.size();
        generation++;
        cv_work.notify_all();
        cv_done.wait(lk, [&] { return pending == 0; });
    }
    int size() const { return (int)workers.size(); }
};

CpuPool *cpu_pool_create(int n_threads) { return new CpuPool(n_threads); }
void cpu_pool_destroy(CpuPool *p) { delete p; }
int cpu_pool_size(const CpuPool *p) { return p->size(); }

// ------------------------------------------------------------------ kernels

template <int DM>
__attribute__((target("avx2,f16c"))) static void adam_range_avx2(const uint16_t *g16, uint16_t *p16, float *pp,
                                                                  float *pm, float *pv, size_t n,
                                                                  const AdamScalars &s) {
    const __m256 inv_scale = _mm256_set1_ps(s.inv_scale), beta1 = _mm256_set1_ps(s.beta1),
                 beta2 = _mm256_set1_ps(s.beta2), omb1 = _mm256_set1_ps(s.omb1), omb2 = _mm256_set1_ps(s.omb2),
                 eps = _mm256_set1_ps(s.eps), wd = _mm256_set1_ps(s.wd), decay = _mm256_set1_ps(s.decay),
                 c2 = _mm256_set1_ps(s.c2), step_size = _mm256_set1_ps(s.step_size);
    size_t i = 0;
    alignas(32) uint16_t gbuf[8], hbuf[8];
    alignas(32) float pbuf[8], mbuf[8], vbuf[8];
    while (i < n) {
        const size_t left = n - i;
        const bool full = left >= 8;
        __m128i gh;
        __m256 p, m, v;
        if (full) {
            gh = _mm_loadu_si128(reinterpret_cast<const __m128i *>(g16 + i));
            p = _mm256_loadu_ps(pp + i);
            m = _mm256_loadu_ps(pm + i);
            v = _mm256_loadu_ps(pv + i);
        } else {                       // ragged end: through small buffers, lanes beyond the end compute on zeros
            for (size_t k = 0; k < 8; k++) {
                gbuf[k] = k < left ? g16[i + k] : 0;
                pbuf[k] = k < left ? pp[i + k] : 0.0f;
                mbuf[k] = k < left ? pm[i + k] : 0.0f;
                vbuf[k] = k < left ? pv[i + k] : 0.0f;
            }
            gh = _mm_load_si128(reinterpret_cast<const __m128i *>(gbuf));
            p = _mm256_load_ps(pbuf);
            m = _mm256_load_ps(mbuf);
            v = _mm256_load_ps(vbuf);
        }
        __m256 g = _mm256_mul_ps(_mm256_cvtph_ps(gh), inv_scale);
        if (DM == 1) g = _mm256_add_ps(g, _mm256_mul_ps(wd, p));
        if (DM == 2) p = _mm256_mul_ps(p, decay);
        m = _mm256_add_ps(_mm256_mul_ps(beta1, m), _mm256_mul_ps(omb1, g));
        v = _mm256_add_ps(_mm256_mul_ps(beta2, v), _mm256_mul_ps(_mm256_mul_ps(omb2, g), g));
        const __m256 den = _mm256_add_ps(_mm256_mul_ps(_mm256_sqrt_ps(v), c2), eps);
        p = _mm256_sub_ps(p, _mm256_mul_ps(step_size, _mm256_div_ps(m, den)));
        const __m128i h = _mm256_cvtps_ph(p, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
        if (full) {
            _mm256_storeu_ps(pp + i, p);
            _mm256_storeu_ps(pm + i, m);
            _mm256_storeu_ps(pv + i, v);
            _mm_storeu_si128(reinterpret_cast<__m128i *>(p16 + i), h);
            i += 8;
        } else {
            _mm256_store_ps(pbuf, p);
            _mm256_store_ps(mbuf, m);
            _mm256_store_ps(vbuf, v);
            _mm_store_si128(reinterpret_cast<__m128i *>(hbuf), h);
            for (size_t k = 0; k < left; k++) {
                pp[i + k] = pbuf[k]; pm[i + k] = mbuf[k]; pv[i + k] = vbuf[k]; p16[i + k] = hbuf[k];
            }
            i = n;
        }
    }
}

__attribute__((target("avx2,f16c"))) static void recast_range_avx2(uint16_t *p16, const float *pp, size_t n) {
    size_t i = 0;
    for (; i + 8 <= n; i += 8)
        _mm_storeu_si128(reinterpret_cast<__m128i *>(p16 + i),
                         _mm256_cvtps_ph(_mm256_loadu_ps(pp + i), _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC));
    if (i < n) {
        alignas(32) float pbuf[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        alignas(32) uint16_t hbuf[8];
        for (size_t k = 0; i + k < n; k++) pbuf[k] = pp[i + k];
        _mm_store_si128(reinterpret_cast<__m128i *>(hbuf),
                        _mm256_cvtps_ph(_mm256_load_ps(pbuf), _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC));
        for (size_t k = 0; i + k < n; k++) p16[i + k] = hbuf[k];
    }
}

// The same with 16 lanes where the host has AVX-512 (F + BW + VL); the ragged end uses lane masks.
template <int DM>
__attribute__((target("avx512f,avx512bw,avx512vl"))) static void adam_range_avx512(const uint16_t *g16, uint16_t *p16,
                                                                                  float *pp, float *pm, float *pv,
                                                                                  size_t n, const AdamScalars &s) {
    const __m512 inv_scale = _mm512_set1_ps(s.inv_scale), beta1 = _mm512_set1_ps(s.beta1),
                 beta2 = _mm512_set1_ps(s.beta2), omb1 = _mm512_set1_ps(s.omb1), omb2 = _mm512_set1_ps(s.omb2),
                 eps = _mm512_set1_ps(s.eps), wd = _mm512_set1_ps(s.wd), decay = _mm512_set1_ps(s.decay),
                 c2 = _mm512_set1_ps(s.c2), step_size = _mm512_set1_ps(s.step_size);
    for (size_t i = 0; i < n; i += 16) {
        const size_t left = n - i;
        const __mmask16 k = left >= 16 ? (__mmask16)0xFFFF : (__mmask16)((1u << left) - 1u);
        const __m256i gh = _mm256_maskz_loadu_epi16(k, g16 + i);
        __m512 p = _mm512_maskz_loadu_ps(k, pp + i);
        __m512 m = _mm512_maskz_loadu_ps(k, pm + i);
        __m512 v = _mm512_maskz_loadu_ps(k, pv + i);
        __m512 g = _mm512_mul_ps(_mm512_cvtph_ps(gh), inv_scale);
        if (DM == 1) g = _mm512_add_ps(g, _mm512_mul_ps(wd, p));
        if (DM == 2) p = _mm512_mul_ps(p, decay);
        m = _mm512_add_ps(_mm512_mul_ps(beta1, m), _mm512_mul_ps(omb1, g));
        v = _mm512_add_ps(_mm512_mul_ps(beta2, v), _mm512_mul_ps(_mm512_mul_ps(omb2, g), g));
        const __m512 den = _mm512_add_ps(_mm512_mul_ps(_mm512_sqrt_ps(v), c2), eps);
        p = _mm512_sub_ps(p, _mm512_mul_ps(step_size, _mm512_div_ps(m, den)));
        const __m256i h = _mm512_cvtps_ph(p, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
        _mm512_mask_storeu_ps(pp + i, k, p);
        _mm512_mask_storeu_ps(pm + i, k, m);
        _mm512_mask_storeu_ps(pv + i, k, v);
        _mm256_mask_storeu_epi16(p16 + i, k, h);
    }
}

static bool have_avx512() {
    return __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512vl");
}

template <int DM>
static void adam_range(bool wide, const uint16_t *g16, uint16_t *p16, float *p, float *m, float *v, size_t n,
                       const AdamScalars &s) {
    if (wide) adam_range_avx512<DM>(g16, p16, p, m, v, n, s);
    else adam_range_avx2<DM>(g16, p16, p, m, v, n, s);
}

// One tile, split evenly (in multiples of 16 elements) over the pool.  isa: 0 = widest the host has, 1 = AVX2.
void cpu_adam_tile(CpuPool *pool, const uint16_t *g16, uint16_t *p16, float *p, float *m, float *v, size_t n,
                   const AdamScalars &s, int isa) {
    const bool wide = isa == 0 && have_avx512();
    const int nt = pool->size();
    const size_t per = ((n + nt - 1) / nt + 15) & ~(size_t)15;
    pool->parallel([&](int w) {
        const size_t lo = (size_t)w * per;
        if (lo >= n) return;
        const size_t cnt = n - lo < per ? n - lo : per;
        switch (s.decay_mode) {
            case 0: adam_range<0>(wide, g16 + lo, p16 + lo, p + lo, m + lo, v + lo, cnt, s); break;
            case 1: adam_range<1>(wide, g16 + lo, p16 + lo, p + lo, m + lo, v + lo, cnt, s); break;
            default: adam_range<2>(wide, g16 + lo, p16 + lo, p + lo, m + lo, v + lo, cnt, s); break;
        }
    });
}

void cpu_recast_tile(CpuPool *pool, uint16_t *p16, const float *p, size_t n) {
    const int nt = pool->size();
    const size_t per = ((n + nt - 1) / nt + 15) & ~(size_t)15;
    pool->parallel([&](int w) {
        const size_t lo = (size_t)w * per;
        if (lo >= n) return;
        recast_range_avx2(p16 + lo, p + lo, n - lo < per ? n - lo : per);
    });
}

}  // namespace psx
