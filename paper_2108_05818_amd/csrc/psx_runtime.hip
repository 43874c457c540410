// Host runtime behind the C ABI: context, descriptor tables, the multi-tensor
// pack/unpack and overflow-check calls, and the Adam step: one launch over the
// HBM-resident chunks and, for host-resident chunks, a launch that works on the
// pinned buffers over the link, a staged H2D / update / D2H pipeline, or the
// host cores (fp16 tiles copied out and in around an in-place host update).
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "psx_internal.h"

using namespace psx;

namespace {

constexpr int kRing = 4;        // pinned upload buffers per table
constexpr int kCpuSlots = 3;    // tiles in flight of the host-core pipeline

// A descriptor table on the device, with the content last uploaded kept on the
// host so that an unchanged table (the steady state of a training loop) is not
// uploaded again.  Uploads are ordered on the caller's stream, after earlier
// kernels that may still read the table.
struct Table {
    void *dev = nullptr;
    size_t cap = 0;                       // bytes
    std::vector<unsigned char> shadow;    // content on the device (as of the last enqueued upload)
    void *pinned[kRing] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t done[kRing] = {nullptr, nullptr, nullptr, nullptr};
    bool pending[kRing] = {false, false, false, false};
    int next = 0;
};

int32_t table_free(Table &t) {
    for (int i = 0; i < kRing; i++) {
        if (t.pinned[i]) PSX_HIP(hipHostFree(t.pinned[i]));
        if (t.done[i]) PSX_HIP(hipEventDestroy(t.done[i]));
        t.pinned[i] = nullptr; t.done[i] = nullptr; t.pending[i] = false;
    }
    if (t.dev) PSX_HIP(hipFree(t.dev));
    t.dev = nullptr; t.cap = 0; t.shadow.clear();
    return PSX_OK;
}

int32_t table_reserve(Table &t, size_t bytes) {
    if (bytes <= t.cap) return PSX_OK;
    // growing is rare (first call with a larger list): drain the device, then reallocate
    PSX_HIP(hipDeviceSynchronize());
    int32_t rc = table_free(t);
    if (rc != PSX_OK) return rc;
    size_t cap = bytes + bytes / 2 + 4096;
    PSX_HIP(hipMalloc(&t.dev, cap));
    for (int i = 0; i < kRing; i++) {
        PSX_HIP(hipHostMalloc(&t.pinned[i], cap, hipHostMallocDefault));
        PSX_HIP(hipEventCreateWithFlags(&t.done[i], hipEventDisableTiming));
    }
    t.cap = cap;
    return PSX_OK;
}

// Is `s` being recorded into a HIP graph?  (A failing query counts as "no": the next call reports the error.)
bool capturing(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return st != hipStreamCaptureStatusNone;
}

int32_t table_upload(Table &t, const void *data, size_t bytes, hipStream_t s) {
    if (bytes == 0) return PSX_OK;
    if (t.shadow.size() == bytes && memcmp(t.shadow.data(), data, bytes) == 0) return PSX_OK;
    // the upload reads a pinned buffer that later calls reuse: a graph must not replay it
    if (capturing(s))
        return fail(PSX_ECAPTURE, "the descriptor table of this call differs from the one on the device and cannot be uploaded while the "
                                  "stream is being captured: issue the same call once outside the capture first");
    int32_t rc = table_reserve(t, bytes);
    if (rc != PSX_OK) return rc;
    const int k = t.next;
    t.next = (t.next + 1) % kRing;
    if (t.pending[k]) { PSX_HIP(hipEventSynchronize(t.done[k])); t.pending[k] = false; }
    memcpy(t.pinned[k], data, bytes);
    PSX_HIP(hipMemcpyAsync(t.dev, t.pinned[k], bytes, hipMemcpyHostToDevice, s));
    PSX_HIP(hipEventRecord(t.done[k], s));
    t.pending[k] = true;
    t.shadow.assign(static_cast<const unsigned char *>(data), static_cast<const unsigned char *>(data) + bytes);
    return PSX_OK;
}

// Uploads descriptors followed by the dense array of their first tiles; returns device pointers to both.
template <typename D>
int32_t upload_described(Table &t, const std::vector<D> &v, std::vector<unsigned char> &blob, hipStream_t s,
                         const D **items, const uint64_t **begins) {
    const size_t nd = v.size() * sizeof(D);
    blob.resize(nd + v.size() * sizeof(uint64_t));
    if (!v.empty()) memcpy(blob.data(), v.data(), nd);
    uint64_t *b = reinterpret_cast<uint64_t *>(blob.data() + nd);
    for (size_t i = 0; i < v.size(); i++) b[i] = v[i].tile_begin;
    int32_t rc = table_upload(t, blob.data(), blob.size(), s);
    if (rc != PSX_OK) return rc;
    *items = static_cast<const D *>(t.dev);
    *begins = reinterpret_cast<const uint64_t *>(static_cast<const unsigned char *>(t.dev) + nd);
    return PSX_OK;
}

// Copy segments: descriptors, their first tiles, and a coarse index over the tiles (at most kMaxHints groups of
// 2^shift tiles; hints[g] = the segment that owns the first tile of group g) that narrows the owner search of
// a tile from log2(n) dependent loads to a lookup and a step or two.
int32_t upload_segments(Table &t, const std::vector<CopySeg> &v, uint64_t n_tiles, std::vector<unsigned char> &blob,
                        hipStream_t s, const CopySeg **items, const uint64_t **begins, const uint32_t **hints, uint32_t *shift_out) {
    uint32_t shift = 0;
    while (((n_tiles + ((1ull << shift) - 1)) >> shift) > kMaxHints) shift++;
    const size_t groups = (size_t)((n_tiles + ((1ull << shift) - 1)) >> shift);
    const size_t nd = v.size() * sizeof(CopySeg), nb = v.size() * sizeof(uint64_t);
    blob.resize(nd + nb + (groups + 1) * sizeof(uint32_t));
    if (!v.empty()) memcpy(blob.data(), v.data(), nd);
    uint64_t *b = reinterpret_cast<uint64_t *>(blob.data() + nd);
    for (size_t i = 0; i < v.size(); i++) b[i] = v[i].tile_begin;
    uint32_t *h = reinterpret_cast<uint32_t *>(blob.data() + nd + nb);
    size_t seg = 0;
    for (size_t g = 0; g < groups; g++) {
        const uint64_t first = (uint64_t)g << shift;
        while (seg + 1 < v.size() && v[seg + 1].tile_begin <= first) seg++;
        h[g] = (uint32_t)seg;
    }
    h[groups] = v.empty() ? 0u : (uint32_t)(v.size() - 1);
    int32_t rc = table_upload(t, blob.data(), blob.size(), s);
    if (rc != PSX_OK) return rc;
    const unsigned char *base = static_cast<const unsigned char *>(t.dev);
    *items = reinterpret_cast<const CopySeg *>(base);
    *begins = reinterpret_cast<const uint64_t *>(base + nd);
    *hints = reinterpret_cast<const uint32_t *>(base + nd + nb);
    *shift_out = shift;
    return PSX_OK;
}

// beta^t as what it is defined to be here: the product of t factors, each multiplication rounded to double.
// (libm's pow approximates the real power more closely and is, for that very reason, not always the same
// double; once in a long while the difference moves a scalar rounded to fp32: with beta2 = 0.999999, c2 of
// step 12314 is one fp32 ulp apart between the two.)
// A training loop asks for t, t, t+1, t+2, ...: the product of this thread's last call is continued when
// beta is the same and t has not gone back, so the usual call costs one multiplication.
struct PowerByProduct {
    double beta = -1.0, prod = 1.0;
    uint64_t t = 0;
    double operator()(double b, uint64_t steps) {
        if (b != beta || steps < t) { beta = b; prod = 1.0; t = 0; }
        while (t < steps) {
            if (prod == 0.0) { t = steps; break; }      // underflowed: every further factor leaves it at zero
            prod = prod * b;
            t++;
        }
        return prod;
    }
};
thread_local PowerByProduct g_pow1, g_pow2;

struct TimedSpan {
    hipEvent_t a = nullptr, b = nullptr;
    bool valid = false;
};

}  // namespace

namespace {

struct CpuTile {
    const uint16_t *g16;   // device
    uint16_t *p16;         // device
    float *p, *m, *v;      // pinned host, updated in place
    uint64_t n;
    bool alias;
};

struct SpillTile {
    size_t run;            // index into the table (its AdamRun)
    const float *src[3];   // host sources (H2D) or NULL
    float *stage[3];       // device targets of the H2D / sources of the D2H
    float *dst[3];         // host targets (D2H) or NULL
    uint64_t n;
    bool alias;
};

}  // namespace

struct psx_ctx {
    int device = 0;
    int n_cu = 0;
    psx_ctx_config cfg{};
    Tuning tune;
    Table adam_tbl, move_tbl, check_tbl, pack_tbl, unpack_tbl, out_tbl;
    uint32_t *flags_dev = nullptr;     // [0] global, [1 + c] chunk c
    uint32_t *flags_host = nullptr;    // pinned read-back buffer
    size_t flags_n = 0;
    float *staging = nullptr;          // staging_slots x {p, m, v} x staging_tile_elems
    hipStream_t h2d = nullptr, d2h = nullptr;
    std::vector<hipEvent_t> ev_h2d, ev_k, ev_free;
    hipEvent_t ev_entry = nullptr, ev_h2d_end = nullptr, ev_d2h_end = nullptr;
    bool prof = false;
    TimedSpan t_pack, t_unpack, t_check, t_adam, t_spill;
    uint64_t adam_elems = 0, spill_elems = 0, h2d_bytes = 0, d2h_bytes = 0;
    std::vector<AdamRun> runs;         // scratch for table building
    std::vector<MoveRun> moves;
    std::vector<CopySeg> segs;
    std::vector<OutSeg> outs;          // output ranges of the fused fp16 unpack, sorted by (chunk, offset)
    std::vector<uint32_t> out_first;   // per resident run: index of its first range (one entry more than runs)
    std::vector<unsigned char> blob;   // scratch: descriptors + first tiles, as uploaded
    std::vector<SpillTile> spill_tiles;   // scratch of psx_chunk_adam_step (kept to keep their capacity)
    std::vector<CpuTile> cpu_tiles;
    // pinned ranges already shown to be device-accessible, by chunk index: {p32_host, m_host, v_host, used}
    struct HostSeen { const void *p[3]; uint64_t used; };
    std::vector<HostSeen> host_seen;
    int copy_unroll_now = 1;           // tile shape the segments in `segs` were cut for
    // step state on the device (PSX_STEP_DEVICE_STATE)
    StepState *state_dev = nullptr;
    StepState *state_host = nullptr;   // pinned read-back buffer
    bool state_on = false;
    psx_adam_hyper state_hyper{};      // the hyper-parameters the state was initialised with
    // host-core execution (PSX_EXEC_CPU), allocated on first use
    CpuPool *pool = nullptr;
    hipStream_t aux = nullptr;         // H2D of the fp16 parameter tiles
    uint16_t *cpu_g[kCpuSlots] = {nullptr, nullptr, nullptr};   // pinned: fp16 gradient tiles from the GPU
    uint16_t *cpu_h[kCpuSlots] = {nullptr, nullptr, nullptr};   // pinned: fp16 parameter tiles for the GPU
    hipEvent_t ev_cg[kCpuSlots] = {nullptr, nullptr, nullptr}, ev_ch[kCpuSlots] = {nullptr, nullptr, nullptr};
    hipEvent_t ev_flag = nullptr, ev_cpu_end = nullptr;
    uint64_t cpu_tile_alloc = 0;
    float cpu_ms = 0.0f;
    uint64_t cpu_elems = 0;
};

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int32_t span_begin(psx_ctx *c, TimedSpan &t, hipStream_t s) {
    t.valid = false;
    if (!c->prof || capturing(s)) return PSX_OK;
    PSX_HIP(hipEventRecord(t.a, s));
    return PSX_OK;
}
int32_t span_end(psx_ctx *c, TimedSpan &t, hipStream_t s) {
    if (!c->prof || capturing(s)) return PSX_OK;
    PSX_HIP(hipEventRecord(t.b, s));
    t.valid = true;
    return PSX_OK;
}

int32_t set_device_guard(psx_ctx *c) {
    int cur = -1;
    PSX_HIP(hipGetDevice(&cur));
    if (cur != c->device)
        return fail(PSX_EINVAL, "context belongs to device %d but device %d is current", c->device, cur);
    return PSX_OK;
}

// Append the runs of one chunk list section; returns the number of tiles.
uint64_t push_run(std::vector<AdamRun> &v, const void *g16, void *p16, void *p, void *m, void *vv,
                  uint64_t n, uint64_t tile_begin, uint64_t tile_elems, uint32_t chunk) {
    AdamRun r;
    r.g16 = static_cast<const uint16_t *>(g16);
    r.p16 = static_cast<uint16_t *>(p16);
    r.p = static_cast<float *>(p); r.m = static_cast<float *>(m); r.v = static_cast<float *>(vv);
    r.n = n; r.tile_begin = tile_begin; r.chunk = chunk; r.pad = 0;
    v.push_back(r);
    return (n + tile_elems - 1) / tile_elems;
}

}  // namespace

// ====================================================================== context

extern "C" int32_t psx_ctx_create(const psx_ctx_config *cfg, psx_ctx **out) {
    if (cfg == nullptr || out == nullptr) return fail(PSX_EINVAL, "psx_ctx_create: NULL argument");
    *out = nullptr;
    if (cfg->max_chunks == 0 || cfg->max_chunks > (1ull << 24))
        return fail(PSX_EINVAL, "psx_ctx_create: max_chunks %llu out of range", (unsigned long long)cfg->max_chunks);
    if (cfg->staging_tile_elems != 0) {
        if (cfg->staging_slots < 2 || cfg->staging_slots > 8)
            return fail(PSX_EINVAL, "psx_ctx_create: staging_slots must be 2..8");
        if (cfg->staging_tile_elems % 8 != 0)
            return fail(PSX_EINVAL, "psx_ctx_create: staging_tile_elems must be a multiple of 8");
    }
    psx_ctx *c = new psx_ctx();
    c->cfg = *cfg;
    auto bail = [&](int32_t rc) { psx_ctx_destroy(c); return rc; };
#define PSX_TRY(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return bail(fail(PSX_EHIP, "%s -> %s", #call, hipGetErrorString(e_))); } while (0)
    PSX_TRY(hipGetDevice(&c->device));
    PSX_TRY(hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device));
    if (c->n_cu <= 0) c->n_cu = 256;
    c->tune.lds_per_cu = query_lds_per_cu(c->device);
    c->flags_n = 1 + (size_t)cfg->max_chunks;
    PSX_TRY(hipMalloc(reinterpret_cast<void **>(&c->flags_dev), c->flags_n * sizeof(uint32_t)));
    PSX_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->flags_host), c->flags_n * sizeof(uint32_t), hipHostMallocDefault));
    PSX_TRY(hipMemset(c->flags_dev, 0, c->flags_n * sizeof(uint32_t)));
    PSX_TRY(hipMalloc(reinterpret_cast<void **>(&c->state_dev), sizeof(StepState)));
    PSX_TRY(hipHostMalloc(reinterpret_cast<void **>(&c->state_host), sizeof(StepState), hipHostMallocDefault));
    PSX_TRY(hipMemset(c->state_dev, 0, sizeof(StepState)));
    PSX_TRY(hipStreamCreateWithFlags(&c->h2d, hipStreamNonBlocking));
    PSX_TRY(hipStreamCreateWithFlags(&c->d2h, hipStreamNonBlocking));
    PSX_TRY(hipEventCreateWithFlags(&c->ev_entry, hipEventDisableTiming));
    PSX_TRY(hipEventCreateWithFlags(&c->ev_h2d_end, hipEventDisableTiming));
    PSX_TRY(hipEventCreateWithFlags(&c->ev_d2h_end, hipEventDisableTiming));
    const uint32_t ring = cfg->staging_tile_elems ? cfg->staging_slots : 2;
    c->ev_h2d.resize(ring); c->ev_k.resize(ring); c->ev_free.resize(ring);
    for (uint32_t i = 0; i < ring; i++) {
        PSX_TRY(hipEventCreateWithFlags(&c->ev_h2d[i], hipEventDisableTiming));
        PSX_TRY(hipEventCreateWithFlags(&c->ev_k[i], hipEventDisableTiming));
        PSX_TRY(hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
    }
    for (TimedSpan *t : {&c->t_pack, &c->t_unpack, &c->t_check, &c->t_adam, &c->t_spill}) {
        PSX_TRY(hipEventCreate(&t->a));
        PSX_TRY(hipEventCreate(&t->b));
    }
    if (cfg->staging_tile_elems) {
        const size_t bytes = (size_t)3 * cfg->staging_slots * cfg->staging_tile_elems * sizeof(float);
        PSX_TRY(hipMalloc(reinterpret_cast<void **>(&c->staging), bytes));
    }
#undef PSX_TRY
    int32_t rc;
    const size_t tiles_guess = cfg->staging_tile_elems ? 64 : 0;
    if ((rc = table_reserve(c->adam_tbl, (3 * cfg->max_chunks + tiles_guess) * (sizeof(AdamRun) + 8))) != PSX_OK) return bail(rc);
    if ((rc = table_reserve(c->move_tbl, cfg->max_chunks * (sizeof(MoveRun) + 8))) != PSX_OK) return bail(rc);
    if ((rc = table_reserve(c->check_tbl, cfg->max_chunks * (sizeof(AdamRun) + 8))) != PSX_OK) return bail(rc);
    const size_t segs = (size_t)cfg->max_tensors + (size_t)cfg->max_chunks + 1;
    if ((rc = table_reserve(c->pack_tbl, segs * (sizeof(CopySeg) + 8) + (kMaxHints + 1) * 4)) != PSX_OK) return bail(rc);
    if ((rc = table_reserve(c->unpack_tbl, segs * (sizeof(CopySeg) + 8) + (kMaxHints + 1) * 4)) != PSX_OK) return bail(rc);
    *out = c;
    return PSX_OK;
}

extern "C" int32_t psx_ctx_destroy(psx_ctx *c) {
    if (c == nullptr) return PSX_OK;
    int32_t rc = PSX_OK;
    auto note = [&](hipError_t e, const char *what) {
        if (e != hipSuccess && rc == PSX_OK) rc = fail(PSX_EHIP, "psx_ctx_destroy: %s -> %s", what, hipGetErrorString(e));
    };
    note(hipDeviceSynchronize(), "hipDeviceSynchronize");
    for (Table *t : {&c->adam_tbl, &c->move_tbl, &c->check_tbl, &c->pack_tbl, &c->unpack_tbl, &c->out_tbl}) {
        int32_t r = table_free(*t);
        if (r != PSX_OK && rc == PSX_OK) rc = r;
    }
    if (c->flags_dev) note(hipFree(c->flags_dev), "hipFree(flags)");
    if (c->flags_host) note(hipHostFree(c->flags_host), "hipHostFree(flags)");
    if (c->staging) note(hipFree(c->staging), "hipFree(staging)");
    if (c->state_dev) note(hipFree(c->state_dev), "hipFree(state)");
    if (c->state_host) note(hipHostFree(c->state_host), "hipHostFree(state)");
    if (c->pool) cpu_pool_destroy(c->pool);
    if (c->aux) note(hipStreamDestroy(c->aux), "hipStreamDestroy");
    for (int i = 0; i < kCpuSlots; i++) {
        if (c->cpu_g[i]) note(hipHostFree(c->cpu_g[i]), "hipHostFree(cpu_g)");
        if (c->cpu_h[i]) note(hipHostFree(c->cpu_h[i]), "hipHostFree(cpu_h)");
        if (c->ev_cg[i]) note(hipEventDestroy(c->ev_cg[i]), "hipEventDestroy");
        if (c->ev_ch[i]) note(hipEventDestroy(c->ev_ch[i]), "hipEventDestroy");
    }
    if (c->ev_flag) note(hipEventDestroy(c->ev_flag), "hipEventDestroy");
    if (c->ev_cpu_end) note(hipEventDestroy(c->ev_cpu_end), "hipEventDestroy");
    if (c->h2d) note(hipStreamDestroy(c->h2d), "hipStreamDestroy");
    if (c->d2h) note(hipStreamDestroy(c->d2h), "hipStreamDestroy");
    for (hipEvent_t e : {c->ev_entry, c->ev_h2d_end, c->ev_d2h_end})
        if (e) note(hipEventDestroy(e), "hipEventDestroy");
    for (auto *vec : {&c->ev_h2d, &c->ev_k, &c->ev_free})
        for (hipEvent_t e : *vec)
            if (e) note(hipEventDestroy(e), "hipEventDestroy");
    for (TimedSpan *t : {&c->t_pack, &c->t_unpack, &c->t_check, &c->t_adam, &c->t_spill}) {
        if (t->a) note(hipEventDestroy(t->a), "hipEventDestroy");
        if (t->b) note(hipEventDestroy(t->b), "hipEventDestroy");
    }
    delete c;
    return rc;
}

extern "C" int32_t psx_ctx_set_tuning(psx_ctx *c, uint32_t key, int64_t value) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_ctx_set_tuning: ctx is NULL");
    switch (key) {
        case PSX_TUNE_ADAM_BLOCKS_PER_CU:
            if (value < 0 || value > 64) return fail(PSX_EINVAL, "adam blocks per CU must be 0..64");
            c->tune.adam_blocks_per_cu = (int)value;
            break;
        case PSX_TUNE_ADAM_UNROLL:
            if (value != 1 && value != 2 && value != 4) return fail(PSX_EINVAL, "adam unroll must be 1, 2 or 4");
            c->tune.adam_unroll = (int)value;
            break;
        case PSX_TUNE_NONTEMPORAL:
            c->tune.nontemporal = value != 0;
            break;
        case PSX_TUNE_COPY_BLOCKS_PER_CU:
            if (value < 0 || value > 64) return fail(PSX_EINVAL, "copy blocks per CU must be 0..64");
            c->tune.copy_blocks_per_cu = (int)value;
            break;
        case PSX_TUNE_COPY_UNROLL:
            if (value != 0 && value != 1 && value != 4) return fail(PSX_EINVAL, "copy unroll must be 0 (by tensor count), 1 or 4");
            c->tune.copy_unroll = (int)value;
            break;
        case PSX_TUNE_COPY_THREADS:
            if (value != 64 && value != 256) return fail(PSX_EINVAL, "copy threads must be 64 or 256");
            c->tune.copy_threads = (int)value;
            break;
        case PSX_TUNE_FUSED_UNPACK:
            if (value < 0 || value > 2) return fail(PSX_EINVAL, "fused unpack must be 0 (by alignment), 1 (always) or 2 (never)");
            c->tune.fused_unpack = (int)value;
            break;
        case PSX_TUNE_HOST_MODE:
            if (value != 0 && value != 1) return fail(PSX_EINVAL, "host mode must be 0 (staged copies) or 1 (direct access)");
            c->tune.host_mode = (int)value;
            break;
        case PSX_TUNE_HOST_GRID:
            if (value < 1 || value > 65536) return fail(PSX_EINVAL, "host grid must be 1..65536 workgroups");
            c->tune.host_grid = (int)value;
            break;
        case PSX_TUNE_HOST_UNROLL:
            if (value != 1 && value != 2 && value != 4) return fail(PSX_EINVAL, "host unroll must be 1, 2 or 4");
            c->tune.host_unroll = (int)value;
            break;
        case PSX_TUNE_CPU_THREADS:
            if (value < 0 || value > 256) return fail(PSX_EINVAL, "cpu threads must be 0..256");
            if (c->pool && (int)value != c->tune.cpu_threads) { cpu_pool_destroy(c->pool); c->pool = nullptr; }
            c->tune.cpu_threads = (int)value;
            break;
        case PSX_TUNE_CPU_ISA:
            if (value != 0 && value != 1) return fail(PSX_EINVAL, "cpu isa must be 0 (widest available) or 1 (AVX2)");
            c->tune.cpu_isa = (int)value;
            break;
        case PSX_TUNE_CPU_TILE_ELEMS:
            if (value < 16 || value % 16 != 0 || value > (1ll << 28)) return fail(PSX_EINVAL, "cpu tile must be a multiple of 16 in 16..2^28");
            c->tune.cpu_tile_elems = (uint64_t)value;
            break;
        case PSX_TUNE_ADAM_THREADS:
            if (value != 64 && value != 256) return fail(PSX_EINVAL, "adam threads must be 64 or 256");
            c->tune.adam_threads = (int)value;
            break;
        case PSX_TUNE_ADAM_WG_PER_CU:
            if (value < 0 || value > 64) return fail(PSX_EINVAL, "adam workgroups per CU must be 0..64");
            c->tune.adam_wg_per_cu = (int)value;
            break;
        default:
            return fail(PSX_EINVAL, "psx_ctx_set_tuning: unknown key %u", key);
    }
    // tile sizes enter the cached tables: force a rebuild and upload
    c->adam_tbl.shadow.clear();
    return PSX_OK;
}

extern "C" int32_t psx_ctx_set_profiling(psx_ctx *c, int32_t on) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_ctx_set_profiling: ctx is NULL");
    c->prof = on != 0;
    for (TimedSpan *t : {&c->t_pack, &c->t_unpack, &c->t_check, &c->t_adam, &c->t_spill}) t->valid = false;
    return PSX_OK;
}

extern "C" int32_t psx_ctx_get_timing(psx_ctx *c, psx_timing *out) {
    if (c == nullptr || out == nullptr) return fail(PSX_EINVAL, "psx_ctx_get_timing: NULL argument");
    memset(out, 0, sizeof(*out));
    float *dst[5] = {&out->pack_ms, &out->unpack_ms, &out->check_ms, &out->adam_ms, &out->spill_ms};
    TimedSpan *src[5] = {&c->t_pack, &c->t_unpack, &c->t_check, &c->t_adam, &c->t_spill};
    for (int i = 0; i < 5; i++) {
        if (!src[i]->valid) continue;
        PSX_HIP(hipEventSynchronize(src[i]->b));
        PSX_HIP(hipEventElapsedTime(dst[i], src[i]->a, src[i]->b));
    }
    out->adam_elems = c->adam_elems;
    out->spill_elems = c->spill_elems;
    out->h2d_bytes = c->h2d_bytes;
    out->d2h_bytes = c->d2h_bytes;
    out->cpu_ms = c->cpu_ms;
    out->cpu_threads = c->pool ? (uint32_t)cpu_pool_size(c->pool) : 0u;
    out->cpu_elems = c->cpu_elems;
    return PSX_OK;
}

extern "C" int32_t psx_copy_bytes(psx_ctx *c, void *dst, const void *src, uint64_t n_bytes, void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_copy_bytes: ctx is NULL");
    if (n_bytes == 0) return PSX_OK;
    if (dst == nullptr || src == nullptr) return fail(PSX_EINVAL, "psx_copy_bytes: NULL pointer");
    if (!aligned16(dst) || !aligned16(src) || n_bytes % 16 != 0)
        return fail(PSX_EALIGN, "psx_copy_bytes: pointers and size must be multiples of 16");
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    PSX_HIP(launch_copy_bytes(dst, src, n_bytes, c->tune, c->n_cu, static_cast<hipStream_t>(stream)));
    return PSX_OK;
}

extern "C" int32_t psx_pinned_alloc(uint64_t n_bytes, void **out) {
    if (out == nullptr) return fail(PSX_EINVAL, "psx_pinned_alloc: out is NULL");
    *out = nullptr;
    if (n_bytes == 0) return fail(PSX_EINVAL, "psx_pinned_alloc: zero bytes");
    PSX_HIP(hipHostMalloc(out, n_bytes, hipHostMallocDefault));
    return PSX_OK;
}

extern "C" int32_t psx_pinned_free(void *ptr) {
    if (ptr == nullptr) return PSX_OK;
    PSX_HIP(hipHostFree(ptr));
    return PSX_OK;
}

extern "C" int32_t psx_measure_link(psx_ctx *c, uint64_t mib, uint32_t reps, psx_link_rates *out) {
    if (c == nullptr || out == nullptr) return fail(PSX_EINVAL, "psx_measure_link: NULL argument");
    if (mib == 0 || mib > 16384 || reps == 0) return fail(PSX_EINVAL, "psx_measure_link: mib must be 1..16384, reps > 0");
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    const size_t nb = (size_t)mib << 20;
    void *h_src = nullptr, *h_dst = nullptr, *d_in = nullptr, *d_out = nullptr;
    auto cleanup = [&]() {
        if (h_src) (void)hipHostFree(h_src);
        if (h_dst) (void)hipHostFree(h_dst);
        if (d_in) (void)hipFree(d_in);
        if (d_out) (void)hipFree(d_out);
    };
#define PSX_TRY(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { cleanup(); return fail(PSX_EHIP, "%s -> %s", #call, hipGetErrorString(e_)); } } while (0)
    PSX_TRY(hipHostMalloc(&h_src, nb, hipHostMallocDefault));
    PSX_TRY(hipHostMalloc(&h_dst, nb, hipHostMallocDefault));
    PSX_TRY(hipMalloc(&d_in, nb));
    PSX_TRY(hipMalloc(&d_out, nb));
    memset(h_src, 1, nb);
    memset(h_dst, 0, nb);
    PSX_TRY(hipMemset(d_out, 2, nb));
    PSX_TRY(hipDeviceSynchronize());
    double best[3] = {0, 0, 0};
    for (int mode = 0; mode < 3; mode++) {                  // 0 H2D alone, 1 D2H alone, 2 both
        for (uint32_t r = 0; r < reps + 2; r++) {
            const auto t0 = std::chrono::steady_clock::now();
            if (mode != 1) PSX_TRY(hipMemcpyAsync(d_in, h_src, nb, hipMemcpyHostToDevice, c->h2d));
            if (mode != 0) PSX_TRY(hipMemcpyAsync(h_dst, d_out, nb, hipMemcpyDeviceToHost, c->d2h));
            PSX_TRY(hipStreamSynchronize(c->h2d));
            PSX_TRY(hipStreamSynchronize(c->d2h));
            const double dt = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
            const double rate = (double)nb / dt / 1e9;
            if (r >= 2 && rate > best[mode]) best[mode] = rate;
        }
    }
#undef PSX_TRY
    cleanup();
    out->h2d_alone = best[0];
    out->d2h_alone = best[1];
    out->each_way_both = best[2];
    return PSX_OK;
}

// ====================================================================== pack / unpack

namespace {

// Cut every tensor into pieces that lie inside one chunk and emit one copy
// segment per piece.  to_chunk selects the direction.
int32_t build_segments(psx_ctx *c, const char *who, uint32_t dtype, const void *const *tensors,
                       const psx_slot *slots, size_t n, const void *const *chunks, size_t n_chunks,
                       uint64_t chunk_elems, bool to_chunk, uint64_t *n_tiles_out, uint64_t *n_elems_out) {
    if (c == nullptr) return fail(PSX_EINVAL, "%s: ctx is NULL", who);
    if (dtype != PSX_F16 && dtype != PSX_F32) return fail(PSX_EINVAL, "%s: dtype %u is neither PSX_F16 nor PSX_F32", who, dtype);
    if (chunk_elems == 0) return fail(PSX_EINVAL, "%s: chunk_elems is 0", who);
    if (n != 0 && (tensors == nullptr || slots == nullptr)) return fail(PSX_EINVAL, "%s: tensors/slots is NULL", who);
    if (n_chunks != 0 && chunks == nullptr) return fail(PSX_EINVAL, "%s: chunks is NULL", who);
    if (n_chunks > c->cfg.max_chunks) return fail(PSX_ECAP, "%s: %zu chunks, context holds %llu", who, n_chunks, (unsigned long long)c->cfg.max_chunks);
    if (n > c->cfg.max_tensors) return fail(PSX_ECAP, "%s: %zu tensors, context holds %llu", who, n, (unsigned long long)c->cfg.max_tensors);
    const uint32_t es = dtype == PSX_F16 ? 2u : 4u;
    c->copy_unroll_now = copy_unroll_for(c->tune, n);
    const uint64_t tile_elems = copy_tile_bytes(c->tune, c->copy_unroll_now) / es;
    const uint64_t total = (uint64_t)n_chunks * chunk_elems;
    for (size_t k = 0; k < n_chunks; k++) {
        if (chunks[k] == nullptr) return fail(PSX_EINVAL, "%s: chunk %zu is NULL", who, k);
        if (reinterpret_cast<uintptr_t>(chunks[k]) % es) return fail(PSX_EALIGN, "%s: chunk %zu is not element-aligned", who, k);
    }
    c->segs.clear();
    uint64_t tiles = 0, elems = 0;
    for (size_t i = 0; i < n; i++) {
        const uint64_t s = slots[i].numel;
        if (s == 0) continue;
        if (tensors[i] == nullptr) return fail(PSX_EINVAL, "%s: tensor %zu is NULL", who, i);
        if (reinterpret_cast<uintptr_t>(tensors[i]) % es) return fail(PSX_EALIGN, "%s: tensor %zu is not element-aligned", who, i);
        if (slots[i].offset > chunk_elems) return fail(PSX_EINVAL, "%s: slot %zu offset beyond the chunk", who, i);
        const uint64_t lin = (uint64_t)slots[i].chunk * chunk_elems + slots[i].offset;
        if (lin > total || s > total - lin)
            return fail(PSX_EINVAL, "%s: slot %zu (chunk %u offset %llu numel %llu) runs past the chunk list", who, i,
                        slots[i].chunk, (unsigned long long)slots[i].offset, (unsigned long long)s);
        uint64_t done = 0;
        while (done < s) {
            const uint64_t p = lin + done;
            const uint64_t ck = p / chunk_elems, off = p % chunk_elems;
            const uint64_t take = s - done < chunk_elems - off ? s - done : chunk_elems - off;
            const unsigned char *t = static_cast<const unsigned char *>(tensors[i]) + done * es;
            const unsigned char *k = static_cast<const unsigned char *>(chunks[ck]) + off * es;
            CopySeg g;
            g.src = to_chunk ? t : k;
            g.dst = const_cast<unsigned char *>(to_chunk ? k : t);
            g.n = take; g.tile_begin = tiles; g.chunk = (uint32_t)ck; g.pad = 0;
            c->segs.push_back(g);
            tiles += copy_tiles_of(g.dst, take, es, tile_elems);
            done += take;
        }
        elems += s;
    }
    *n_tiles_out = tiles;
    *n_elems_out = elems;
    return PSX_OK;
}

int32_t run_copy(psx_ctx *c, Table &tbl, TimedSpan &span, uint32_t dtype, uint64_t tiles, bool check, hipStream_t s) {
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    if (tiles == 0) return PSX_OK;
    if (c->segs.size() > 0xFFFFFFFFull) return fail(PSX_ECAP, "too many copy segments");
    const CopySeg *segs_dev = nullptr;
    const uint64_t *begins_dev = nullptr;
    const uint32_t *hints_dev = nullptr;
    uint32_t shift = 0;
    rc = upload_segments(tbl, c->segs, tiles, c->blob, s, &segs_dev, &begins_dev, &hints_dev, &shift);
    if (rc != PSX_OK) return rc;
    if ((rc = span_begin(c, span, s)) != PSX_OK) return rc;
    Tuning tn = c->tune;
    tn.copy_unroll = c->copy_unroll_now;
    PSX_HIP(launch_copy(SegView{segs_dev, begins_dev, (uint32_t)c->segs.size(), hints_dev, shift}, tiles,
                        dtype == PSX_F16 ? 2u : 4u, check ? c->flags_dev : nullptr,
                        check ? c->flags_dev + 1 : nullptr, tn, c->n_cu, s));
    return span_end(c, span, s);
}

}  // namespace

extern "C" int32_t psx_pack(psx_ctx *c, uint32_t dtype, const void *const *tensors, const psx_slot *slots,
                            size_t n, void *const *chunks, size_t n_chunks, uint64_t chunk_elems,
                            uint32_t flags, void *stream) {
    if (flags & ~PSX_PACK_CHECK_OVERFLOW) return fail(PSX_EINVAL, "psx_pack: unknown flags 0x%x", flags);
    if ((flags & PSX_PACK_CHECK_OVERFLOW) && dtype != PSX_F16)
        return fail(PSX_EINVAL, "psx_pack: PSX_PACK_CHECK_OVERFLOW needs PSX_F16");
    uint64_t tiles = 0, elems = 0;
    int32_t rc = build_segments(c, "psx_pack", dtype, tensors, slots, n, chunks, n_chunks, chunk_elems, true, &tiles, &elems);
    if (rc != PSX_OK) return rc;
    return run_copy(c, c->pack_tbl, c->t_pack, dtype, tiles, (flags & PSX_PACK_CHECK_OVERFLOW) != 0, static_cast<hipStream_t>(stream));
}

extern "C" int32_t psx_unpack(psx_ctx *c, uint32_t dtype, void *const *tensors, const psx_slot *slots,
                              size_t n, const void *const *chunks, size_t n_chunks, uint64_t chunk_elems,
                              uint32_t flags, void *stream) {
    if (flags != 0) return fail(PSX_EINVAL, "psx_unpack: unknown flags 0x%x", flags);
    uint64_t tiles = 0, elems = 0;
    int32_t rc = build_segments(c, "psx_unpack", dtype, tensors, slots, n, chunks, n_chunks, chunk_elems, false, &tiles, &elems);
    if (rc != PSX_OK) return rc;
    return run_copy(c, c->unpack_tbl, c->t_unpack, dtype, tiles, false, static_cast<hipStream_t>(stream));
}

// ====================================================================== overflow flag

extern "C" int32_t psx_overflow_reset(psx_ctx *c, void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_overflow_reset: ctx is NULL");
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    PSX_HIP(launch_fill_u32(c->flags_dev, c->flags_n, 0u, static_cast<hipStream_t>(stream)));
    return PSX_OK;
}

extern "C" int32_t psx_overflow_read(psx_ctx *c, uint32_t *per_chunk, size_t n_chunks, uint32_t *flag_out,
                                     void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_overflow_read: ctx is NULL");
    if (per_chunk != nullptr && n_chunks > c->cfg.max_chunks)
        return fail(PSX_ECAP, "psx_overflow_read: %zu chunks, context holds %llu", n_chunks, (unsigned long long)c->cfg.max_chunks);
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (capturing(s)) return fail(PSX_ECAPTURE, "psx_overflow_read synchronises and cannot be recorded into a graph");
    const size_t cnt = 1 + (per_chunk ? n_chunks : 0);
    PSX_HIP(hipMemcpyAsync(c->flags_host, c->flags_dev, cnt * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    PSX_HIP(hipStreamSynchronize(s));
    if (flag_out) *flag_out = c->flags_host[0] ? 1u : 0u;
    if (per_chunk)
        for (size_t k = 0; k < n_chunks; k++) per_chunk[k] = c->flags_host[1 + k] ? 1u : 0u;
    return PSX_OK;
}

extern "C" int32_t psx_overflow_check(psx_ctx *c, const void *const *g16_chunks, const uint64_t *used,
                                      size_t n_chunks, uint32_t *per_chunk, uint32_t *flag_out, void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_overflow_check: ctx is NULL");
    if (n_chunks != 0 && (g16_chunks == nullptr || used == nullptr)) return fail(PSX_EINVAL, "psx_overflow_check: NULL array");
    if (n_chunks > c->cfg.max_chunks)
        return fail(PSX_ECAP, "psx_overflow_check: %zu chunks, context holds %llu", n_chunks, (unsigned long long)c->cfg.max_chunks);
    c->runs.clear();
    uint64_t tiles = 0;
    for (size_t k = 0; k < n_chunks; k++) {
        if (used[k] == 0) continue;
        if (g16_chunks[k] == nullptr) return fail(PSX_EINVAL, "psx_overflow_check: chunk %zu is NULL", k);
        if (!aligned16(g16_chunks[k])) return fail(PSX_EALIGN, "psx_overflow_check: chunk %zu is not 16-byte aligned", k);
        tiles += push_run(c->runs, g16_chunks[k], nullptr, nullptr, nullptr, nullptr, used[k], tiles, kCheckTileElems, (uint32_t)k);
    }
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((per_chunk != nullptr || flag_out != nullptr) && capturing(s))
        return fail(PSX_ECAPTURE, "psx_overflow_check: reading the flags back synchronises and cannot be recorded into a graph (pass NULL for both outputs)");
    const AdamRun *runs_dev = nullptr;
    const uint64_t *begins_dev = nullptr;
    rc = upload_described(c->check_tbl, c->runs, c->blob, s, &runs_dev, &begins_dev);
    if (rc != PSX_OK) return rc;
    PSX_HIP(launch_fill_u32(c->flags_dev, c->flags_n, 0u, s));
    if ((rc = span_begin(c, c->t_check, s)) != PSX_OK) return rc;
    PSX_HIP(launch_check(RunView{runs_dev, begins_dev, (uint32_t)c->runs.size()}, tiles,
                         c->flags_dev, c->flags_dev + 1, c->tune, c->n_cu, s));
    if ((rc = span_end(c, c->t_check, s)) != PSX_OK) return rc;
    if (per_chunk != nullptr || flag_out != nullptr) return psx_overflow_read(c, per_chunk, n_chunks, flag_out, stream);
    return PSX_OK;
}

// ====================================================================== step state on the device

extern "C" int32_t psx_step_state_init(psx_ctx *c, const psx_adam_hyper *hyper, const psx_scaler *scaler, void *stream) {
    if (c == nullptr || hyper == nullptr || scaler == nullptr) return fail(PSX_EINVAL, "psx_step_state_init: NULL argument");
    if (scaler->step == 0) return fail(PSX_EINVAL, "psx_step_state_init: scaler->step is 1-based");
    if (scaler->growth_interval == 0) return fail(PSX_EINVAL, "psx_step_state_init: growth_interval is 0");
    if (!(scaler->scale >= 1.0f) || !std::isfinite(scaler->scale)) return fail(PSX_EINVAL, "psx_step_state_init: the loss scale must be finite and at least 1");
    psx_adam_hyper h = *hyper;
    h.step = scaler->step;
    h.loss_scale = (double)scaler->scale;
    AdamScalars sc;
    int32_t rc = prepare_adam_scalars(&h, "psx_step_state_init", &sc);
    if (rc != PSX_OK) return rc;
    if ((rc = set_device_guard(c)) != PSX_OK) return rc;
    StepState init{};
    init.sc = sc;                       // the step-varying three are derived again on the device
    init.scale = scaler->scale;
    init.growth_interval = scaler->growth_interval;
    init.good_steps = scaler->good_steps;
    init.step = scaler->step;
    init.b1t = PowerByProduct{}(h.beta1, scaler->step);
    init.b2t = PowerByProduct{}(h.beta2, scaler->step);
    init.lr = h.lr; init.beta1 = h.beta1; init.beta2 = h.beta2;
    PSX_HIP(launch_step_state_init(c->state_dev, init, static_cast<hipStream_t>(stream)));
    c->state_hyper = h;
    c->state_on = true;
    return PSX_OK;
}

extern "C" int32_t psx_step_state_advance(psx_ctx *c, uint32_t flags, void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_step_state_advance: ctx is NULL");
    if (flags & ~PSX_ADVANCE_CLEAR_FLAGS) return fail(PSX_EINVAL, "psx_step_state_advance: unknown flags 0x%x", flags);
    if (!c->state_on) return fail(PSX_EINVAL, "psx_step_state_advance: psx_step_state_init has not been called");
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    PSX_HIP(launch_step_state_advance(c->state_dev, c->flags_dev, (flags & PSX_ADVANCE_CLEAR_FLAGS) ? c->flags_n : 0,
                                      static_cast<hipStream_t>(stream)));
    return PSX_OK;
}

extern "C" int32_t psx_step_state_read(psx_ctx *c, psx_scaler *scaler, uint32_t *last_flag, uint64_t *skipped, void *stream) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_step_state_read: ctx is NULL");
    if (!c->state_on) return fail(PSX_EINVAL, "psx_step_state_read: psx_step_state_init has not been called");
    int32_t rc = set_device_guard(c);
    if (rc != PSX_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (capturing(s)) return fail(PSX_ECAPTURE, "psx_step_state_read synchronises and cannot be recorded into a graph");
    PSX_HIP(hipMemcpyAsync(c->state_host, c->state_dev, sizeof(StepState), hipMemcpyDeviceToHost, s));
    PSX_HIP(hipStreamSynchronize(s));
    const StepState &st = *c->state_host;
    if (scaler != nullptr) {
        scaler->scale = st.scale;
        scaler->growth_interval = st.growth_interval;
        scaler->good_steps = st.good_steps;
        scaler->reserved = 0;
        scaler->step = st.step;
    }
    if (last_flag != nullptr) *last_flag = st.last_flag;
    if (skipped != nullptr) *skipped = st.skipped;
    return PSX_OK;
}

// ====================================================================== Adam step

namespace psx {

// Step-wide scalars of the update: derived in double from the caller's doubles, each rounded to fp32 once.
int32_t prepare_adam_scalars(const psx_adam_hyper *h, const char *who, AdamScalars *s) {
    if (!(h->loss_scale > 0.0) || !std::isfinite(h->loss_scale)) return fail(PSX_EINVAL, "%s: loss_scale must be positive and finite", who);
    if (h->step == 0) return fail(PSX_EINVAL, "%s: step is 1-based", who);
    if (!(h->beta1 >= 0.0 && h->beta1 < 1.0) || !(h->beta2 >= 0.0 && h->beta2 < 1.0))
        return fail(PSX_EINVAL, "%s: betas must lie in [0, 1)", who);
    const double b1t = g_pow1(h->beta1, h->step);
    const double b2t = g_pow2(h->beta2, h->step);
    s->step_size = (float)(h->lr / (1.0 - b1t));
    s->c2 = (float)(1.0 / std::sqrt(1.0 - b2t));
    s->inv_scale = (float)(1.0 / h->loss_scale);
    s->beta1 = (float)h->beta1;
    s->beta2 = (float)h->beta2;
    s->omb1 = (float)(1.0 - h->beta1);
    s->omb2 = (float)(1.0 - h->beta2);
    s->eps = (float)h->eps;
    s->wd = (float)h->weight_decay;
    s->decay = (float)(1.0 - h->lr * h->weight_decay);
    s->decay_mode = s->wd == 0.0f ? 0u : (h->adamw_mode ? 2u : 1u);
    return PSX_OK;
}

}  // namespace psx

extern "C" int32_t psx_adam_step_scalars(const psx_adam_hyper *hyper, float *out) {
    if (hyper == nullptr || out == nullptr) return fail(PSX_EINVAL, "psx_adam_step_scalars: NULL argument");
    AdamScalars s;
    const int32_t rc = prepare_adam_scalars(hyper, "psx_adam_step_scalars", &s);
    if (rc != PSX_OK) return rc;
    const float v[10] = {s.step_size, s.c2, s.inv_scale, s.beta1, s.beta2, s.omb1, s.omb2, s.eps, s.wd, s.decay};
    memcpy(out, v, sizeof(v));
    return PSX_OK;
}

namespace {

// Resources of the host-core path: worker pool, a stream for the fp16 parameter uploads, pinned
// staging for fp16 gradient and parameter tiles, events.
int32_t ensure_cpu(psx_ctx *c) {
    if (c->pool == nullptr) {
        int n = c->tune.cpu_threads;
        if (n <= 0) {
            n = (int)std::thread::hardware_concurrency();
            if (n <= 0) n = 1;
            if (n > 16) n = 16;
        }
        c->pool = cpu_pool_create(n);
    }
    if (c->aux == nullptr) {
        PSX_HIP(hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking));
        PSX_HIP(hipEventCreateWithFlags(&c->ev_flag, hipEventDisableTiming));
        PSX_HIP(hipEventCreateWithFlags(&c->ev_cpu_end, hipEventDisableTiming));
        for (int i = 0; i < kCpuSlots; i++) {
            PSX_HIP(hipEventCreateWithFlags(&c->ev_cg[i], hipEventDisableTiming));
            PSX_HIP(hipEventCreateWithFlags(&c->ev_ch[i], hipEventDisableTiming));
        }
    }
    if (c->cpu_tile_alloc < c->tune.cpu_tile_elems) {
        PSX_HIP(hipDeviceSynchronize());
        for (int i = 0; i < kCpuSlots; i++) {
            if (c->cpu_g[i]) PSX_HIP(hipHostFree(c->cpu_g[i]));
            if (c->cpu_h[i]) PSX_HIP(hipHostFree(c->cpu_h[i]));
            c->cpu_g[i] = c->cpu_h[i] = nullptr;
        }
        c->cpu_tile_alloc = 0;
        for (int i = 0; i < kCpuSlots; i++) {
            PSX_HIP(hipHostMalloc(reinterpret_cast<void **>(&c->cpu_g[i]), c->tune.cpu_tile_elems * 2, hipHostMallocDefault));
            PSX_HIP(hipHostMalloc(reinterpret_cast<void **>(&c->cpu_h[i]), c->tune.cpu_tile_elems * 2, hipHostMallocDefault));
        }
        c->cpu_tile_alloc = c->tune.cpu_tile_elems;
    }
    return PSX_OK;
}

// Everything that can be wrong with the chunk list is found here, before any work is enqueued.
int32_t validate_step(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks, bool dev_state, bool recording) {
    const uint64_t T = c->cfg.staging_tile_elems;
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.loc_in > PSX_LOC_HOST || ch.loc_out > PSX_LOC_HOST)
            return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu has a bad residency (%u -> %u)", k, ch.loc_in, ch.loc_out);
        if (ch.used == 0) continue;
        if (recording && (ch.loc_in != PSX_LOC_HBM || ch.loc_out != PSX_LOC_HBM))
            return fail(PSX_ECAPTURE, "psx_chunk_adam_step: chunk %zu has a host side; only HBM-resident chunk lists can be recorded into a graph", k);
        if (ch.g16 == nullptr || ch.p16 == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu g16/p16 is NULL", k);
        if (!aligned16(ch.g16) || !aligned16(ch.p16)) return fail(PSX_EALIGN, "psx_chunk_adam_step: chunk %zu g16/p16 not 16-byte aligned", k);
        const bool dev_side = ch.loc_in == PSX_LOC_HBM || ch.loc_out == PSX_LOC_HBM;
        const bool host_side = ch.loc_in == PSX_LOC_HOST || ch.loc_out == PSX_LOC_HOST;
        if (dev_side) {
            if (!ch.p32 || !ch.m || !ch.v) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu needs device p32/m/v", k);
            if (!aligned16(ch.p32) || !aligned16(ch.m) || !aligned16(ch.v)) return fail(PSX_EALIGN, "psx_chunk_adam_step: chunk %zu device states not 16-byte aligned", k);
        }
        if (ch.exec > PSX_EXEC_CPU) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu has a bad exec value %u", k, ch.exec);
        if (ch.exec == PSX_EXEC_CPU) {
            if (ch.loc_in != PSX_LOC_HOST || ch.loc_out != PSX_LOC_HOST)
                return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu: PSX_EXEC_CPU needs a chunk that stays on the host", k);
            if (!cpu_adam_supported()) return fail(PSX_EINVAL, "psx_chunk_adam_step: PSX_EXEC_CPU needs a host CPU with AVX2 and F16C");
            if (dev_state) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu: PSX_EXEC_CPU needs the step scalars on the host, not PSX_STEP_DEVICE_STATE", k);
        }
        if (host_side) {
            if (!ch.p32_host || !ch.m_host || !ch.v_host) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu needs pinned p32/m/v", k);
            if (!aligned16(ch.p32_host) || !aligned16(ch.m_host) || !aligned16(ch.v_host)) return fail(PSX_EALIGN, "psx_chunk_adam_step: chunk %zu host states not 16-byte aligned", k);
            const bool staged = ch.exec != PSX_EXEC_CPU && c->tune.host_mode != 1;
            if (staged && T == 0) return fail(PSX_ENOSTAGING, "psx_chunk_adam_step: chunk %zu is host-resident but the context has no staging", k);
            if (!staged && ch.exec != PSX_EXEC_CPU) {
                // the kernel will dereference these host pointers: they must be page-locked memory the
                // device can reach, over their whole used range, or the launch would fault the GPU.
                // Asking the driver costs microseconds per pointer, so a chunk whose three ranges are the
                // ones this context saw at the same index last time is not asked about again (the caller
                // keeps a host-resident chunk's buffers page-locked while it passes them).
                const void *hp[3] = {ch.p32_host, ch.m_host, ch.v_host};
                if (c->host_seen.size() < n_chunks) c->host_seen.resize(n_chunks, psx_ctx::HostSeen{{nullptr, nullptr, nullptr}, 0});
                psx_ctx::HostSeen &seen = c->host_seen[k];
                if (seen.p[0] == hp[0] && seen.p[1] == hp[1] && seen.p[2] == hp[2] && seen.used >= ch.used) continue;
                seen = psx_ctx::HostSeen{{nullptr, nullptr, nullptr}, 0};
                for (int j = 0; j < 3; j++) {
                    const char *ends[2] = {static_cast<const char *>(hp[j]), static_cast<const char *>(hp[j]) + (ch.used * sizeof(float) - 1)};
                    for (const char *q : ends) {
                        hipPointerAttribute_t at;
                        const hipError_t e = hipPointerGetAttributes(&at, q);
                        if (e != hipSuccess || at.type != hipMemoryTypeHost) {
                            (void)hipGetLastError();
                            return fail(PSX_EINVAL, "psx_chunk_adam_step: chunk %zu: host state %d is not pinned, device-accessible memory "
                                                    "(allocate it with hipHostMalloc / psx_pinned_alloc, or select PSX_TUNE_HOST_MODE 0)", k, j);
                        }
                    }
                }
                seen = psx_ctx::HostSeen{{hp[0], hp[1], hp[2]}, ch.used};
            }
        }
    }
    return PSX_OK;
}

// What one call of psx_chunk_adam_step launches, derived from the chunk list: the sections of the run table
// (in upload order: resident | re-cast | check | staged tiles | direct | direct re-cast) with their tile
// counts, the byte counts of the part with a host side, and the launch shape of the kernels that work on
// host memory.  The descriptors themselves are left in the context's scratch vectors.
struct StepPlan {
    uint64_t adam_tile = 0, recast_tile = 0;
    uint64_t res_tiles = 0, res_elems = 0, recast_tiles = 0, check_tiles = 0;
    size_t n_res = 0, n_recast = 0, n_check = 0;
    uint64_t cpu_elems = 0, spill_elems = 0, h2d_bytes = 0, d2h_bytes = 0;
    Tuning td;
    size_t direct_off = 0, n_direct = 0, n_direct_recast = 0;
    uint64_t direct_tiles = 0, direct_recast_tiles = 0, move_tiles = 0;
};

// Fills c->runs, c->moves, c->spill_tiles and c->cpu_tiles from the (validated) chunk list.
void plan_step(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks, bool use_flag, bool check_first, StepPlan &p) {
    const uint64_t T = c->cfg.staging_tile_elems;
    p.adam_tile = adam_tile_elems(c->tune);
    p.recast_tile = kRecastTileElems;
    c->runs.clear();
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.used == 0 || ch.loc_in != PSX_LOC_HBM || ch.loc_out != PSX_LOC_HBM) continue;
        p.res_tiles += push_run(c->runs, ch.g16, ch.p16, ch.p32, ch.m, ch.v, ch.used, p.res_tiles, p.adam_tile, (uint32_t)k);
        p.res_elems += ch.used;
    }
    p.n_res = c->runs.size();
    if (use_flag)
        for (size_t k = 0; k < n_chunks; k++) {
            const psx_chunk &ch = chunks[k];
            if (ch.used == 0 || ch.loc_in != PSX_LOC_HBM || ch.loc_out != PSX_LOC_HBM || ch.g16 != ch.p16) continue;
            p.recast_tiles += push_run(c->runs, ch.g16, ch.p16, ch.p32, ch.m, ch.v, ch.used, p.recast_tiles, p.recast_tile, (uint32_t)k);
        }
    p.n_recast = c->runs.size() - p.n_res;
    if (check_first)
        for (size_t k = 0; k < n_chunks; k++) {
            if (chunks[k].used == 0) continue;
            p.check_tiles += push_run(c->runs, chunks[k].g16, nullptr, nullptr, nullptr, nullptr, chunks[k].used, p.check_tiles, kCheckTileElems, (uint32_t)k);
        }
    p.n_check = c->runs.size() - p.n_res - p.n_recast;

    std::vector<SpillTile> &tiles = c->spill_tiles;
    std::vector<CpuTile> &cpu_tiles = c->cpu_tiles;
    tiles.clear();
    cpu_tiles.clear();
    uint64_t slot_counter = 0;
    const bool direct = c->tune.host_mode == 1;
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.used == 0 || (ch.loc_in == PSX_LOC_HBM && ch.loc_out == PSX_LOC_HBM)) continue;
        const bool in_host = ch.loc_in == PSX_LOC_HOST, out_host = ch.loc_out == PSX_LOC_HOST;
        if (ch.exec == PSX_EXEC_CPU) {                // updated by the host cores: the last part of psx_chunk_adam_step
            const uint64_t ct = c->tune.cpu_tile_elems;
            for (uint64_t off = 0; off < ch.used; off += ct) {
                CpuTile t;
                t.g16 = static_cast<const uint16_t *>(ch.g16) + off;
                t.p16 = static_cast<uint16_t *>(ch.p16) + off;
                t.p = static_cast<float *>(ch.p32_host) + off;
                t.m = static_cast<float *>(ch.m_host) + off;
                t.v = static_cast<float *>(ch.v_host) + off;
                t.n = ch.used - off < ct ? ch.used - off : ct;
                t.alias = ch.g16 == ch.p16;
                cpu_tiles.push_back(t);
            }
            p.cpu_elems += ch.used;
            continue;
        }
        p.spill_elems += ch.used;
        if (direct) {                                 // handled below: the kernels work on the host buffers
            if (in_host) p.h2d_bytes += 3 * ch.used * sizeof(float);
            if (out_host) p.d2h_bytes += 3 * ch.used * sizeof(float);
            continue;
        }
        for (uint64_t off = 0; off < ch.used; off += T) {
            const uint64_t n = ch.used - off < T ? ch.used - off : T;
            SpillTile t{};
            t.n = n;
            t.alias = ch.g16 == ch.p16;
            float *dev[3];
            if (in_host && out_host) {
                const uint64_t slot = slot_counter % c->cfg.staging_slots;
                for (int j = 0; j < 3; j++) dev[j] = c->staging + ((size_t)slot * 3 + j) * T;
            } else {
                dev[0] = static_cast<float *>(ch.p32) + off;
                dev[1] = static_cast<float *>(ch.m) + off;
                dev[2] = static_cast<float *>(ch.v) + off;
            }
            slot_counter++;
            const float *hs[3] = {static_cast<const float *>(ch.p32_host), static_cast<const float *>(ch.m_host), static_cast<const float *>(ch.v_host)};
            for (int j = 0; j < 3; j++) {
                t.stage[j] = dev[j];
                t.src[j] = in_host ? hs[j] + off : nullptr;
                t.dst[j] = out_host ? const_cast<float *>(hs[j]) + off : nullptr;
            }
            if (in_host) p.h2d_bytes += 3 * n * sizeof(float);
            if (out_host) p.d2h_bytes += 3 * n * sizeof(float);
            t.run = c->runs.size();
            push_run(c->runs, static_cast<const uint16_t *>(ch.g16) + off, static_cast<uint16_t *>(ch.p16) + off,
                     dev[0], dev[1], dev[2], n, 0, p.adam_tile, (uint32_t)k);
            tiles.push_back(t);
        }
    }
    // host-resident chunks updated in place over the link: the kernel reads and writes pinned memory
    p.td = c->tune;
    p.td.adam_threads = 256; p.td.adam_unroll = c->tune.host_unroll; p.td.adam_wg_per_cu = 0;
    p.td.grid_override = c->tune.host_grid;
    const uint64_t direct_tile = adam_tile_elems(p.td);
    p.direct_off = c->runs.size();
    c->moves.clear();
    if (direct) {
        for (size_t k = 0; k < n_chunks; k++) {
            const psx_chunk &ch = chunks[k];
            if (ch.used == 0 || ch.loc_in != PSX_LOC_HOST || ch.loc_out != PSX_LOC_HOST || ch.exec == PSX_EXEC_CPU) continue;
            p.direct_tiles += push_run(c->runs, ch.g16, ch.p16, ch.p32_host, ch.m_host, ch.v_host, ch.used, p.direct_tiles, direct_tile, (uint32_t)k);
        }
        p.n_direct = c->runs.size() - p.direct_off;
        // chunks that change residence: read from the home they leave, written to the one they move to
        for (size_t k = 0; k < n_chunks; k++) {
            const psx_chunk &ch = chunks[k];
            if (ch.used == 0 || ch.loc_in == ch.loc_out) continue;
            const bool in_host = ch.loc_in == PSX_LOC_HOST;
            MoveRun r{};
            r.g16 = static_cast<const uint16_t *>(ch.g16);
            r.p16 = static_cast<uint16_t *>(ch.p16);
            r.p = static_cast<const float *>(in_host ? ch.p32_host : ch.p32);
            r.m = static_cast<const float *>(in_host ? ch.m_host : ch.m);
            r.v = static_cast<const float *>(in_host ? ch.v_host : ch.v);
            r.po = static_cast<float *>(in_host ? ch.p32 : ch.p32_host);
            r.mo = static_cast<float *>(in_host ? ch.m : ch.m_host);
            r.vo = static_cast<float *>(in_host ? ch.v : ch.v_host);
            r.n = ch.used; r.tile_begin = p.move_tiles; r.chunk = (uint32_t)k;
            c->moves.push_back(r);
            p.move_tiles += (ch.used + kMoveTileElems - 1) / kMoveTileElems;
        }
        // skipped step with the gradients in the fp16 parameter chunk: the parameters are cast back from
        // the home the states were read from (a skipped step leaves it valid)
        if (use_flag)
            for (size_t k = 0; k < n_chunks; k++) {
                const psx_chunk &ch = chunks[k];
                if (ch.used == 0 || (ch.loc_in == PSX_LOC_HBM && ch.loc_out == PSX_LOC_HBM) || ch.g16 != ch.p16 || ch.exec == PSX_EXEC_CPU) continue;
                const bool in_host = ch.loc_in == PSX_LOC_HOST;
                p.direct_recast_tiles += push_run(c->runs, ch.g16, ch.p16, in_host ? ch.p32_host : ch.p32, in_host ? ch.m_host : ch.m,
                                                in_host ? ch.v_host : ch.v, ch.used, p.direct_recast_tiles, p.recast_tile, (uint32_t)k);
            }
        p.n_direct_recast = c->runs.size() - p.direct_off - p.n_direct;
    }
}

// Where psx_chunk_adam_step_unpack is to leave the fp16 parameters besides the chunk list.
struct OutSpec {
    void *const *tensors;
    const psx_slot *slots;
    size_t n;
    uint64_t chunk_elems;
};

// The fused unpack runs inside the resident launch at its default shape: every chunk must stay in HBM.
int32_t validate_out(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks, const OutSpec &o) {
    const char *who = "psx_chunk_adam_step_unpack";
    if (o.chunk_elems == 0) return fail(PSX_EINVAL, "%s: chunk_elems is 0", who);
    if (o.n != 0 && (o.tensors == nullptr || o.slots == nullptr)) return fail(PSX_EINVAL, "%s: tensors/slots is NULL", who);
    if (o.n > c->cfg.max_tensors) return fail(PSX_ECAP, "%s: %zu tensors, context holds %llu", who, o.n, (unsigned long long)c->cfg.max_tensors);
    if (c->tune.adam_threads != 64 || c->tune.adam_unroll != 1)
        return fail(PSX_EINVAL, "%s: runs at the default launch shape only (PSX_TUNE_ADAM_THREADS 64, PSX_TUNE_ADAM_UNROLL 1)", who);
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.used == 0) continue;
        if (ch.loc_in != PSX_LOC_HBM || ch.loc_out != PSX_LOC_HBM || ch.exec != PSX_EXEC_GPU)
            return fail(PSX_EINVAL, "%s: chunk %zu: only chunks that stay in HBM and are updated by the GPU", who, k);
        if (ch.used > o.chunk_elems) return fail(PSX_EINVAL, "%s: chunk %zu uses more than chunk_elems elements", who, k);
    }
    const uint64_t total = (uint64_t)n_chunks * o.chunk_elems;
    for (size_t i = 0; i < o.n; i++) {
        const uint64_t sz = o.slots[i].numel;
        if (sz == 0) continue;
        if (o.tensors[i] == nullptr) return fail(PSX_EINVAL, "%s: tensor %zu is NULL", who, i);
        if (reinterpret_cast<uintptr_t>(o.tensors[i]) % 2) return fail(PSX_EALIGN, "%s: tensor %zu is not element-aligned", who, i);
        if (o.slots[i].offset > o.chunk_elems) return fail(PSX_EINVAL, "%s: slot %zu offset beyond the chunk", who, i);
        const uint64_t lin = (uint64_t)o.slots[i].chunk * o.chunk_elems + o.slots[i].offset;
        if (lin > total || sz > total - lin)
            return fail(PSX_EINVAL, "%s: slot %zu (chunk %u offset %llu numel %llu) runs past the chunk list", who, i,
                        o.slots[i].chunk, (unsigned long long)o.slots[i].offset, (unsigned long long)sz);
    }
    return PSX_OK;
}

// Cuts every tensor into its pieces per chunk, keeps what lies inside the chunk's used prefix (the update
// produces nothing behind it), orders the pieces by chunk and offset and refuses overlapping ones; then
// notes for each resident run (c->runs[0 .. n_res), ascending in chunk) where its pieces start.
int32_t build_out(psx_ctx *c, const psx_chunk *chunks, const OutSpec &o, size_t n_res) {
    c->outs.clear();
    for (size_t i = 0; i < o.n; i++) {
        const uint64_t sz = o.slots[i].numel;
        const uint64_t lin = (uint64_t)o.slots[i].chunk * o.chunk_elems + o.slots[i].offset;
        uint64_t done = 0;
        while (done < sz) {
            const uint64_t p = lin + done;
            const uint64_t ck = p / o.chunk_elems, off = p % o.chunk_elems;
            const uint64_t take = sz - done < o.chunk_elems - off ? sz - done : o.chunk_elems - off;
            const uint64_t used = chunks[ck].used;
            if (off < used) {
                OutSeg g;
                g.dst = static_cast<uint16_t *>(o.tensors[i]) + done;
                g.off = off;
                g.n = take < used - off ? take : used - off;
                g.pad = ck;                             // the chunk, for the ordering below; the kernel does not read it
                c->outs.push_back(g);
            }
            done += take;
        }
    }
    std::stable_sort(c->outs.begin(), c->outs.end(),
                     [](const OutSeg &a, const OutSeg &b) { return a.pad != b.pad ? a.pad < b.pad : a.off < b.off; });
    for (size_t j = 1; j < c->outs.size(); j++)
        if (c->outs[j].pad == c->outs[j - 1].pad && c->outs[j].off < c->outs[j - 1].off + c->outs[j - 1].n)
            return fail(PSX_EINVAL, "psx_chunk_adam_step_unpack: two slots overlap in chunk %llu", (unsigned long long)c->outs[j].pad);
    if (c->outs.size() > 0xFFFFFFFFull) return fail(PSX_ECAP, "psx_chunk_adam_step_unpack: too many output ranges");
    c->out_first.assign(n_res + 1, (uint32_t)c->outs.size());
    size_t j = 0;
    for (size_t r = 0; r < n_res; r++) {
        while (j < c->outs.size() && c->outs[j].pad < c->runs[r].chunk) j++;
        c->out_first[r] = (uint32_t)j;
    }
    return PSX_OK;
}

int32_t upload_out(psx_ctx *c, hipStream_t s, OutView *view) {
    const size_t nd = c->outs.size() * sizeof(OutSeg), nf = c->out_first.size() * sizeof(uint32_t);
    c->blob.resize(nd + nf);
    if (nd) memcpy(c->blob.data(), c->outs.data(), nd);
    memcpy(c->blob.data() + nd, c->out_first.data(), nf);
    const int32_t rc = table_upload(c->out_tbl, c->blob.data(), c->blob.size(), s);
    if (rc != PSX_OK) return rc;
    const unsigned char *base = static_cast<const unsigned char *>(c->out_tbl.dev);
    view->segs = reinterpret_cast<const OutSeg *>(base);
    view->first = reinterpret_cast<const uint32_t *>(base + nd);
    return PSX_OK;
}

int32_t adam_step_impl(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks, const psx_adam_hyper *hyper, uint32_t flags,
                       void *stream, const OutSpec *out);

}  // namespace

extern "C" int32_t psx_chunk_adam_step(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks,
                                       const psx_adam_hyper *hyper, uint32_t flags, void *stream) {
    return adam_step_impl(c, chunks, n_chunks, hyper, flags, stream, nullptr);
}

extern "C" int32_t psx_chunk_adam_step_unpack(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks,
                                              const psx_adam_hyper *hyper, uint32_t flags,
                                              void *const *p16_tensors, const psx_slot *slots, size_t n_tensors,
                                              uint64_t chunk_elems, void *stream) {
    const OutSpec out{p16_tensors, slots, n_tensors, chunk_elems};
    return adam_step_impl(c, chunks, n_chunks, hyper, flags, stream, &out);
}

namespace {

int32_t adam_step_impl(psx_ctx *c, const psx_chunk *chunks, size_t n_chunks, const psx_adam_hyper *hyper, uint32_t flags,
                       void *stream, const OutSpec *out) {
    if (c == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step: ctx is NULL");
    if (hyper == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step: hyper is NULL");
    if (n_chunks != 0 && chunks == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step: chunks is NULL");
    if (flags & ~(PSX_STEP_USE_FLAG | PSX_STEP_CHECK_FIRST | PSX_STEP_DEVICE_STATE)) return fail(PSX_EINVAL, "psx_chunk_adam_step: unknown flags 0x%x", flags);
    const bool dev_state = (flags & PSX_STEP_DEVICE_STATE) != 0;
    if (dev_state) {
        if (!c->state_on) return fail(PSX_EINVAL, "psx_chunk_adam_step: PSX_STEP_DEVICE_STATE needs psx_step_state_init first");
        const psx_adam_hyper &a = *hyper, &b = c->state_hyper;
        if (a.lr != b.lr || a.beta1 != b.beta1 || a.beta2 != b.beta2 || a.eps != b.eps || a.weight_decay != b.weight_decay ||
            (a.adamw_mode != 0) != (b.adamw_mode != 0))
            return fail(PSX_EINVAL, "psx_chunk_adam_step: with PSX_STEP_DEVICE_STATE lr, betas, eps, weight_decay and adamw_mode must be "
                                    "those given to psx_step_state_init (step and loss_scale are taken from the device)");
    }
    if (n_chunks > c->cfg.max_chunks)
        return fail(PSX_ECAP, "psx_chunk_adam_step: %zu chunks, context holds %llu", n_chunks, (unsigned long long)c->cfg.max_chunks);
    AdamScalars sc;
    int32_t rc = prepare_adam_scalars(hyper, "psx_chunk_adam_step", &sc);
    if (rc != PSX_OK) return rc;
    const bool check_first = (flags & PSX_STEP_CHECK_FIRST) != 0;
    const bool use_flag = check_first || (flags & PSX_STEP_USE_FLAG) != 0;
    // a stream that is being recorded into a graph: only what replays as kernel launches on that one stream
    const bool recording = capturing(static_cast<hipStream_t>(stream));
    if (recording && !dev_state)
        return fail(PSX_ECAPTURE, "psx_chunk_adam_step: a captured step would replay this call's t and loss scale for ever: use PSX_STEP_DEVICE_STATE");

    if ((rc = validate_step(c, chunks, n_chunks, dev_state, recording)) != PSX_OK) return rc;
    if (out != nullptr && (rc = validate_out(c, chunks, n_chunks, *out)) != PSX_OK) return rc;
    if ((rc = set_device_guard(c)) != PSX_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const AdamScalars *sc_dev = dev_state ? &c->state_dev->sc : nullptr;

    // ---- descriptors of everything this call launches, then their upload (a no-op when nothing changed)
    StepPlan pl;
    plan_step(c, chunks, n_chunks, use_flag, check_first, pl);
    std::vector<SpillTile> &tiles = c->spill_tiles;
    std::vector<CpuTile> &cpu_tiles = c->cpu_tiles;
    if (c->runs.size() > 0xFFFFFFFFull) return fail(PSX_ECAP, "psx_chunk_adam_step: too many runs");
    const AdamRun *tbl = nullptr;
    const uint64_t *tbl_begins = nullptr;
    if ((rc = upload_described(c->adam_tbl, c->runs, c->blob, s, &tbl, &tbl_begins)) != PSX_OK) return rc;
    const MoveRun *mtbl = nullptr;
    const uint64_t *mtbl_begins = nullptr;
    if (!c->moves.empty() && (rc = upload_described(c->move_tbl, c->moves, c->blob, s, &mtbl, &mtbl_begins)) != PSX_OK) return rc;
    auto view = [&](size_t off, size_t n) { return RunView{tbl + off, tbl_begins + off, (uint32_t)n}; };
    const uint32_t *flag = use_flag ? c->flags_dev : nullptr;
    // the fp16 tensors: written from inside the resident launch, or by an unpack launch behind it when most of
    // their memory is not aligned like their slots (tile pieces would end inside the tensors' 128-byte lines)
    OutView out_view{nullptr, nullptr};
    bool fuse_out = false;
    SegView unpack_view{nullptr, nullptr, 0, nullptr, 0};
    uint64_t unpack_tiles = 0;
    if (out != nullptr) {
        if ((rc = build_out(c, chunks, *out, pl.n_res)) != PSX_OK) return rc;
        uint64_t aligned = 0, covered = 0;
        for (const OutSeg &g : c->outs) {
            covered += g.n;
            if ((reinterpret_cast<uintptr_t>(g.dst) - 2 * g.off) % 128 == 0) aligned += g.n;
        }
        fuse_out = c->tune.fused_unpack == 1 || (c->tune.fused_unpack == 0 && 2 * aligned >= covered);
        if (fuse_out) {
            if ((rc = upload_out(c, s, &out_view)) != PSX_OK) return rc;
        } else {
            c->copy_unroll_now = copy_unroll_for(c->tune, c->outs.size());
            const uint64_t tile_elems = copy_tile_bytes(c->tune, c->copy_unroll_now) / 2;
            c->segs.clear();
            for (const OutSeg &g : c->outs) {
                CopySeg q;
                q.src = static_cast<const unsigned char *>(chunks[g.pad].p16) + g.off * 2;
                q.dst = reinterpret_cast<unsigned char *>(g.dst);
                q.n = g.n; q.tile_begin = unpack_tiles; q.chunk = (uint32_t)g.pad; q.pad = 0;
                c->segs.push_back(q);
                unpack_tiles += copy_tiles_of(q.dst, q.n, 2, tile_elems);
            }
            if (unpack_tiles != 0 &&
                (rc = upload_segments(c->unpack_tbl, c->segs, unpack_tiles, c->blob, s, &unpack_view.segs, &unpack_view.begins,
                                      &unpack_view.hints, &unpack_view.shift)) != PSX_OK)
                return rc;
            unpack_view.n = (uint32_t)c->segs.size();
        }
    }

    // ---- overflow check over every gradient chunk
    if (check_first) {
        PSX_HIP(launch_fill_u32(c->flags_dev, c->flags_n, 0u, s));
        if ((rc = span_begin(c, c->t_check, s)) != PSX_OK) return rc;
        PSX_HIP(launch_check(view(pl.n_res + pl.n_recast, pl.n_check), pl.check_tiles, c->flags_dev, c->flags_dev + 1, c->tune, c->n_cu, s));
        if ((rc = span_end(c, c->t_check, s)) != PSX_OK) return rc;
    }

    // ---- the side streams may start once earlier work on the caller's stream (and the check) is done
    const bool any_cpu = !cpu_tiles.empty();
    if (any_cpu && (rc = ensure_cpu(c)) != PSX_OK) return rc;
    const bool any_side = !tiles.empty() || pl.n_direct != 0 || pl.move_tiles != 0 || any_cpu;
    c->t_spill.valid = false;
    if (any_side) {
        PSX_HIP(hipEventRecord(c->ev_entry, s));
        PSX_HIP(hipStreamWaitEvent(c->h2d, c->ev_entry, 0));
        PSX_HIP(hipStreamWaitEvent(c->d2h, c->ev_entry, 0));
        if (any_cpu) PSX_HIP(hipStreamWaitEvent(c->aux, c->ev_entry, 0));
        if (c->prof) PSX_HIP(hipEventRecord(c->t_spill.a, c->h2d));
    }
    // the host cores need the flag's value: fetch it now, ahead of the resident launch
    if (any_cpu && use_flag) {
        PSX_HIP(hipMemcpyAsync(c->flags_host, c->flags_dev, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
        PSX_HIP(hipEventRecord(c->ev_flag, s));
    }

    // Everything from here on is enqueued inside one function, so that whatever it returns the side
    // streams are joined back into the caller's stream below: after an error part of the work may be
    // running on them, and the caller's next work on `stream` must still come after it.
    bool any_h2d = false, any_d2h = false;
    auto enqueue = [&]() -> int32_t {
        // ---- HBM-resident chunks: one launch over all of them
        c->adam_elems = pl.res_elems;
        c->t_adam.valid = false;
        if (pl.res_tiles != 0) {
            if ((rc = span_begin(c, c->t_adam, s)) != PSX_OK) return rc;
            if (fuse_out) PSX_HIP(launch_adam_out(view(0, pl.n_res), pl.res_tiles, sc, flag, c->tune, c->n_cu, s, sc_dev, out_view));
            else PSX_HIP(launch_adam(view(0, pl.n_res), pl.res_tiles, sc, flag, c->tune, c->n_cu, s, sc_dev));
            if ((rc = span_end(c, c->t_adam, s)) != PSX_OK) return rc;
            if (pl.n_recast != 0)
                PSX_HIP(launch_recast_if_flag(view(pl.n_res, pl.n_recast), pl.recast_tiles, flag, c->tune, c->n_cu, s));
            if (out != nullptr && !fuse_out && unpack_tiles != 0) {
                if ((rc = span_begin(c, c->t_unpack, s)) != PSX_OK) return rc;
                Tuning tn = c->tune;
                tn.copy_unroll = c->copy_unroll_now;
                PSX_HIP(launch_copy(unpack_view, unpack_tiles, 2u, nullptr, nullptr, tn, c->n_cu, s));
                if ((rc = span_end(c, c->t_unpack, s)) != PSX_OK) return rc;
            }
        }

        // ---- host-resident chunks, direct mode: one persistent launch on the side stream, concurrent with
        // the resident launch; every load and store of p/m/v crosses the host link once, in both directions at once
        c->spill_elems = pl.spill_elems; c->h2d_bytes = pl.h2d_bytes; c->d2h_bytes = pl.d2h_bytes;
        if (pl.n_direct != 0 || pl.move_tiles != 0) {
            if (pl.n_direct != 0)
                PSX_HIP(launch_adam(view(pl.direct_off, pl.n_direct), pl.direct_tiles, sc, flag, pl.td, c->n_cu, c->h2d, sc_dev));
            if (pl.move_tiles != 0)
                PSX_HIP(launch_adam_move(MoveView{mtbl, mtbl_begins, (uint32_t)c->moves.size()}, pl.move_tiles, sc, flag, c->tune,
                                         (uint32_t)c->tune.host_grid, c->h2d, sc_dev));
            if (pl.n_direct_recast != 0)
                PSX_HIP(launch_recast_if_flag(view(pl.direct_off + pl.n_direct, pl.n_direct_recast), pl.direct_recast_tiles, flag, pl.td, c->n_cu, c->h2d));
            any_h2d = true;
        }

        // ---- chunks with a host side, staged: H2D (copy stream) -> update (caller's stream) -> D2H (copy stream)
        const size_t ring = c->ev_k.size();
        for (size_t i = 0; i < tiles.size(); i++) {
            const SpillTile &t = tiles[i];
            const size_t e = i % ring;
            const size_t bytes = t.n * sizeof(float);
            if (t.src[0] != nullptr) {
                if (i >= ring) PSX_HIP(hipStreamWaitEvent(c->h2d, c->ev_free[e], 0));   // staging slot drained
                for (int j = 0; j < 3; j++)
                    PSX_HIP(hipMemcpyAsync(t.stage[j], t.src[j], bytes, hipMemcpyHostToDevice, c->h2d));
                PSX_HIP(hipEventRecord(c->ev_h2d[e], c->h2d));
                PSX_HIP(hipStreamWaitEvent(s, c->ev_h2d[e], 0));
                any_h2d = true;
            }
            Tuning tn = c->tune;
            PSX_HIP(launch_adam(view(t.run, 1), (t.n + pl.adam_tile - 1) / pl.adam_tile, sc, flag, tn, c->n_cu, s, sc_dev));
            if (use_flag && t.alias)
                PSX_HIP(launch_recast_if_flag(view(t.run, 1), (t.n + pl.recast_tile - 1) / pl.recast_tile, flag, tn, c->n_cu, s));
            if (t.dst[0] != nullptr) {
                PSX_HIP(hipEventRecord(c->ev_k[e], s));
                PSX_HIP(hipStreamWaitEvent(c->d2h, c->ev_k[e], 0));
                for (int j = 0; j < 3; j++)
                    PSX_HIP(hipMemcpyAsync(t.dst[j], t.stage[j], bytes, hipMemcpyDeviceToHost, c->d2h));
                PSX_HIP(hipEventRecord(c->ev_free[e], c->d2h));
                any_d2h = true;
            } else {
                PSX_HIP(hipEventRecord(c->ev_free[e], s));
            }
        }
        // ---- host-resident chunks executed by the host cores: everything above is already running on the GPU;
        // this thread now pipelines  D2H fp16 gradient tile -> update of p/m/v in place -> H2D fp16 parameter tile
        c->cpu_elems = pl.cpu_elems;
        c->cpu_ms = 0.0f;
        if (any_cpu) {
            bool skip = false;
            if (use_flag) {
                PSX_HIP(hipEventSynchronize(c->ev_flag));
                skip = c->flags_host[0] != 0;
            }
            if (skip) {                                   // nothing to update; aliased fp16 chunks get their params back
                size_t w = 0;
                for (size_t i = 0; i < cpu_tiles.size(); i++)
                    if (cpu_tiles[i].alias) cpu_tiles[w++] = cpu_tiles[i];
                cpu_tiles.resize(w);
            }
            PSX_HIP(hipEventSynchronize(c->ev_cpu_end));   // the previous call's uploads have left the staging
            const auto t0 = std::chrono::steady_clock::now();
            const size_t nt = cpu_tiles.size();
            size_t issued = 0;
            auto fetch = [&](size_t i) -> int32_t {
                const int slot = (int)(i % kCpuSlots);
                PSX_HIP(hipMemcpyAsync(c->cpu_g[slot], cpu_tiles[i].g16, cpu_tiles[i].n * 2, hipMemcpyDeviceToHost, c->d2h));
                PSX_HIP(hipEventRecord(c->ev_cg[slot], c->d2h));
                return PSX_OK;
            };
            if (!skip)
                for (; issued < nt && issued < (size_t)kCpuSlots; issued++)
                    if ((rc = fetch(issued)) != PSX_OK) return rc;
            for (size_t i = 0; i < nt; i++) {
                const CpuTile &t = cpu_tiles[i];
                const int slot = (int)(i % kCpuSlots);
                if (!skip) PSX_HIP(hipEventSynchronize(c->ev_cg[slot]));            // gradient tile has arrived
                if (i >= (size_t)kCpuSlots) PSX_HIP(hipEventSynchronize(c->ev_ch[slot]));   // parameter staging sent
                if (!skip) cpu_adam_tile(c->pool, c->cpu_g[slot], c->cpu_h[slot], t.p, t.m, t.v, t.n, sc, c->tune.cpu_isa);
                else cpu_recast_tile(c->pool, c->cpu_h[slot], t.p, t.n);
                PSX_HIP(hipMemcpyAsync(t.p16, c->cpu_h[slot], t.n * 2, hipMemcpyHostToDevice, c->aux));
                PSX_HIP(hipEventRecord(c->ev_ch[slot], c->aux));
                if (!skip && issued < nt) {               // this slot's gradient staging is free again
                    if ((rc = fetch(issued)) != PSX_OK) return rc;
                    issued++;
                }
            }
            PSX_HIP(hipEventRecord(c->ev_cpu_end, c->aux));
            PSX_HIP(hipStreamWaitEvent(s, c->ev_cpu_end, 0));
            any_d2h = true;
            c->cpu_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
        }
        return PSX_OK;
    };
    const int32_t rc_enqueue = enqueue();
    if (any_side) {
        // on the error path every side stream that may hold work is joined, whatever was reached
        const bool all = rc_enqueue != PSX_OK;
        int32_t rc_join = PSX_OK;
        auto join = [&](hipStream_t side, hipEvent_t ev) {
            hipError_t e = hipEventRecord(ev, side);
            if (e == hipSuccess) e = hipStreamWaitEvent(s, ev, 0);
            if (e != hipSuccess && rc_join == PSX_OK && rc_enqueue == PSX_OK)
                rc_join = fail(PSX_EHIP, "psx_chunk_adam_step: joining a side stream -> %s", hipGetErrorString(e));
        };
        if (any_h2d || all) join(c->h2d, c->ev_h2d_end);
        if (any_d2h || all) join(c->d2h, c->ev_d2h_end);
        if (all && any_cpu && c->aux != nullptr) join(c->aux, c->ev_cpu_end);
        if (rc_enqueue != PSX_OK) return rc_enqueue;
        if (rc_join != PSX_OK) return rc_join;
        if (c->prof) { PSX_HIP(hipEventRecord(c->t_spill.b, s)); c->t_spill.valid = true; }
    }
    return rc_enqueue;
}

}  // namespace
