// psx_chunk_adam_step_noalloc: the Adam step over HBM-resident chunks for
// callers that cannot allocate.  Everything psx_chunk_adam_step keeps in
// memory a context allocated (the overflow flags and the run descriptor
// tables the kernels search) lives here in one file-scope device array; the
// descriptors travel to it as kernel arguments of a small writer kernel, so
// the call issues kernel launches and nothing else: no hipMalloc, no hipFree,
// no memcpy from pageable memory, no memset.
#include <mutex>

#include "psx_internal.h"

using namespace psx;

namespace {

constexpr uint32_t kMaxChunks = PSX_NOALLOC_MAX_CHUNKS;
constexpr int kMaxDevices = 64;
constexpr int kSections = 3;                       // resident runs, re-cast runs, check runs
constexpr uint32_t kBatch = 32;                    // descriptors per writer launch (2 KiB of kernel arguments)

// Layout of the scratch array: flags (global + one per chunk), then per section
// kMaxChunks descriptors, then per section kMaxChunks first-tile indices.
constexpr size_t kFlagsBytes = ((1 + (size_t)kMaxChunks) * sizeof(uint32_t) + 255) & ~(size_t)255;
constexpr size_t kRunsOff = kFlagsBytes;
constexpr size_t kBeginsOff = kRunsOff + (size_t)kSections * kMaxChunks * sizeof(AdamRun);
constexpr size_t kScratchBytes = kBeginsOff + (size_t)kSections * kMaxChunks * sizeof(uint64_t);
static_assert(kScratchBytes <= PSX_NOALLOC_SCRATCH_BYTES, "the header states the size of the array");
static_assert(sizeof(AdamRun) == 64, "descriptor size");

// One copy per GPU, at an address of its own on each; held until the process ends.
// Host code must never pass this name to a kernel: it goes through dev_state().ptr.
static __device__ __align__(256) unsigned char scratch[PSX_NOALLOC_SCRATCH_BYTES];

struct RunBatch {
    AdamRun r[kBatch];
};

// Writes n descriptors and, into the dense array the kernels search, their first tiles.
__global__ __launch_bounds__(64) void table_write_kernel(AdamRun *runs, uint64_t *begins, RunBatch b, uint32_t n) {
    const uint32_t i = threadIdx.x;
    if (i < n) {
        runs[i] = b.r[i];
        begins[i] = b.r[i].tile_begin;
    }
}

__global__ void flag_copy_kernel(uint32_t *dst, const uint32_t *src) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src != 0 ? 1u : 0u;
}

struct DevState {
    unsigned char *ptr = nullptr;   // this device's address of `scratch`
    int n_cu = 0;
    int lds_per_cu = 0;
};
DevState g_dev[kMaxDevices];
std::mutex g_mu;

// Once per device, with that device current: ask the runtime where this GPU keeps the array.
int32_t dev_state(int device, DevState *out) {
    if (device < 0 || device >= kMaxDevices) return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: device %d out of range", device);
    std::lock_guard<std::mutex> lock(g_mu);
    DevState &d = g_dev[device];
    if (d.ptr == nullptr) {
        void *p = nullptr;
        PSX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return fail(PSX_EHIP, "psx_chunk_adam_step_noalloc: hipGetSymbolAddress returned NULL");
        int n_cu = 0;
        PSX_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device));
        d.n_cu = n_cu > 0 ? n_cu : 256;
        d.lds_per_cu = query_lds_per_cu(device);
        d.ptr = static_cast<unsigned char *>(p);
    }
    *out = d;
    return PSX_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Collects descriptors of one section and sends them to the device table in batches.
struct SectionWriter {
    AdamRun *runs_dev;
    uint64_t *begins_dev;
    hipStream_t s;
    RunBatch batch;
    uint32_t in_batch = 0, written = 0;
    uint64_t tiles = 0;

    hipError_t flush() {
        if (in_batch == 0) return hipSuccess;
        hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(64), 0, s, runs_dev + written, begins_dev + written, batch, in_batch);
        written += in_batch;
        in_batch = 0;
        return hipGetLastError();
    }
    hipError_t push(const psx_chunk &ch, uint32_t chunk, uint64_t tile_elems) {
        AdamRun &r = batch.r[in_batch];
        r.g16 = static_cast<const uint16_t *>(ch.g16);
        r.p16 = static_cast<uint16_t *>(ch.p16);
        r.p = static_cast<float *>(ch.p32); r.m = static_cast<float *>(ch.m); r.v = static_cast<float *>(ch.v);
        r.n = ch.used; r.tile_begin = tiles; r.chunk = chunk; r.pad = 0;
        tiles += (ch.used + tile_elems - 1) / tile_elems;
        if (++in_batch == kBatch) return flush();
        return hipSuccess;
    }
};

}  // namespace

extern "C" int32_t psx_chunk_adam_step_noalloc(const psx_chunk *chunks, size_t n_chunks, const psx_adam_hyper *hyper,
                                               uint32_t flags, uint32_t *flag_out_dev, void *stream) {
    if (hyper == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: hyper is NULL");
    if (n_chunks != 0 && chunks == nullptr) return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: chunks is NULL");
    if (flags & ~PSX_STEP_CHECK_FIRST)
        return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: flags 0x%x: only PSX_STEP_CHECK_FIRST is known here "
                                "(there is no context whose flag an earlier call could have set)", flags);
    if (n_chunks > kMaxChunks)
        return fail(PSX_ECAP, "psx_chunk_adam_step_noalloc: %zu chunks, the static table holds %u", n_chunks, kMaxChunks);
    const bool check_first = (flags & PSX_STEP_CHECK_FIRST) != 0;
    if (flag_out_dev != nullptr && !check_first)
        return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: flag_out_dev needs PSX_STEP_CHECK_FIRST");
    AdamScalars sc;
    int32_t rc = prepare_adam_scalars(hyper, "psx_chunk_adam_step_noalloc", &sc);
    if (rc != PSX_OK) return rc;
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.loc_in != PSX_LOC_HBM || ch.loc_out != PSX_LOC_HBM || ch.exec != PSX_EXEC_GPU)
            return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: chunk %zu: only chunks that stay in HBM and are updated by the GPU", k);
        if (ch.used == 0) continue;
        if (!ch.g16 || !ch.p16 || !ch.p32 || !ch.m || !ch.v)
            return fail(PSX_EINVAL, "psx_chunk_adam_step_noalloc: chunk %zu has a NULL buffer", k);
        if (!aligned16(ch.g16) || !aligned16(ch.p16) || !aligned16(ch.p32) || !aligned16(ch.m) || !aligned16(ch.v))
            return fail(PSX_EALIGN, "psx_chunk_adam_step_noalloc: chunk %zu is not 16-byte aligned", k);
    }
    int device = -1;
    PSX_HIP(hipGetDevice(&device));
    DevState d;
    if ((rc = dev_state(device, &d)) != PSX_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t *flags_dev = reinterpret_cast<uint32_t *>(d.ptr);
    AdamRun *runs_dev = reinterpret_cast<AdamRun *>(d.ptr + kRunsOff);
    uint64_t *begins_dev = reinterpret_cast<uint64_t *>(d.ptr + kBeginsOff);
    Tuning tune;                                         // the library's default launch shapes
    tune.lds_per_cu = d.lds_per_cu;
    const uint64_t tile_elems[kSections] = {adam_tile_elems(tune), kRecastTileElems, kCheckTileElems};

    // ---- descriptor tables: every section is rewritten by every call (the array keeps the last call's content)
    SectionWriter w[kSections];
    for (int j = 0; j < kSections; j++) {
        w[j].runs_dev = runs_dev + (size_t)j * kMaxChunks;
        w[j].begins_dev = begins_dev + (size_t)j * kMaxChunks;
        w[j].s = s;
    }
    for (size_t k = 0; k < n_chunks; k++) {
        const psx_chunk &ch = chunks[k];
        if (ch.used == 0) continue;
        PSX_HIP(w[0].push(ch, (uint32_t)k, tile_elems[0]));
        if (check_first) {
            if (ch.g16 == ch.p16) PSX_HIP(w[1].push(ch, (uint32_t)k, tile_elems[1]));
            PSX_HIP(w[2].push(ch, (uint32_t)k, tile_elems[2]));
        }
    }
    for (int j = 0; j < kSections; j++) PSX_HIP(w[j].flush());
    auto view = [&](int j) { return RunView{w[j].runs_dev, w[j].begins_dev, w[j].written}; };

    // ---- overflow test over every gradient chunk; the flags must start at zero (no memset: a fill kernel)
    const uint32_t *flag = nullptr;
    if (check_first) {
        PSX_HIP(launch_fill_u32(flags_dev, 1 + (uint64_t)kMaxChunks, 0u, s));
        PSX_HIP(launch_check(view(2), w[2].tiles, flags_dev, flags_dev + 1, tune, d.n_cu, s));
        flag = flags_dev;
    }
    // ---- the update (skipped if the flag is set), then fp16(p32) into reused chunks on a skipped step
    PSX_HIP(launch_adam(view(0), w[0].tiles, sc, flag, tune, d.n_cu, s));
    if (check_first && w[1].written != 0)
        PSX_HIP(launch_recast_if_flag(view(1), w[1].tiles, flag, tune, d.n_cu, s));
    if (flag_out_dev != nullptr) {
        hipLaunchKernelGGL(flag_copy_kernel, dim3(1), dim3(64), 0, s, flag_out_dev, flags_dev);
        PSX_HIP(hipGetLastError());
    }
    return PSX_OK;
}
