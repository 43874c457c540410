// Internal declarations shared by the host runtime and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "psx.h"

namespace psx {

// ---- error reporting (thread-local message behind psx_last_error) ----
int32_t fail(int32_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
#define PSX_HIP(call)                                                                     \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess)                                                             \
            return ::psx::fail(PSX_EHIP, "%s -> %s (%s:%d)", #call, hipGetErrorString(e_), \
                               __FILE__, __LINE__);                                       \
    } while (0)

// ---- device-side descriptors ----

// One contiguous run of elements handled by the element-wise kernels.  Runs are
// cut into tiles; tile_begin is the index of the run's first tile in the launch.
struct AdamRun {
    const uint16_t *g16;
    uint16_t *p16;
    float *p, *m, *v;
    uint64_t n;
    uint64_t tile_begin;
    uint32_t chunk;      // index into the per-chunk overflow flags
    uint32_t pad;
};

// A run whose fp32 states change residence while they are updated: read from one
// home (p, m, v), written to the other (po, mo, vo); one of the two is pinned host
// memory.  The home read from is left as it was.
struct MoveRun {
    const uint16_t *g16;
    uint16_t *p16;
    const float *p, *m, *v;
    float *po, *mo, *vo;
    uint64_t n;
    uint64_t tile_begin;
    uint32_t chunk;
    uint32_t pad;
    uint64_t pad2;
};

struct CopySeg {
    const void *src;
    void *dst;
    uint64_t n;          // elements
    uint64_t tile_begin;
    uint32_t chunk;      // destination (pack) chunk index, for the fused overflow test
    uint32_t pad;
};

// Step-wide fp32 scalars of the Adam update, prepared on the host in double.
struct AdamScalars {
    float step_size, c2, inv_scale, beta1, beta2, omb1, omb2, eps, wd, decay;
    uint32_t decay_mode;   // 0 none, 1 L2 into the gradient, 2 decoupled
};

// The step state kept on the device for steps that take t and the loss scale from there (PSX_STEP_DEVICE_STATE):
// what psx_scaler holds on the host, the running products beta^t, and the scalars of the next update.
struct StepState {
    AdamScalars sc;            // scalars of the update with index `step`
    float scale;               // loss scale
    uint32_t growth_interval, good_steps;
    uint32_t last_flag;        // overflow flag of the step that was closed last (0 / 1)
    uint32_t pad;
    uint64_t step;             // t of the next update to apply
    uint64_t skipped;          // steps skipped so far
    double b1t, b2t;           // beta1^step, beta2^step as products of `step` factors
    double lr, beta1, beta2;
};

// Validates the hyper-parameters and derives the scalars (`who` names the entry point in messages).
int32_t prepare_adam_scalars(const psx_adam_hyper *h, const char *who, AdamScalars *s);

struct Tuning {
    int adam_threads = 64;         // 64 or 256 threads per workgroup
    int adam_unroll = 1;           // rows of 4 elements per thread
    int adam_blocks_per_cu = 0;    // 0: one tile per workgroup; >0: persistent grid-stride
    int adam_wg_per_cu = 14;       // cap on resident workgroups per CU (0: none)
    int nontemporal = 1;
    int copy_blocks_per_cu = 0;
    int copy_unroll = 0;           // 16-byte vectors per thread and tile of pack/unpack: 1 or 4; 0 = by tensor count
    int copy_threads = 64;         // threads per workgroup of pack/unpack: 64 or 256
    int host_mode = 1;             // host-resident chunks: 0 staged H2D/kernel/D2H, 1 kernel works on pinned memory
    int host_grid = 12;            // direct mode: persistent workgroups (256 threads) of the host launch: 12 keep
                                   // about 150 KB of reads in flight, the link's bandwidth-delay product; more
                                   // only queue up where the resident launch's HBM requests must pass
    int host_unroll = 1;           // direct mode: rows of 4 elements per thread
    int grid_override = 0;         // internal: absolute grid size of a launch (0: derive from blocks_per_cu)
    int lds_per_cu = 160 * 1024;   // internal: LDS bytes of one CU as the device reports them (what the occupancy cap divides)
    int cpu_threads = 0;           // PSX_EXEC_CPU: worker threads (0: min(hardware threads, 16))
    uint64_t cpu_tile_elems = 4u << 20;   // PSX_EXEC_CPU: elements per pipeline tile
    int cpu_isa = 0;               // PSX_EXEC_CPU: 0 widest vectors the host has (AVX-512 or AVX2), 1 AVX2
    int fused_unpack = 0;          // psx_chunk_adam_step_unpack: 0 by the alignment of the slots, 1 always inside the launch, 2 never
};

// Elements per tile of the Adam kernel (threads x 4 elements x unroll).
constexpr uint32_t kThreads = 256;
inline uint64_t adam_tile_elems(const Tuning &t) { return (uint64_t)t.adam_threads * 4u * (uint64_t)t.adam_unroll; }
constexpr uint64_t kRecastTileElems = (uint64_t)kThreads * 4u * 2u;
constexpr uint64_t kMoveTileElems = (uint64_t)kThreads * 4u;
constexpr uint64_t kCheckTileElems = (uint64_t)kThreads * 8u * 4u;   // 8192 fp16 per tile
// Small tiles of one wavefront copy fastest (measured: 6.7 TB/s against 6.3 with 256 threads).  Every tile pays one
// owner search; the coarse tile index (SegView::hints) keeps it to a lookup and a step or two even with thousands of
// tensors, so 1 KiB tiles win there as well (5000-tensor workload: 0.93 ms against 0.99 with 4 KiB tiles).
inline int copy_unroll_for(const Tuning &t, size_t) { return t.copy_unroll != 0 ? t.copy_unroll : 1; }
// Tiles of one copy segment (n elements of es bytes written to dst): a first tile of the elements in front
// of the destination's first kCopyCutBytes boundary, if any, then whole tiles from that boundary on, so that
// every whole tile writes whole 128-byte lines (a tile that starts in the middle of a line shares its first
// and last line with the tiles next to it, which run on other XCDs: two partial writes per line instead of
// one full one).  The copy kernel maps tile indices to elements by the same rule.
constexpr uint32_t kCopyCutBytes = 128;
inline uint64_t copy_head_elems(const void *dst, uint64_t n, uint32_t es) {
    const uint64_t a = ((kCopyCutBytes - (uint32_t)(reinterpret_cast<uintptr_t>(dst) & (kCopyCutBytes - 1u))) & (kCopyCutBytes - 1u)) / es;
    return a > n ? n : a;
}
inline uint64_t copy_tiles_of(const void *dst, uint64_t n, uint32_t es, uint64_t tile_elems) {
    const uint64_t a = copy_head_elems(dst, n, es);
    return (a != 0 ? 1u : 0u) + (n - a + tile_elems - 1) / tile_elems;
}
inline uint64_t copy_tile_bytes(const Tuning &t, int unroll) { return (uint64_t)(t.copy_threads == 64 ? 64 : 256) * 16u * (uint64_t)(unroll == 1 ? 1 : 4); }

// A section of a descriptor table on the device: n descriptors and, in a dense array of its own,
// the first tile of each (what the kernels search to find the owner of a tile).
struct RunView {
    const AdamRun *runs;
    const uint64_t *begins;
    uint32_t n;
};
struct MoveView {
    const MoveRun *runs;
    const uint64_t *begins;
    uint32_t n;
};
// One fp16 output range of the fused parameter unpack: elements [off, off + n) of a chunk go to dst[0, n).
struct OutSeg {
    uint16_t *dst;
    uint64_t off, n;
    uint64_t pad;
};
static_assert(sizeof(OutSeg) == 32, "descriptor size");
// The output ranges of every run of a RunView: those of run r are segs[first[r] .. first[r + 1]), ascending
// in `off` and disjoint (first has one entry more than there are runs).
struct OutView {
    const OutSeg *segs;
    const uint32_t *first;
};
struct SegView {
    const CopySeg *segs;
    const uint64_t *begins;
    uint32_t n;
    // coarse index over the tiles: hints[t >> shift] = owner of tile (t >> shift) << shift, one entry more
    // than there are groups (the last holds n - 1), so the owner of t lies in [hints[g], hints[g + 1]]
    const uint32_t *hints;
    uint32_t shift;
};
constexpr uint32_t kMaxHints = 4096;

// LDS bytes per CU of `device` as the runtime reports them; 160 KiB (gfx950) if it reports nothing usable.
int query_lds_per_cu(int device);

// ---- launchers (psx_kernels.hip).  All enqueue on `s` and return the launch status. ----
// sc_dev != NULL: the kernel takes its scalars from there (device memory) instead of `sc`; the decay mode,
// which selects the kernel, always comes from `sc`.
hipError_t launch_adam(const RunView &rv, uint64_t n_tiles,
                       const AdamScalars &sc, const uint32_t *flag_dev, const Tuning &t,
                       int n_cu, hipStream_t s, const AdamScalars *sc_dev = nullptr);
// The same update with the fp16 parameters written a second time, to the ranges of `out` (the tensors'
// own memory): psx_unpack without reading the chunk back.  Fixed launch shape: one wavefront per workgroup
// and tile of 256 elements; the runs' tile_begin must count tiles of that size.
hipError_t launch_adam_out(const RunView &rv, uint64_t n_tiles, const AdamScalars &sc, const uint32_t *flag_dev,
                           const Tuning &t, int n_cu, hipStream_t s, const AdamScalars *sc_dev, const OutView &out);
// Same update for runs that change residence, on `grid` persistent workgroups.  With *flag_dev != 0
// the states are copied to their new home unchanged and p16 is left alone.
hipError_t launch_adam_move(const MoveView &mv, uint64_t n_tiles, const AdamScalars &sc,
                            const uint32_t *flag_dev, const Tuning &t, uint32_t grid, hipStream_t s,
                            const AdamScalars *sc_dev = nullptr);
// Device-resident step state: write `init` and derive its scalars; close a step (loss-scale bookkeeping from
// flags_dev[0], then the scalars of the next update; n_clear != 0: the first n_clear flags are cleared once read).
hipError_t launch_step_state_init(StepState *st, const StepState &init, hipStream_t s);
hipError_t launch_step_state_advance(StepState *st, uint32_t *flags_dev, uint64_t n_clear, hipStream_t s);
// skipped step with p16 aliasing g16: p16 = fp16(p32), only when *flag_dev != 0
hipError_t launch_recast_if_flag(const RunView &rv, uint64_t n_tiles,
                                 const uint32_t *flag_dev, const Tuning &t, int n_cu, hipStream_t s);
hipError_t launch_check(const RunView &rv, uint64_t n_tiles,
                        uint32_t *flag_dev, uint32_t *per_chunk_dev, const Tuning &t, int n_cu,
                        hipStream_t s);
hipError_t launch_copy(const SegView &sv, uint64_t n_tiles,
                       uint32_t elem_size, uint32_t *flag_dev, uint32_t *per_chunk_dev,
                       const Tuning &t, int n_cu, hipStream_t s);
hipError_t launch_fill_u32(uint32_t *dst, uint64_t n, uint32_t value, hipStream_t s);
hipError_t launch_copy_bytes(void *dst, const void *src, uint64_t n_bytes, const Tuning &t,
                             int n_cu, hipStream_t s);

// ---- host-core Adam (psx_cpu.cpp) ----
struct CpuPool;
bool cpu_adam_supported();
CpuPool *cpu_pool_create(int n_threads);
void cpu_pool_destroy(CpuPool *p);
int cpu_pool_size(const CpuPool *p);
void cpu_adam_tile(CpuPool *pool, const uint16_t *g16, uint16_t *p16, float *p, float *m, float *v, size_t n,
                   const AdamScalars &s, int isa);
void cpu_recast_tile(CpuPool *pool, uint16_t *p16, const float *p, size_t n);

}  // namespace psx
