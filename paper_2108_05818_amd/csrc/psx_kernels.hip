// HIP kernels for gfx950 (MI355X): fused chunk Adam, overflow check,
// multi-tensor pack/unpack copy.  All of them are streaming, HBM-bound
// element-wise passes: 64-wide wavefronts issue one 16-byte (fp32) or 8-byte
// (fp16) access per lane and instruction, so every instruction of a wavefront
// covers one contiguous 1 KiB / 512 B span; no LDS and no matrix cores are
// involved because nothing is reused or contracted.
//
// Floating-point discipline (the results are compared bit for bit with a
// scalar CPU statement of the same formulas): no contraction into fused
// multiply-add, IEEE-correct division and square root (hipcc's default for
// HIP), denormals kept, round-to-nearest-even conversions.
#include "psx_internal.h"

#pragma clang fp contract(off)

namespace psx {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

// Pointers read from a descriptor table are generic; every buffer of this
// library is global memory, and saying so lets the compiler emit global_load /
// global_store instead of flat accesses.
#define PSX_GLOBAL __attribute__((address_space(1)))
template <typename V, typename T>
__device__ __forceinline__ const PSX_GLOBAL V *gptr(const T *p) {
    return (const PSX_GLOBAL V *)(p);
}
template <typename V, typename T>
__device__ __forceinline__ PSX_GLOBAL V *gptr(T *p) {
    return (PSX_GLOBAL V *)(p);
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const PSX_GLOBAL T *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(PSX_GLOBAL T *p, T v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Index of the run (or segment) that owns `tile`: the last one whose first
// tile is <= tile.  The first tiles are kept in a dense array of their own
// (8 bytes per run) so that the search stays inside a few cache lines of the
// scalar cache even with hundreds of runs; searching through the 64-byte
// descriptors instead touches one line per probe and, past a few dozen runs,
// misses the 16 KiB scalar cache on every step (measured: -13 % bandwidth at
// 193 chunks).  Uniform across the workgroup, so the loads are scalar.
__device__ __forceinline__ uint32_t find_owner(const uint64_t *__restrict__ begins, uint32_t n, uint64_t tile) {
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (begins[mid] <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

// The same with a coarse index in front: hints[g] is the owner of the first tile of group g = tile >> shift and
// hints[g + 1] that of the next group's (the last entry is n - 1), so only the few entries between them are searched.
__device__ __forceinline__ uint32_t find_owner_hinted(const uint64_t *__restrict__ begins, const uint32_t *__restrict__ hints,
                                                      uint32_t shift, uint64_t tile) {
    const uint64_t g = tile >> shift;
    uint32_t lo = hints[g], hi = hints[g + 1] + 1;
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (begins[mid] <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

// ------------------------------------------------------------------ Adam

// One element of the update: the formulas of include/psx.h as they stand there.  Contraction is off
// for this file, so every product, sum, quotient and root below is rounded to fp32 on its own, in
// the order the parentheses give.  gs is the fp16 gradient converted to fp32 (exact), still scaled.
template <int DM>
__device__ __forceinline__ void adam_elem(float gs, float &p, float &m, float &v,
                                          const AdamScalars &s) {
    float g = gs * s.inv_scale;
    if constexpr (DM == 1) g = g + s.wd * p;             // L2 decay enters through the gradient
    if constexpr (DM == 2) p = p * s.decay;              // decoupled decay shrinks the parameter first
    m = s.beta1 * m + s.omb1 * g;
    v = s.beta2 * v + (s.omb2 * g) * g;
    p = p - s.step_size * (m / (__builtin_sqrtf(v) * s.c2 + s.eps));
}

// T threads per workgroup, U rows of 4 elements per thread: a tile is T*4*U
// elements of every stream.  Small tiles dispatched in order (one tile per
// workgroup) keep the window of addresses the chip works on compact, which is
// what the HBM controllers reward; the launch may also reserve LDS it never
// touches, only to cap the workgroups resident per CU (see launch_adam).
template <int T, int U, bool NT, int DM>
__global__ __launch_bounds__(T) void adam_kernel(const AdamRun *__restrict__ runs,
                                                 const uint64_t *__restrict__ begins,
                                                 uint32_t n_runs, uint64_t n_tiles,
                                                 AdamScalars sc,
                                                 const AdamScalars *__restrict__ sc_dev,
                                                 const uint32_t *__restrict__ flag) {
    if (flag != nullptr && *flag != 0) return;          // overflow: the whole step is skipped
    if (sc_dev != nullptr) sc = *sc_dev;                // step-wide scalars kept on the device (uniform: scalar loads)
    constexpr uint32_t ROW = T * 4;
    constexpr uint32_t TILE = ROW * U;
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner(begins, n_runs, tile);
        const uint16_t *g16 = runs[r].g16;
        uint16_t *p16 = runs[r].p16;
        float *pp = runs[r].p, *pm = runs[r].m, *pv = runs[r].v;
        const uint64_t n = runs[r].n;
        const uint64_t base = (tile - runs[r].tile_begin) * TILE;
        if (n - base >= TILE) {
            f16x4 g[U];
            f32x4 p[U], m[U], v[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint64_t i = base + (uint64_t)u * ROW + tid * 4;
                g[u] = ld<NT>(gptr<f16x4>(g16 + i));
                p[u] = ld<NT>(gptr<f32x4>(pp + i));
                m[u] = ld<NT>(gptr<f32x4>(pm + i));
                v[u] = ld<NT>(gptr<f32x4>(pv + i));
            }
            f16x4 h[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    float pk = p[u][k], mk = m[u][k], vk = v[u][k];
                    adam_elem<DM>((float)g[u][k], pk, mk, vk, sc);
                    p[u][k] = pk; m[u][k] = mk; v[u][k] = vk;
                    h[u][k] = (_Float16)pk;
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                const uint64_t i = base + (uint64_t)u * ROW + tid * 4;
                st<NT>(gptr<f32x4>(pp + i), p[u]);
                st<NT>(gptr<f32x4>(pm + i), m[u]);
                st<NT>(gptr<f32x4>(pv + i), v[u]);
                st<NT>(gptr<f16x4>(p16 + i), h[u]);
            }
        } else {
            // last, partial tile of a run: whole groups of 4 as above, then a scalar tail
            for (int u = 0; u < U; u++) {
                const uint64_t i = base + (uint64_t)u * ROW + tid * 4;
                if (i + 4 <= n) {
                    f16x4 g = *gptr<f16x4>(g16 + i);
                    f32x4 p = *gptr<f32x4>(pp + i);
                    f32x4 m = *gptr<f32x4>(pm + i);
                    f32x4 v = *gptr<f32x4>(pv + i);
                    f16x4 h;
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        float pk = p[k], mk = m[k], vk = v[k];
                        adam_elem<DM>((float)g[k], pk, mk, vk, sc);
                        p[k] = pk; m[k] = mk; v[k] = vk;
                        h[k] = (_Float16)pk;
                    }
                    *gptr<f32x4>(pp + i) = p;
                    *gptr<f32x4>(pm + i) = m;
                    *gptr<f32x4>(pv + i) = v;
                    *gptr<f16x4>(p16 + i) = h;
                } else {
                    for (uint64_t k = i; k < n; k++) {
                        float pk = *gptr<float>(pp + k), mk = *gptr<float>(pm + k), vk = *gptr<float>(pv + k);
                        _Float16 gk = *gptr<_Float16>(g16 + k);
                        adam_elem<DM>((float)gk, pk, mk, vk, sc);
                        *gptr<float>(pp + k) = pk; *gptr<float>(pm + k) = mk; *gptr<float>(pv + k) = vk;
                        *gptr<_Float16>(p16 + k) = (_Float16)pk;
                    }
                }
            }
        }
    }
}

template <int T, int U, bool NT>
static hipError_t launch_adam_dm(const RunView &rv, uint64_t n_tiles,
                                 const AdamScalars &sc, const AdamScalars *sc_dev, const uint32_t *flag, uint32_t grid,
                                 uint32_t lds, hipStream_t s) {
    switch (sc.decay_mode) {
        case 0: hipLaunchKernelGGL((adam_kernel<T, U, NT, 0>), dim3(grid), dim3(T), lds, s, rv.runs, rv.begins, rv.n, n_tiles, sc, sc_dev, flag); break;
        case 1: hipLaunchKernelGGL((adam_kernel<T, U, NT, 1>), dim3(grid), dim3(T), lds, s, rv.runs, rv.begins, rv.n, n_tiles, sc, sc_dev, flag); break;
        default: hipLaunchKernelGGL((adam_kernel<T, U, NT, 2>), dim3(grid), dim3(T), lds, s, rv.runs, rv.begins, rv.n, n_tiles, sc, sc_dev, flag); break;
    }
    return hipGetLastError();
}

template <int T, bool NT>
static hipError_t launch_adam_u(int unroll, const RunView &rv, uint64_t n_tiles,
                                const AdamScalars &sc, const AdamScalars *sc_dev, const uint32_t *flag, uint32_t grid,
                                uint32_t lds, hipStream_t s) {
    switch (unroll) {
        case 1: return launch_adam_dm<T, 1, NT>(rv, n_tiles, sc, sc_dev, flag, grid, lds, s);
        case 4: return launch_adam_dm<T, 4, NT>(rv, n_tiles, sc, sc_dev, flag, grid, lds, s);
        default: return launch_adam_dm<T, 2, NT>(rv, n_tiles, sc, sc_dev, flag, grid, lds, s);
    }
}

// Bytes of LDS to reserve per workgroup so that at most wg_per_cu workgroups
// fit the LDS of a CU (0 = no cap).  The kernels never touch it.
static uint32_t throttle_lds(int wg_per_cu, int lds_per_cu) {
    if (wg_per_cu <= 0) return 0;
    uint32_t bytes = ((uint32_t)lds_per_cu / (uint32_t)wg_per_cu) & ~511u;
    if (bytes > 64u * 1024u - 512u) bytes = 64u * 1024u - 512u;   // stay under the 64 KiB a launch may ask for by default
    return bytes;
}

int query_lds_per_cu(int device) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device) != hipSuccess) {
        (void)hipGetLastError();
        v = 0;
    }
    // a CU's LDS is never smaller than what one workgroup may use (64 KiB); anything below that is not a
    // per-CU figure, and the chip this library is written for has 160 KiB
    return v >= 64 * 1024 ? v : 160 * 1024;
}

// blocks_per_cu == 0: one tile per workgroup, handed out in order by the dispatcher.
static uint32_t grid_for(uint64_t n_tiles, int blocks_per_cu, int n_cu) {
    uint64_t cap = blocks_per_cu > 0 ? (uint64_t)blocks_per_cu * (uint64_t)n_cu : 0x7FFFFFFFull;
    if (cap > 0x7FFFFFFFull) cap = 0x7FFFFFFFull;
    uint64_t g = n_tiles < cap ? n_tiles : cap;
    return (uint32_t)(g ? g : 1);
}

hipError_t launch_adam(const RunView &rv, uint64_t n_tiles, const AdamScalars &sc,
                       const uint32_t *flag, const Tuning &t, int n_cu, hipStream_t s, const AdamScalars *sc_dev) {
    if (n_tiles == 0) return hipSuccess;
    const uint32_t grid = t.grid_override > 0 ? (uint32_t)(n_tiles < (uint64_t)t.grid_override ? n_tiles : (uint64_t)t.grid_override)
                                              : grid_for(n_tiles, t.adam_blocks_per_cu, n_cu);
    const uint32_t lds = throttle_lds(t.adam_wg_per_cu, t.lds_per_cu);
    const bool nt = t.nontemporal != 0;
    if (t.adam_threads == 64)
        return nt ? launch_adam_u<64, true>(t.adam_unroll, rv, n_tiles, sc, sc_dev, flag, grid, lds, s)
                  : launch_adam_u<64, false>(t.adam_unroll, rv, n_tiles, sc, sc_dev, flag, grid, lds, s);
    return nt ? launch_adam_u<256, true>(t.adam_unroll, rv, n_tiles, sc, sc_dev, flag, grid, lds, s)
              : launch_adam_u<256, false>(t.adam_unroll, rv, n_tiles, sc, sc_dev, flag, grid, lds, s);
}

// ------------------------------------------------------------------ Adam with the fp16 unpack fused in
// adam_kernel's update (one wavefront, one tile of 256 elements, one row) that stores the fp16 parameters
// twice: into the param fp16 chunk and into the tensors' own memory, found through the run's output
// ranges.  A tile that lies inside one range takes one more 8-byte store per lane (shifted across lanes
// first if the destination is off the 8-byte grid); a tile that spans tensors writes its elements one by
// one, each lane walking on from the tile's first range.
__device__ __forceinline__ void scatter_f16(const OutSeg *__restrict__ segs, uint32_t s, uint32_t s_end,
                                            uint64_t e0, uint32_t cnt, const _Float16 *vals) {
    for (uint32_t k = 0; k < cnt; k++) {
        const uint64_t e = e0 + k;
        while (s < s_end && e >= segs[s].off + segs[s].n) s++;
        if (s < s_end && e >= segs[s].off) *gptr<_Float16>(segs[s].dst + (e - segs[s].off)) = vals[k];
    }
}

template <bool NT, int DM>
__global__ __launch_bounds__(64) void adam_out_kernel(const AdamRun *__restrict__ runs,
                                                      const uint64_t *__restrict__ begins,
                                                      uint32_t n_runs, uint64_t n_tiles,
                                                      AdamScalars sc,
                                                      const AdamScalars *__restrict__ sc_dev,
                                                      const uint32_t *__restrict__ flag,
                                                      const OutSeg *__restrict__ segs,
                                                      const uint32_t *__restrict__ first) {
    if (flag != nullptr && *flag != 0) return;          // overflow: nothing is updated and nothing is written
    if (sc_dev != nullptr) sc = *sc_dev;
    constexpr uint32_t TILE = 256;
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner(begins, n_runs, tile);
        const uint16_t *g16 = runs[r].g16;
        uint16_t *p16 = runs[r].p16;
        float *pp = runs[r].p, *pm = runs[r].m, *pv = runs[r].v;
        const uint64_t n = runs[r].n;
        const uint64_t base = (tile - runs[r].tile_begin) * TILE;
        // the first output range of this run that ends behind the tile's first element (uniform: scalar loads)
        const uint32_t s_end = first[r + 1];
        uint32_t lo = first[r], hi = s_end;
        while (lo < hi) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (segs[mid].off + segs[mid].n > base) hi = mid;
            else lo = mid + 1;
        }
        const uint32_t s0 = lo;
        const uint64_t i = base + tid * 4;
        if (n - base >= TILE) {
            const f16x4 g = ld<NT>(gptr<f16x4>(g16 + i));
            f32x4 p = ld<NT>(gptr<f32x4>(pp + i));
            f32x4 m = ld<NT>(gptr<f32x4>(pm + i));
            f32x4 v = ld<NT>(gptr<f32x4>(pv + i));
            f16x4 h;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                float pk = p[k], mk = m[k], vk = v[k];
                adam_elem<DM>((float)g[k], pk, mk, vk, sc);
                p[k] = pk; m[k] = mk; v[k] = vk;
                h[k] = (_Float16)pk;
            }
            st<NT>(gptr<f32x4>(pp + i), p);
            st<NT>(gptr<f32x4>(pm + i), m);
            st<NT>(gptr<f32x4>(pv + i), v);
            st<NT>(gptr<f16x4>(p16 + i), h);
            uint16_t *dst = nullptr;                    // where the tile's first element goes, if one range holds the whole tile
            if (s0 < s_end) {
                const uint64_t off = segs[s0].off, cnt = segs[s0].n;
                if (off <= base && base + TILE <= off + cnt) dst = segs[s0].dst + (base - off);
            }
            if (dst != nullptr) {
                const uint32_t a = (4u - ((uint32_t)(reinterpret_cast<uintptr_t>(dst) >> 1) & 3u)) & 3u;   // elements up to the first 8-byte boundary
                if (a == 0) {
                    st<NT>(gptr<f16x4>(dst + tid * 4), h);
                } else {
                    // The destination is off by a elements (uniform for the tile): the 8-byte word behind the
                    // boundary in front of lane j's last 4 - a elements is made of those and of the first a
                    // elements of lane j + 1, handed over by a wavefront shift.  Lane 0 also writes the a
                    // elements in front of the first boundary, lane 63 its last 4 - a, one by one.
                    const u16x4 hb = __builtin_bit_cast(u16x4, h);
                    const uint32_t w0 = (uint32_t)hb[0] | ((uint32_t)hb[1] << 16), w1 = (uint32_t)hb[2] | ((uint32_t)hb[3] << 16);
                    const uint32_t n0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w0, 0x130, 0xf, 0xf, false);
                    const uint32_t n1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w1, 0x130, 0xf, 0xf, false);
                    uint32_t o0, o1;
                    if (a == 1) { o0 = __builtin_amdgcn_alignbyte(w1, w0, 2); o1 = __builtin_amdgcn_alignbyte(n0, w1, 2); }
                    else if (a == 2) { o0 = w1; o1 = n0; }
                    else { o0 = __builtin_amdgcn_alignbyte(n0, w1, 2); o1 = __builtin_amdgcn_alignbyte(n1, n0, 2); }
                    uint16_t *mine = dst + tid * 4;
                    if (tid != 63) {
                        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                        const u32x2 word = {o0, o1};
                        st<NT>(gptr<u32x2>(mine + a), word);
                    } else {
                        for (uint32_t k = a; k < 4; k++) *gptr<uint16_t>(mine + k) = hb[k];
                    }
                    if (tid == 0)
                        for (uint32_t k = 0; k < a; k++) *gptr<uint16_t>(mine + k) = hb[k];
                }
            } else {
                const _Float16 vals[4] = {h[0], h[1], h[2], h[3]};
                scatter_f16(segs, s0, s_end, i, 4, vals);
            }
        } else if (i < n) {
            // last, partial tile of a run: element by element
            const uint32_t cnt = n - i < 4 ? (uint32_t)(n - i) : 4u;
            _Float16 vals[4];
            for (uint32_t k = 0; k < cnt; k++) {
                float pk = *gptr<float>(pp + i + k), mk = *gptr<float>(pm + i + k), vk = *gptr<float>(pv + i + k);
                const _Float16 gk = *gptr<_Float16>(g16 + i + k);
                adam_elem<DM>((float)gk, pk, mk, vk, sc);
                *gptr<float>(pp + i + k) = pk; *gptr<float>(pm + i + k) = mk; *gptr<float>(pv + i + k) = vk;
                vals[k] = (_Float16)pk;
                *gptr<_Float16>(p16 + i + k) = vals[k];
            }
            scatter_f16(segs, s0, s_end, i, cnt, vals);
        }
    }
}

hipError_t launch_adam_out(const RunView &rv, uint64_t n_tiles, const AdamScalars &sc, const uint32_t *flag,
                           const Tuning &t, int n_cu, hipStream_t s, const AdamScalars *sc_dev, const OutView &out) {
    if (n_tiles == 0) return hipSuccess;
    const uint32_t grid = grid_for(n_tiles, t.adam_blocks_per_cu, n_cu);
    const uint32_t lds = throttle_lds(t.adam_wg_per_cu, t.lds_per_cu);
#define PSX_LAUNCH_OUT(NT_, DM_)                                                                                   \
    hipLaunchKernelGGL((adam_out_kernel<NT_, DM_>), dim3(grid), dim3(64), lds, s, rv.runs, rv.begins, rv.n, n_tiles, \
                       sc, sc_dev, flag, out.segs, out.first)
    if (t.nontemporal != 0) {
        switch (sc.decay_mode) {
            case 0: PSX_LAUNCH_OUT(true, 0); break;
            case 1: PSX_LAUNCH_OUT(true, 1); break;
            default: PSX_LAUNCH_OUT(true, 2); break;
        }
    } else {
        switch (sc.decay_mode) {
            case 0: PSX_LAUNCH_OUT(false, 0); break;
            case 1: PSX_LAUNCH_OUT(false, 1); break;
            default: PSX_LAUNCH_OUT(false, 2); break;
        }
    }
#undef PSX_LAUNCH_OUT
    return hipGetLastError();
}

// ------------------------------------------------------------------ Adam on runs that change residence
// The fp32 states are read from the home they leave and written to the home
// they move to, so each crosses the host link once and no copy comes before or
// after.  Meant for a few persistent workgroups: the link, not HBM, is the
// bound.  On a skipped step the states still move, unchanged.
template <bool NT, int DM>
__global__ __launch_bounds__(kThreads) void adam_move_kernel(const MoveRun *__restrict__ runs,
                                                             const uint64_t *__restrict__ begins,
                                                             uint32_t n_runs, uint64_t n_tiles,
                                                             AdamScalars sc,
                                                             const AdamScalars *__restrict__ sc_dev,
                                                             const uint32_t *__restrict__ flag) {
    const bool skip = flag != nullptr && *flag != 0;
    if (sc_dev != nullptr) sc = *sc_dev;
    constexpr uint32_t TILE = kThreads * 4;
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner(begins, n_runs, tile);
        const uint16_t *g16 = runs[r].g16;
        uint16_t *p16 = runs[r].p16;
        const float *pp = runs[r].p, *pm = runs[r].m, *pv = runs[r].v;
        float *po = runs[r].po, *mo = runs[r].mo, *vo = runs[r].vo;
        const uint64_t n = runs[r].n;
        const uint64_t i = (tile - runs[r].tile_begin) * TILE + tid * 4;
        if (i + 4 <= n) {
            f32x4 p = ld<NT>(gptr<f32x4>(pp + i));
            f32x4 m = ld<NT>(gptr<f32x4>(pm + i));
            f32x4 v = ld<NT>(gptr<f32x4>(pv + i));
            if (!skip) {
                const f16x4 g = ld<NT>(gptr<f16x4>(g16 + i));
                f16x4 h;
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    float pk = p[k], mk = m[k], vk = v[k];
                    adam_elem<DM>((float)g[k], pk, mk, vk, sc);
                    p[k] = pk; m[k] = mk; v[k] = vk;
                    h[k] = (_Float16)pk;
                }
                st<NT>(gptr<f16x4>(p16 + i), h);
            }
            st<NT>(gptr<f32x4>(po + i), p);
            st<NT>(gptr<f32x4>(mo + i), m);
            st<NT>(gptr<f32x4>(vo + i), v);
        } else {
            for (uint64_t k = i; k < n; k++) {
                float pk = *gptr<float>(pp + k), mk = *gptr<float>(pm + k), vk = *gptr<float>(pv + k);
                if (!skip) {
                    const _Float16 gk = *gptr<_Float16>(g16 + k);
                    adam_elem<DM>((float)gk, pk, mk, vk, sc);
                    *gptr<_Float16>(p16 + k) = (_Float16)pk;
                }
                *gptr<float>(po + k) = pk; *gptr<float>(mo + k) = mk; *gptr<float>(vo + k) = vk;
            }
        }
    }
}

template <bool NT>
static hipError_t launch_adam_move_nt(const MoveView &mv, uint64_t n_tiles, const AdamScalars &sc,
                                      const AdamScalars *sc_dev, const uint32_t *flag, uint32_t grid, hipStream_t s) {
    switch (sc.decay_mode) {
        case 0: hipLaunchKernelGGL((adam_move_kernel<NT, 0>), dim3(grid), dim3(kThreads), 0, s, mv.runs, mv.begins, mv.n, n_tiles, sc, sc_dev, flag); break;
        case 1: hipLaunchKernelGGL((adam_move_kernel<NT, 1>), dim3(grid), dim3(kThreads), 0, s, mv.runs, mv.begins, mv.n, n_tiles, sc, sc_dev, flag); break;
        default: hipLaunchKernelGGL((adam_move_kernel<NT, 2>), dim3(grid), dim3(kThreads), 0, s, mv.runs, mv.begins, mv.n, n_tiles, sc, sc_dev, flag); break;
    }
    return hipGetLastError();
}

hipError_t launch_adam_move(const MoveView &mv, uint64_t n_tiles, const AdamScalars &sc,
                            const uint32_t *flag, const Tuning &t, uint32_t grid, hipStream_t s,
                            const AdamScalars *sc_dev) {
    if (n_tiles == 0) return hipSuccess;
    if (grid == 0) grid = 1;
    if ((uint64_t)grid > n_tiles) grid = (uint32_t)n_tiles;
    return t.nontemporal ? launch_adam_move_nt<true>(mv, n_tiles, sc, sc_dev, flag, grid, s)
                         : launch_adam_move_nt<false>(mv, n_tiles, sc, sc_dev, flag, grid, s);
}

// ------------------------------------------------------------------ re-cast on a skipped step
// Runs with the same tiling as the Adam kernel (unroll 2).  Does work only when the
// overflow flag is set: the fp16 chunk, which held gradients, receives fp16(p32).
__global__ __launch_bounds__(kThreads) void recast_kernel(const AdamRun *__restrict__ runs,
                                                          const uint64_t *__restrict__ begins,
                                                          uint32_t n_runs, uint64_t n_tiles,
                                                          const uint32_t *__restrict__ flag) {
    if (*flag == 0) return;
    constexpr uint32_t ROW = kThreads * 4;
    constexpr uint32_t TILE = ROW * 2;
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner(begins, n_runs, tile);
        uint16_t *p16 = runs[r].p16;
        const float *pp = runs[r].p;
        const uint64_t n = runs[r].n;
        const uint64_t base = (tile - runs[r].tile_begin) * TILE;
        for (int u = 0; u < 2; u++) {
            const uint64_t i = base + (uint64_t)u * ROW + tid * 4;
            if (i + 4 <= n) {
                f32x4 p = *gptr<f32x4>(pp + i);
                f16x4 h;
#pragma unroll
                for (int k = 0; k < 4; k++) h[k] = (_Float16)p[k];
                *gptr<f16x4>(p16 + i) = h;
            } else {
                for (uint64_t k = i; k < n; k++)
                    *gptr<_Float16>(p16 + k) = (_Float16)*gptr<float>(pp + k);
            }
        }
    }
}

hipError_t launch_recast_if_flag(const RunView &rv, uint64_t n_tiles,
                                 const uint32_t *flag, const Tuning &t, int n_cu, hipStream_t s) {
    if (n_tiles == 0) return hipSuccess;
    // A persistent grid: on all steps but the rare skipped one every workgroup only reads the flag and leaves, and a
    // launch of one workgroup per tile would spend 0.1 ms per 10^9 elements on that.
    const uint64_t cap = t.grid_override > 0 ? (uint64_t)t.grid_override : (uint64_t)n_cu * 16u;
    const uint32_t grid = (uint32_t)(n_tiles < cap ? n_tiles : cap);
    hipLaunchKernelGGL(recast_kernel, dim3(grid), dim3(kThreads), 0, s, rv.runs, rv.begins, rv.n, n_tiles, flag);
    return hipGetLastError();
}

// ------------------------------------------------------------------ overflow check
// A 32-bit word holds two fp16 values; one of them is inf/nan iff its five exponent bits are all set.
__device__ __forceinline__ uint32_t word_has_infnan(uint32_t w) {
    const uint32_t t = w & 0x7C007C00u;
    return (uint32_t)((t & 0xFFFFu) == 0x7C00u) | (uint32_t)((t >> 16) == 0x7C00u);
}
__device__ __forceinline__ uint32_t half_is_infnan(uint16_t h) { return (h & 0x7C00u) == 0x7C00u; }

// A wavefront that saw an inf/nan raises the global and the per-chunk flag once
// (ballot, then lane 0 writes); in the common all-finite case nothing is written.
__device__ __forceinline__ void raise_flags(uint32_t bad, uint32_t *flag, uint32_t *per_chunk,
                                            uint32_t chunk) {
    const unsigned long long b = __ballot(bad != 0);
    if (b != 0 && (threadIdx.x & 63u) == 0) {
        atomicOr(flag, 1u);
        if (per_chunk != nullptr) atomicOr(per_chunk + chunk, 1u);
    }
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void check_kernel(const AdamRun *__restrict__ runs,
                                                         const uint64_t *__restrict__ begins,
                                                         uint32_t n_runs, uint64_t n_tiles,
                                                         uint32_t *flag, uint32_t *per_chunk) {
    constexpr uint32_t ROW = kThreads * 8;                // 8 fp16 = 16 bytes per lane
    constexpr uint32_t TILE = ROW * 4;
    static_assert(TILE == kCheckTileElems, "tile size");
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner(begins, n_runs, tile);
        const uint16_t *g16 = runs[r].g16;
        const uint64_t n = runs[r].n;
        const uint64_t base = (tile - runs[r].tile_begin) * TILE;
        uint32_t bad = 0;
        if (n - base >= TILE) {
            u32x4 w[4];
#pragma unroll
            for (int u = 0; u < 4; u++)
                w[u] = ld<NT>(gptr<u32x4>(g16 + base + (uint64_t)u * ROW + tid * 8));
#pragma unroll
            for (int u = 0; u < 4; u++)
#pragma unroll
                for (int k = 0; k < 4; k++) bad |= word_has_infnan(w[u][k]);
        } else {
            for (int u = 0; u < 4; u++) {
                const uint64_t i = base + (uint64_t)u * ROW + tid * 8;
                if (i + 8 <= n) {
                    u32x4 w = *gptr<u32x4>(g16 + i);
#pragma unroll
                    for (int k = 0; k < 4; k++) bad |= word_has_infnan(w[k]);
                } else {
                    for (uint64_t k = i; k < n; k++) bad |= half_is_infnan(*gptr<uint16_t>(g16 + k));
                }
            }
        }
        raise_flags(bad, flag, per_chunk, runs[r].chunk);
    }
}

hipError_t launch_check(const RunView &rv, uint64_t n_tiles, uint32_t *flag,
                        uint32_t *per_chunk, const Tuning &t, int n_cu, hipStream_t s) {
    if (n_tiles == 0) return hipSuccess;
    const uint32_t grid = grid_for(n_tiles, t.copy_blocks_per_cu, n_cu);
    if (t.nontemporal)
        hipLaunchKernelGGL(check_kernel<true>, dim3(grid), dim3(kThreads), 0, s, rv.runs, rv.begins, rv.n, n_tiles, flag, per_chunk);
    else
        hipLaunchKernelGGL(check_kernel<false>, dim3(grid), dim3(kThreads), 0, s, rv.runs, rv.begins, rv.n, n_tiles, flag, per_chunk);
    return hipGetLastError();
}

// ------------------------------------------------------------------ pack / unpack
// One segment = one contiguous piece of a tensor inside one chunk.  The destination is written with
// 16-byte stores wherever 16 bytes of it are wanted (single elements before the first and after the
// last boundary); the source is read with 16-byte loads as well: directly when it happens to share
// that alignment, else as pairs of aligned vectors shifted into place with v_alignbyte (every access
// is naturally aligned).
template <int ES>
struct ElemT;
template <>
struct ElemT<2> { typedef uint16_t type; };
template <>
struct ElemT<4> { typedef uint32_t type; };

template <int ES, bool CHECK>
__device__ __forceinline__ uint32_t test_vec(const u32x4 &w) {
    if constexpr (CHECK && ES == 2)
        return word_has_infnan(w[0]) | word_has_infnan(w[1]) | word_has_infnan(w[2]) | word_has_infnan(w[3]);
    else
        return 0;
}

// 16 wanted bytes that start `mis` bytes into the aligned vector `lo` and end in the next one, `hi`.
__device__ __forceinline__ u32x4 shift_pair(const u32x4 &lo, const u32x4 &hi, uint32_t mis) {
    const uint32_t q = mis >> 2, b = mis & 3u;          // whole words and bytes to drop (uniform per tile)
    const uint32_t d[9] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3], 0u};
    u32x4 w;
    switch (q) {
        case 0:
#pragma unroll
            for (int k = 0; k < 4; k++) w[k] = __builtin_amdgcn_alignbyte(d[k + 1], d[k], b);
            break;
        case 1:
#pragma unroll
            for (int k = 0; k < 4; k++) w[k] = __builtin_amdgcn_alignbyte(d[k + 2], d[k + 1], b);
            break;
        case 2:
#pragma unroll
            for (int k = 0; k < 4; k++) w[k] = __builtin_amdgcn_alignbyte(d[k + 3], d[k + 2], b);
            break;
        default:
#pragma unroll
            for (int k = 0; k < 4; k++) w[k] = __builtin_amdgcn_alignbyte(d[k + 4], d[k + 3], b);
            break;
    }
    return w;
}

// Tiles of a segment are cut so that the destination of every tile but the first starts on a
// kCopyCutBytes (128-byte) boundary: a segment whose destination is `a` elements short of one gets a
// first tile of just those `a` elements, and tiles of TILE_ELEMS elements after it.  (The host counts
// tiles by the same rule, see copy_tiles_of.)  Whole tiles then write whole lines and never need
// element-wise heads or tails: they are copied with U 16-byte loads and stores per lane, straight when
// the source shares the 16-byte alignment, else from pairs of aligned source vectors shifted into
// place; only a segment's first and last tile take the general path.
template <int ES, bool CHECK, bool NT, int U, int T>
__global__ __launch_bounds__(T) void copy_kernel(const CopySeg *__restrict__ segs,
                                                        const uint64_t *__restrict__ begins,
                                                        const uint32_t *__restrict__ hints, uint32_t shift,
                                                        uint32_t n_segs, uint64_t n_tiles,
                                                        uint32_t *flag, uint32_t *per_chunk) {
    typedef typename ElemT<ES>::type E;
    constexpr uint32_t TILE_BYTES = T * 16u * U;
    constexpr uint32_t TILE_ELEMS = TILE_BYTES / ES;
    const uint32_t tid = threadIdx.x;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t r = find_owner_hinted(begins, hints, shift, tile);
        const uint64_t n = segs[r].n;
        const uint64_t t_in = tile - segs[r].tile_begin;
        uint64_t a = ((kCopyCutBytes - (uint32_t)(reinterpret_cast<uintptr_t>(segs[r].dst) & (kCopyCutBytes - 1u))) & (kCopyCutBytes - 1u)) / ES;   // elements up to the boundary
        if (a > n) a = n;
        uint64_t base;
        uint32_t cnt;
        if (a != 0 && t_in == 0) {
            base = 0;
            cnt = (uint32_t)a;
        } else {
            base = a + (t_in - (a != 0 ? 1u : 0u)) * TILE_ELEMS;
            const uint64_t left = n - base;
            cnt = left < TILE_ELEMS ? (uint32_t)left : TILE_ELEMS;
        }
        const unsigned char *s = static_cast<const unsigned char *>(segs[r].src) + base * ES;
        unsigned char *d = static_cast<unsigned char *>(segs[r].dst) + base * ES;
        const uint32_t nbytes = cnt * ES;
        uint32_t bad = 0;
        uint32_t head = (16u - (uint32_t)(reinterpret_cast<uintptr_t>(d) & 15u)) & 15u;
        if (head > nbytes) head = nbytes;
        const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(s + head) & 15u);
        if (head == 0 && nbytes == TILE_BYTES) {
            u32x4 w[U];
            if (mis == 0) {
                // whole aligned tile: U 16-byte loads in flight per lane, then U stores
#pragma unroll
                for (int u = 0; u < U; u++)
                    w[u] = ld<NT>(gptr<u32x4>(s) + u * T + tid);
            } else {
                // whole tile, source off by `mis` bytes: the two aligned source vectors that cover each
                // output vector (both hold wanted bytes, so no load leaves the tensor's 16-byte blocks)
                const PSX_GLOBAL u32x4 *ab = gptr<u32x4>(s - mis);
                u32x4 lo[U + 1];
#pragma unroll
                for (int u = 0; u < U; u++) lo[u] = ld<NT>(ab + u * T + tid);
                if constexpr (T == 64) {
                    // one wavefront: the vector after a lane's own is its neighbour's, handed over lane to lane
                    // (a wavefront shift); only the vector after the tile's last one is loaded on top, by all
                    // lanes from one address
                    lo[U] = ld<NT>(ab + U * T);
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        u32x4 hi;
#pragma unroll
                        for (int k = 0; k < 4; k++) {
                            // lane i takes lane i+1's word of this row; lane 63 has no neighbour and keeps `old`:
                            // lane 0's word of the next row (for the last row: the extra vector)
                            const uint32_t next_row_lane0 = __builtin_amdgcn_readfirstlane(lo[u + 1][k]);
                            hi[k] = (uint32_t)__builtin_amdgcn_update_dpp((int)next_row_lane0, (int)lo[u][k], 0x130, 0xf, 0xf, false);
                        }
                        w[u] = shift_pair(lo[u], hi, mis);
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < U; u++) {
                        const u32x4 hi = ld<NT>(ab + u * T + tid + 1);
                        w[u] = shift_pair(lo[u], hi, mis);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                bad |= test_vec<ES, CHECK>(w[u]);
                st<NT>(gptr<u32x4>(d) + u * T + tid, w[u]);
            }
        } else {
            const uint32_t head_e = head / ES;
            if (tid < head_e) {
                E x = gptr<E>(s)[tid];
                if constexpr (CHECK && ES == 2) bad |= half_is_infnan(x);
                gptr<E>(d)[tid] = x;
            }
            const unsigned char *sb = s + head;
            unsigned char *db = d + head;
            const uint32_t nvec = (nbytes - head) / 16u;
            if (mis == 0) {
                for (uint32_t i = tid; i < nvec; i += T) {
                    u32x4 w = gptr<u32x4>(sb)[i];
                    bad |= test_vec<ES, CHECK>(w);
                    gptr<u32x4>(db)[i] = w;
                }
            } else {
                // source and destination disagree modulo 16: read the two 16-byte-aligned source vectors
                // that cover the wanted 16 bytes and shift them into place.  `lo` holds the first wanted
                // byte and `hi` the last one, so both loads stay inside 16-byte blocks that contain valid
                // source bytes (never a page the tensor does not touch).
                const PSX_GLOBAL u32x4 *ab = gptr<u32x4>(sb - mis);
                for (uint32_t i = tid; i < nvec; i += T) {
                    const u32x4 lo = ab[i], hi = ab[i + 1];
                    const u32x4 w = shift_pair(lo, hi, mis);
                    bad |= test_vec<ES, CHECK>(w);
                    gptr<u32x4>(db)[i] = w;
                }
            }
            const uint32_t done = head + nvec * 16u;
            const uint32_t tail_e = (nbytes - done) / ES;
            if (tid < tail_e) {
                E x = gptr<E>(s + done)[tid];
                if constexpr (CHECK && ES == 2) bad |= half_is_infnan(x);
                gptr<E>(d + done)[tid] = x;
            }
        }
        if constexpr (CHECK) raise_flags(bad, flag, per_chunk, segs[r].chunk);
    }
}

hipError_t launch_copy(const SegView &sv, uint64_t n_tiles, uint32_t elem_size,
                       uint32_t *flag, uint32_t *per_chunk, const Tuning &t, int n_cu, hipStream_t s) {
    if (n_tiles == 0) return hipSuccess;
    const uint32_t grid = grid_for(n_tiles, t.copy_blocks_per_cu, n_cu);
    const bool check = flag != nullptr;
    const bool nt = t.nontemporal != 0;
#define PSX_LAUNCH_COPY_T(ES, CH, NT_, T_)                                                                    \
    do {                                                                                                      \
        if (t.copy_unroll == 1)                                                                               \
            hipLaunchKernelGGL((copy_kernel<ES, CH, NT_, 1, T_>), dim3(grid), dim3(T_), 0, s, sv.segs,        \
                               sv.begins, sv.hints, sv.shift, sv.n, n_tiles, flag, per_chunk);                                    \
        else                                                                                                  \
            hipLaunchKernelGGL((copy_kernel<ES, CH, NT_, 4, T_>), dim3(grid), dim3(T_), 0, s, sv.segs,        \
                               sv.begins, sv.hints, sv.shift, sv.n, n_tiles, flag, per_chunk);                                    \
    } while (0)
#define PSX_LAUNCH_COPY(ES, CH, NT_)                                                                          \
    do {                                                                                                      \
        if (t.copy_threads == 64) PSX_LAUNCH_COPY_T(ES, CH, NT_, 64);                                         \
        else PSX_LAUNCH_COPY_T(ES, CH, NT_, 256);                                                             \
    } while (0)
    if (elem_size == 2) {
        if (check) { if (nt) PSX_LAUNCH_COPY(2, true, true); else PSX_LAUNCH_COPY(2, true, false); }
        else       { if (nt) PSX_LAUNCH_COPY(2, false, true); else PSX_LAUNCH_COPY(2, false, false); }
    } else {
        if (nt) PSX_LAUNCH_COPY(4, false, true); else PSX_LAUNCH_COPY(4, false, false);
    }
#undef PSX_LAUNCH_COPY_T
#undef PSX_LAUNCH_COPY
    return hipGetLastError();
}

// ------------------------------------------------------------------ step state on the device
// Loss-scale bookkeeping and the step-wide scalars without the host: the same convention as
// psx_loss_scale_update, and the same derivation of the scalars as the step call (in double, each rounded
// to fp32 once), with beta^t kept as a running product of t factors.  Double division and square root
// are IEEE-correct on this target, so the scalars equal the host's.
__device__ __forceinline__ void derive_scalars(StepState *st) {
    st->sc.step_size = (float)(st->lr / (1.0 - st->b1t));
    st->sc.c2 = (float)(1.0 / __builtin_sqrt(1.0 - st->b2t));
    st->sc.inv_scale = (float)(1.0 / (double)st->scale);
}

__global__ void step_state_init_kernel(StepState *st, StepState init) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    *st = init;
    derive_scalars(st);
}

// One workgroup.  Every thread reads the global flag before any of them clears it; thread 0 does the
// bookkeeping; then, if asked to, all of them clear the n_clear flags (global + per chunk) for the next step.
__global__ void step_state_advance_kernel(StepState *st, uint32_t *flags, uint64_t n_clear) {
    if (blockIdx.x != 0) return;
    const uint32_t overflow = flags[0] != 0 ? 1u : 0u;
    __syncthreads();
    for (uint64_t i = threadIdx.x; i < n_clear; i += blockDim.x) flags[i] = 0u;
    if (threadIdx.x != 0) return;
    if (overflow) {
        const float half = st->scale * 0.5f;
        st->scale = half < 1.0f ? 1.0f : half;
        st->good_steps = 0;
        st->skipped += 1;
    } else {
        st->step += 1;
        st->b1t = st->b1t * st->beta1;
        st->b2t = st->b2t * st->beta2;
        st->good_steps += 1;
        if (st->good_steps >= st->growth_interval) {
            st->scale = st->scale * 2.0f;
            st->good_steps = 0;
        }
    }
    st->last_flag = overflow;
    derive_scalars(st);
}

hipError_t launch_step_state_init(StepState *st, const StepState &init, hipStream_t s) {
    hipLaunchKernelGGL(step_state_init_kernel, dim3(1), dim3(64), 0, s, st, init);
    return hipGetLastError();
}

hipError_t launch_step_state_advance(StepState *st, uint32_t *flags_dev, uint64_t n_clear, hipStream_t s) {
    hipLaunchKernelGGL(step_state_advance_kernel, dim3(1), dim3(64), 0, s, st, flags_dev, n_clear);
    return hipGetLastError();
}

// ------------------------------------------------------------------ small helpers
__global__ void fill_u32_kernel(uint32_t *dst, uint64_t n, uint32_t value) {
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < n;
         i += (uint64_t)gridDim.x * blockDim.x)
        dst[i] = value;
}

hipError_t launch_fill_u32(uint32_t *dst, uint64_t n, uint32_t value, hipStream_t s) {
    if (n == 0) return hipSuccess;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, dst, n, value);
    return hipGetLastError();
}

// Plain copy in the launch shape that copies fastest on this chip (found by measurement): one wavefront
// per workgroup, one 16-byte vector per lane, tiles handed out in order, no cap on resident workgroups
// (with only two streams per workgroup, unlike the Adam kernel's eight, a cap starves the memory system).
template <bool NT>
__global__ __launch_bounds__(64) void copy_bytes_kernel(u32x4 *__restrict__ dst,
                                                        const u32x4 *__restrict__ src,
                                                        uint64_t nvec) {
    const uint64_t n_tiles = (nvec + 63) / 64;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t i = tile * 64 + threadIdx.x;
        if (i < nvec) st<NT>(gptr<u32x4>(dst + i), ld<NT>(gptr<u32x4>(src + i)));
    }
}

hipError_t launch_copy_bytes(void *dst, const void *src, uint64_t n_bytes, const Tuning &t, int n_cu,
                             hipStream_t s) {
    const uint64_t nvec = n_bytes / 16;
    if (nvec == 0) return hipSuccess;
    const uint64_t n_tiles = (nvec + 63) / 64;
    const uint32_t grid = grid_for(n_tiles, t.copy_blocks_per_cu, n_cu);
    if (t.nontemporal)
        hipLaunchKernelGGL(copy_bytes_kernel<true>, dim3(grid), dim3(64), 0, s,
                           static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), nvec);
    else
        hipLaunchKernelGGL(copy_bytes_kernel<false>, dim3(grid), dim3(64), 0, s,
                           static_cast<u32x4 *>(dst), static_cast<const u32x4 *>(src), nvec);
    return hipGetLastError();
}

}  // namespace psx
