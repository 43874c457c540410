/*
 * psx.h -- C ABI of the chunked mixed-precision Adam path for MI355X (gfx950).
 *
 * The operations are those of PatrickStar (arXiv 2108.05818): model data is
 * packed, in model-initialisation order, into chunks of one fixed element
 * count; four chunk lists (param fp16, param fp32, momentum, variance) share
 * one tensor->(chunk, offset) map; gradients in fp16 sit in the param fp16
 * slots (or in a chunk list of their own); the ADAM stage converts the fp16
 * gradient chunk to fp32 on the fly, updates the fp32 states and writes the
 * fp16 parameter chunk back.  Optimizer-state chunks may live in GPU memory
 * or in pinned host memory, chunk by chunk.
 *
 * Conventions
 *   - Every call returns a psx status (0 = PSX_OK, negative = error).  No
 *     exception or abort crosses the boundary.  psx_last_error() gives the
 *     calling thread's last message.  Argument errors are detected before any
 *     payload byte is touched.
 *   - "host" pointers are ordinary process memory.  "device" pointers are HIP
 *     device allocations on the current device.  "pinned" pointers are
 *     page-locked host allocations (hipHostMalloc or equivalent).
 *   - The caller owns every payload buffer (tensors, chunks).  The library
 *     owns only what psx_ctx_create() allocates: descriptor tables, flags,
 *     staging tiles, side streams and events.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work on it and return; they are asynchronous unless the
 *     description says the call synchronises.  A context must not be used
 *     from two threads at once.  Calls on one context share its descriptor
 *     tables and flags and are ordered by the stream they are issued on:
 *     issue them on one stream, or order different streams yourself (event
 *     or synchronisation) before the next call on the same context.
 *   - HIP graphs.  A call whose descriptors (tensor list, slots, chunk list)
 *     equal those of the previous call of its kind on the context uploads
 *     nothing and enqueues kernel launches only; in that state
 *     psx_overflow_reset, psx_pack, psx_unpack, psx_overflow_check without
 *     read-back, psx_chunk_adam_step and psx_chunk_adam_step_unpack over
 *     HBM-resident chunks with PSX_STEP_DEVICE_STATE, and
 *     psx_step_state_advance may be recorded into a
 *     graph (stream capture) and replayed: every replay is one more training
 *     step, with t and the loss scale advancing on the device.  Issue the same
 *     calls once outside the capture first.  A call that would have to upload
 *     a descriptor table, to synchronise, or to use the side streams while its
 *     stream is capturing fails with PSX_ECAPTURE and enqueues nothing.
 *   - Chunk base addresses must be 16-byte aligned.  Tensor addresses need
 *     only their element alignment.
 *   - Element counts are in elements, never bytes.
 */
#ifndef PSX_H
#define PSX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------ status */
#define PSX_OK          0
#define PSX_EINVAL     (-1)  /* null pointer, zero chunk size, bad enum, ...          */
#define PSX_ETOOLARGE  (-2)  /* tensor larger than a chunk under PSX_LAYOUT_STRICT    */
#define PSX_ECAP       (-3)  /* an output array or a context table is too small       */
#define PSX_EALIGN     (-4)  /* a chunk base is not 16-byte aligned                   */
#define PSX_EHIP       (-5)  /* the HIP runtime reported an error (see last error)    */
#define PSX_ENOSTAGING (-6)  /* PSX_TUNE_HOST_MODE 0 and a host-side chunk, but no staging   */
#define PSX_ECAPTURE   (-7)  /* the stream is being captured into a HIP graph and this call, as given, cannot be recorded */

/* Message of the last failing call on this thread ("" if none). Host pointer, owned by the library. */
const char *psx_last_error(void);

/* ------------------------------------------------------------------ layout
 * Tensor-Chunk-Mapper (Sec. "Preprocessing Stage"): tensors are appended in
 * the given order into chunks of chunk_elems elements; the same map serves
 * the param fp16, param fp32, momentum and variance lists.  A tensor that
 * does not fit the rest of the current chunk opens the next chunk; the rest
 * stays an unused fragment at the chunk's tail.  A tensor is never split to
 * fill a fragment.  A tensor larger than a whole chunk (the paper avoids it
 * by choosing the chunk size) starts on a fresh chunk and runs over as many
 * consecutive chunks as it needs, unless PSX_LAYOUT_STRICT asks for the
 * paper's behaviour, in which case it is PSX_ETOOLARGE.  A zero-element
 * tensor gets the current position and takes no space.
 */
typedef struct psx_slot {
    uint32_t chunk;     /* index of the chunk holding the tensor's first element */
    uint32_t reserved;  /* 0 */
    uint64_t offset;    /* element offset inside that chunk */
    uint64_t numel;     /* elements; may run past the chunk end for an oversized tensor */
} psx_slot;

#define PSX_LAYOUT_STRICT 1u

/*
 * numel[n]   host, in : element count of each tensor, in model-initialisation order
 * slots[n]   host, out: may be NULL (sizing call)
 * used[cap]  host, out: filled prefix of each chunk, elements; may be NULL
 * n_chunks   host, out: number of chunks (>= 1)
 * Pure host code, deterministic, touches no GPU.  If used != NULL and cap is
 * smaller than the chunk count the call fails with PSX_ECAP (outputs unspecified).
 */
int32_t psx_chunk_layout(const uint64_t *numel, size_t n, uint64_t chunk_elems, uint32_t flags,
                         psx_slot *slots, uint64_t *used, size_t cap, size_t *n_chunks);

/* ------------------------------------------------------------------ context */
typedef struct psx_ctx psx_ctx;

typedef struct psx_ctx_config {
    uint64_t max_chunks;          /* most chunks any call will pass                          */
    uint64_t max_tensors;         /* most tensors any pack/unpack call will pass             */
    uint64_t staging_tile_elems;  /* elements per staging tile for host-resident chunks;     */
                                  /* only PSX_TUNE_HOST_MODE 0 uses staging; 0 = none        */
    uint32_t staging_slots;       /* tiles in flight, 2..8 (ignored when tile_elems == 0)    */
    uint32_t reserved;            /* 0 */
} psx_ctx_config;

/* Allocates the context on the current HIP device: descriptor tables, the
 * overflow flags, 3 * staging_slots * staging_tile_elems floats of device
 * staging, two side streams (default priority) and events.  Synchronous. */
int32_t psx_ctx_create(const psx_ctx_config *cfg, psx_ctx **out);
/* Waits for the context's outstanding work, then frees what create allocated. */
int32_t psx_ctx_destroy(psx_ctx *ctx);

/* ------------------------------------------------------------------ pack / unpack
 * Tensor <-> chunk copies (Sec. "Training Stage": a tensor's data is the piece
 * of chunk payload its slot names; after BWD the fp16 gradient is copied from
 * temporary memory into the slot of its param fp16 tensor).  Bit-exact copies;
 * fragments are neither read nor written.  The chunk list is one virtual
 * array of n_chunks*chunk_elems elements, so an oversized tensor runs on into
 * the following chunk(s).
 *
 * dtype         PSX_F16 (2-byte elements) or PSX_F32 (4-byte elements)
 * tensors[n]    host array of device pointers, tensor i has slots[i].numel elements
 * slots[n]      host, from psx_chunk_layout
 * chunks[]      host array of n_chunks device pointers, each chunk_elems elements (page-locked,
 *               device-accessible host memory works as well, at host-link speed: that is how the
 *               fp32 params of host-resident chunks are packed)
 * flags         PSX_PACK_CHECK_OVERFLOW (psx_pack, PSX_F16 only): while copying,
 *               OR the inf/nan test of every copied element into the context's
 *               overflow flags (see psx_overflow_check; clear them first with
 *               psx_overflow_reset)
 * One multi-tensor launch on `stream`; asynchronous.  The descriptor upload
 * may wait for the context's previous upload to finish.
 */
#define PSX_F16 1u
#define PSX_F32 2u
#define PSX_PACK_CHECK_OVERFLOW 1u

int32_t psx_pack(psx_ctx *ctx, uint32_t dtype, const void *const *tensors, const psx_slot *slots,
                 size_t n, void *const *chunks, size_t n_chunks, uint64_t chunk_elems,
                 uint32_t flags, void *stream);
int32_t psx_unpack(psx_ctx *ctx, uint32_t dtype, void *const *tensors, const psx_slot *slots,
                   size_t n, const void *const *chunks, size_t n_chunks, uint64_t chunk_elems,
                   uint32_t flags, void *stream);

/* ------------------------------------------------------------------ overflow flag
 * Mixed-precision training with loss scaling (the paper's mixed-precision
 * citation) skips the update when any gradient is inf or nan.  The test is
 * taken on the fp16 bit pattern: all five exponent bits set.  Only the first
 * used[c] elements of chunk c are looked at.
 *
 * g16_chunks[]  host array of n_chunks device pointers (fp16 gradient chunks)
 * used[]        host array, elements in use per chunk
 * per_chunk     host, out, n_chunks entries of 0/1; may be NULL
 * flag_out      host, out, OR over all chunks; may be NULL
 * The flags are first cleared, then computed on `stream` and left in the
 * context on the device, where psx_chunk_adam_step(PSX_STEP_USE_FLAG) reads
 * them.  If per_chunk or flag_out is non-NULL the call synchronises `stream`
 * to read them back; otherwise it is asynchronous.
 */
int32_t psx_overflow_check(psx_ctx *ctx, const void *const *g16_chunks, const uint64_t *used,
                           size_t n_chunks, uint32_t *per_chunk, uint32_t *flag_out, void *stream);
/* Clear the context's flags on `stream` (asynchronous). */
int32_t psx_overflow_reset(psx_ctx *ctx, void *stream);
/* Read the context's flags back (synchronises `stream`).  per_chunk may be NULL. */
int32_t psx_overflow_read(psx_ctx *ctx, uint32_t *per_chunk, size_t n_chunks, uint32_t *flag_out,
                          void *stream);

/* ------------------------------------------------------------------ Adam step
 * ADAM stage over a chunk list (Sec. "Training Stage", last paragraph; Adam is
 * Kingma & Ba's Algorithm 1 with bias correction, epsilon added outside the
 * root; fp32 arithmetic, every operation rounded on its own, no fused
 * multiply-add).  Step-wide scalars are derived in double from the doubles
 * below and rounded to fp32 once:
 *   step_size = lr/(1-beta1^t), c2 = 1/sqrt(1-beta2^t), inv_scale = 1/loss_scale,
 *   beta1, beta2, 1-beta1, 1-beta2, eps, weight_decay, decay = 1-lr*weight_decay,
 * where beta^t is the product of t factors beta, each multiplication rounded to
 * double (not libm's pow, which differs from it in the last bits).
 * Per element k < used:
 *   g = f32(g16[k]) * inv_scale
 *   weight_decay != 0, adamw_mode == 0:  g = g + weight_decay*p      (L2)
 *   weight_decay != 0, adamw_mode != 0:  p = p * decay               (decoupled)
 *   m = beta1*m + (1-beta1)*g ;  v = beta2*v + ((1-beta2)*g)*g
 *   p = p - step_size * (m / (sqrt(v)*c2 + eps))
 *   p16[k] = fp16 round-to-nearest-even of p
 */
typedef struct psx_adam_hyper {
    double lr, beta1, beta2, eps, weight_decay, loss_scale;
    uint64_t step;        /* 1-based index t of this update */
    uint32_t adamw_mode;  /* 0 = L2 decay added to the gradient, 1 = decoupled decay */
    uint32_t reserved;    /* 0 */
} psx_adam_hyper;

#define PSX_LOC_HBM  0u   /* fp32 states in device memory  */
#define PSX_LOC_HOST 1u   /* fp32 states in pinned host memory */

#define PSX_EXEC_GPU 0u   /* the chunk is updated by the GPU kernel (host-resident: over the link)       */
#define PSX_EXEC_CPU 1u   /* HOST -> HOST chunks only: updated in place by the host cores (the paper's    */
                          /* placement for host-resident optimizer states): only the fp16 gradient tile   */
                          /* (D2H) and the fp16 parameter tile (H2D) cross the link, 2 + 2 B/element      */

/*
 * One chunk of the four lists.  g16 and p16 are always device memory; p16 may
 * equal g16 (the paper's chunk reuse: the gradient sits in the param fp16
 * chunk and is overwritten by the new fp16 parameters).  The fp32 states are
 * found at entry in the loc_in buffers and left, updated, in the loc_out
 * buffers (Sec. "Device-aware Operator Placement": as many optimizer-state
 * chunks as fit stay in GPU memory, the rest in host memory):
 *   HBM  -> HBM  : updated in place in p32/m/v.
 *   HOST -> HOST : by default the kernel reads and writes the pinned buffers
 *                  directly over the host link (one launch on a side stream,
 *                  concurrent with the resident chunks; the buffers must be
 *                  device-accessible, as hipHostMalloc memory is: the call asks the
 *                  runtime about them the first time this context sees them at
 *                  that chunk index and must find them page-locked from then on,
 *                  for as long as the caller passes them); with
 *                  PSX_TUNE_HOST_MODE 0 they are streamed tile by tile through
 *                  the context's staging (H2D, update, D2H).  p32/m/v may be NULL.
 *   HOST -> HBM  : chunk admitted: the kernel reads the pinned buffers and
 *                  writes p32/m/v (mode 0: copied into p32/m/v, updated there).
 *   HBM  -> HOST : chunk evicted: the kernel reads p32/m/v and writes the
 *                  pinned buffers (mode 0: updated in p32/m/v, then copied out).
 *                  The buffers of the home a chunk leaves hold stale or updated
 *                  values afterwards, depending on the mode: treat them as dead.
 */
typedef struct psx_chunk {
    void *g16;        /* device, fp16 gradients, chunk_elems capacity, first `used` read */
    void *p16;        /* device, fp16 parameters out; may alias g16 */
    void *p32, *m, *v;                  /* device fp32 states, or NULL if never in HBM  */
    void *p32_host, *m_host, *v_host;   /* pinned fp32 states, or NULL if never on host */
    uint64_t used;    /* elements in use (a prefix); the tail fragment is never touched */
    uint8_t loc_in;   /* PSX_LOC_* where the states are at entry */
    uint8_t loc_out;  /* PSX_LOC_* where they must be at exit    */
    uint8_t exec;     /* PSX_EXEC_*; PSX_EXEC_CPU needs loc_in == loc_out == PSX_LOC_HOST */
    uint8_t reserved[5];
} psx_chunk;

#define PSX_STEP_DEVICE_STATE 4u /* take t and the loss scale from the context's step state on the device */
                                 /* (psx_step_state_init) instead of hyper->step / hyper->loss_scale;   */
                                 /* the other fields of *hyper must be those given to that call         */
#define PSX_STEP_USE_FLAG    1u  /* skip the update if the context's overflow flag is set      */
#define PSX_STEP_CHECK_FIRST 2u  /* run the overflow check over all g16 chunks first (implies  */
                                 /* PSX_STEP_USE_FLAG)                                         */
/*
 * chunks[n_chunks]  host array.  All work is enqueued on `stream` and on the
 * context's two copy streams; on return `stream` has been made to wait for
 * them, so work enqueued on `stream` afterwards sees the finished step.
 * Asynchronous with respect to the host, unless a chunk asks for PSX_EXEC_CPU: the GPU work is
 * enqueued first and runs meanwhile, then the calling thread drives the host-core update (worker
 * threads, AVX2 + F16C, same arithmetic and bits as the GPU kernel) and returns when it is done.
 * Skipped step (flag set): p32/m/v keep their bits (states that change
 * residence are still moved); p16 is left alone unless it aliases g16, in which
 * case it is rewritten with fp16(p32) so that the chunk holds parameters again.
 */
int32_t psx_chunk_adam_step(psx_ctx *ctx, const psx_chunk *chunks, size_t n_chunks,
                            const psx_adam_hyper *hyper, uint32_t flags, void *stream);

/* The step-wide fp32 scalars psx_chunk_adam_step derives from *hyper, in the order step_size, c2,
 * inv_scale, beta1, beta2, 1-beta1, 1-beta2, eps, weight_decay, decay (see the formulas above); the
 * same validation as the step call.  out[10], host.  Pure host code: lets a caller (or a test) see
 * exactly which constants the kernels will use at step t. */
int32_t psx_adam_step_scalars(const psx_adam_hyper *hyper, float *out);

/*
 * psx_chunk_adam_step with the fp16 parameter unpack fused in (Sec. "Training Stage", last paragraph: the
 * updated parameters reach the param fp16 chunk; a framework whose fp16 parameter tensors are not views
 * into that chunk needs them copied out, which psx_unpack does by reading the chunk again).  Here the
 * kernel that produces fp16(p32) stores it twice, into chunk.p16 and into the tensor that owns the
 * position, so the chunk is not read back: 30 bytes per element in one launch instead of 28 + 4 in two.
 *   p16_tensors[n_tensors]  host array of device pointers (fp16, element-aligned); slots[n_tensors] as
 *                           returned by psx_chunk_layout for chunk_elems.  Slots must not overlap;
 *                           elements of the chunk list that no slot covers are written to the chunk only.
 * Every chunk with used > 0 must stay in HBM (loc_in == loc_out == PSX_LOC_HBM, PSX_EXEC_GPU) and the Adam
 * launch shape must be the default one, else PSX_EINVAL.  Elements of a slot behind its chunk's `used`
 * are not written.  The fused store pays when the tensors' memory is aligned like their slots (the usual
 * case: 64-element multiples at 128-byte aligned addresses); where most of it is not, pieces of a tile
 * end inside 128-byte lines of the tensors and the two-launch form is faster, so the library then runs
 * the update and the unpack as two launches of its own (PSX_TUNE_FUSED_UNPACK overrides the choice).
 * On a skipped step (overflow flag set) the fused form writes no tensor and the two-launch form rewrites
 * them with the unchanged chunk content: either way they hold the chunk list's parameters if they did
 * before.  Flags, errors, streams and graph capture as for psx_chunk_adam_step; results are bit-identical
 * to psx_chunk_adam_step followed by psx_unpack(PSX_F16) of the p16 chunks.
 */
int32_t psx_chunk_adam_step_unpack(psx_ctx *ctx, const psx_chunk *chunks, size_t n_chunks,
                                   const psx_adam_hyper *hyper, uint32_t flags,
                                   void *const *p16_tensors, const psx_slot *slots, size_t n_tensors,
                                   uint64_t chunk_elems, void *stream);

/*
 * The same step for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context: the overflow flags and the descriptor tables the kernels
 * search live in one static device array of PSX_NOALLOC_SCRATCH_BYTES that every GPU the library runs on
 * holds until the process ends, and the descriptors reach it as kernel arguments.  The call issues kernel
 * launches only: no hipMalloc / hipFree, no memcpy, no memset, nothing that allocates.
 *   chunks[n_chunks]  host array as above, restricted to loc_in == loc_out == PSX_LOC_HBM and
 *                     exec == PSX_EXEC_GPU; n_chunks <= PSX_NOALLOC_MAX_CHUNKS, else PSX_ECAP
 *   flags             0, or PSX_STEP_CHECK_FIRST: test all g16 chunks for inf/nan first and skip the
 *                     update if one is found (p16 that aliases g16 is then rewritten with fp16(p32))
 *   flag_out_dev      device, out, may be NULL: receives 0/1 = step skipped (needs PSX_STEP_CHECK_FIRST)
 * Launch shapes are the library defaults (no tuning knobs).  Asynchronous on `stream`.  Every call on a
 * GPU uses that GPU's one array and rewrites the parts it needs: calls that overlap in time on one GPU
 * (two streams, two threads) race; order them.  Arguments are validated before anything is enqueued.
 */
#define PSX_NOALLOC_MAX_CHUNKS    1024u
#define PSX_NOALLOC_SCRATCH_BYTES 262144u
int32_t psx_chunk_adam_step_noalloc(const psx_chunk *chunks, size_t n_chunks, const psx_adam_hyper *hyper,
                                    uint32_t flags, uint32_t *flag_out_dev, void *stream);

/* ------------------------------------------------------------------ loss scale
 * Dynamic loss scale bookkeeping on the host (a convention of mixed-precision
 * training; not specified by the paper): an overflow halves the scale (floor 1),
 * clears good_steps and leaves step unchanged; otherwise step and good_steps
 * advance and growth_interval good steps in a row double the scale.
 */
typedef struct psx_scaler {
    float scale;
    uint32_t growth_interval;
    uint32_t good_steps;
    uint32_t reserved;
    uint64_t step;        /* t of the next update to apply; starts at 1 */
} psx_scaler;

int32_t psx_loss_scale_update(psx_scaler *s, uint32_t overflow);

/* ------------------------------------------------------------------ step state on the device
 * The same bookkeeping without the host in the loop, so that a whole training step (gradient pack with
 * overflow test, update, loss-scale bookkeeping) can be enqueued without a read-back and recorded into a
 * HIP graph.  The context keeps, in device memory, what psx_scaler holds, beta1^t and beta2^t as running
 * products of t factors, and the step-wide fp32 scalars of the next update (derived from those in double,
 * rounded once, as in the host path).
 *   psx_step_state_init     sets the state from *scaler and *hyper (hyper->step and hyper->loss_scale are
 *                           ignored: scaler->step and scaler->scale count).  Asynchronous on `stream`.
 *   psx_step_state_advance  closes a step on the device: reads the context's overflow flag and applies the
 *                           rules of psx_loss_scale_update (overflow: scale halved with floor 1, good_steps
 *                           cleared, t unchanged; else t and good_steps advance, growth_interval good steps
 *                           double the scale), then derives the scalars of the next update.  One tiny
 *                           launch on `stream`; asynchronous.  With PSX_ADVANCE_CLEAR_FLAGS it also clears
 *                           the context's overflow flags (global and per chunk) once it has read them, so
 *                           the next step needs no psx_overflow_reset: one launch less per step, which is
 *                           what a small model's step consists of.
 *   psx_step_state_read     copies the state back (synchronises `stream`): scaler, the flag of the step
 *                           closed last, the number of steps skipped so far; each may be NULL.
 * psx_chunk_adam_step(PSX_STEP_DEVICE_STATE) updates with the state's t and loss scale. */
int32_t psx_step_state_init(psx_ctx *ctx, const psx_adam_hyper *hyper, const psx_scaler *scaler, void *stream);
#define PSX_ADVANCE_CLEAR_FLAGS 1u
int32_t psx_step_state_advance(psx_ctx *ctx, uint32_t flags, void *stream);
int32_t psx_step_state_read(psx_ctx *ctx, psx_scaler *scaler, uint32_t *last_flag, uint64_t *skipped, void *stream);

/* ------------------------------------------------------------------ tuning and timing
 * Launch shape knobs (for sweeps; defaults are tuned for MI355X):
 *   PSX_TUNE_ADAM_BLOCKS_PER_CU  0 = one tile per workgroup, dispatched in order; n > 0 = n persistent
 *                                workgroups per CU that stride over the tiles
 *   PSX_TUNE_ADAM_UNROLL         rows of 4 elements per thread per tile: 1, 2 or 4
 *   PSX_TUNE_NONTEMPORAL         0/1: non-temporal hints on the streaming loads and stores
 *   PSX_TUNE_COPY_BLOCKS_PER_CU  same as the first, for pack/unpack/check
 *   PSX_TUNE_ADAM_THREADS        threads per workgroup of the Adam kernel: 64 or 256
 *   PSX_TUNE_ADAM_WG_PER_CU      cap on Adam workgroups resident per CU (0 = none)
 *   PSX_TUNE_COPY_UNROLL         16-byte vectors per thread and tile of pack/unpack: 1 or 4; 0 = the library's
 *                                choice (default; 1)
 *   PSX_TUNE_COPY_THREADS        threads per workgroup of pack/unpack: 64 (default) or 256
 *   PSX_TUNE_HOST_MODE           chunks with a host side: 0 = H2D / D2H copies on the copy streams (through
 *                                the context's staging tiles for HOST -> HOST, into / out of the device
 *                                buffers for chunks that change residence); 1 = the kernels read and write
 *                                the pinned buffers directly over the host link (they must be
 *                                device-accessible, which hipHostMalloc memory is; no staging needed)
 *   PSX_TUNE_HOST_GRID           mode 1: persistent workgroups of those launches
 *   PSX_TUNE_HOST_UNROLL         mode 1: rows of 4 elements per thread: 1, 2 or 4
 */
#define PSX_TUNE_ADAM_BLOCKS_PER_CU 1u
#define PSX_TUNE_ADAM_UNROLL        2u
#define PSX_TUNE_NONTEMPORAL        3u
#define PSX_TUNE_COPY_BLOCKS_PER_CU 4u
#define PSX_TUNE_ADAM_THREADS       5u
#define PSX_TUNE_ADAM_WG_PER_CU     6u
#define PSX_TUNE_COPY_UNROLL        7u
#define PSX_TUNE_HOST_MODE          8u
#define PSX_TUNE_HOST_GRID          9u
#define PSX_TUNE_HOST_UNROLL        10u
#define PSX_TUNE_CPU_THREADS        11u  /* worker threads for PSX_EXEC_CPU chunks (default: min(cores, 16)) */
#define PSX_TUNE_CPU_TILE_ELEMS     12u  /* elements per tile of the PSX_EXEC_CPU pipeline (multiple of 16)  */
#define PSX_TUNE_CPU_ISA            13u  /* PSX_EXEC_CPU vectors: 0 = widest the host has (AVX-512, else AVX2), 1 = AVX2 */
#define PSX_TUNE_COPY_THREADS       14u
#define PSX_TUNE_FUSED_UNPACK       15u  /* psx_chunk_adam_step_unpack: 0 = the library decides (default), 1 = always write the tensors from the Adam launch, 2 = always update, then unpack */
int32_t psx_ctx_set_tuning(psx_ctx *ctx, uint32_t key, int64_t value);

/* Kernel timing with HIP events on the caller's stream (off by default). */
typedef struct psx_timing {
    float pack_ms;     /* last psx_pack copy kernel                                        */
    float check_ms;    /* last overflow check kernel                                       */
    float adam_ms;     /* last resident (HBM->HBM) Adam kernel launch                      */
    float spill_ms;    /* last streamed part: first H2D issued to last D2H done            */
    uint64_t adam_elems;   /* elements the resident launch covered                         */
    uint64_t spill_elems;  /* elements of chunks with a host side                          */
    uint64_t h2d_bytes, d2h_bytes;  /* link bytes of the streamed part                     */
    float cpu_ms;          /* last PSX_EXEC_CPU part: host wall time, first tile to last   */
    uint32_t cpu_threads;  /* worker threads it used                                       */
    uint64_t cpu_elems;    /* elements updated by the host cores                           */
    float unpack_ms;       /* last psx_unpack copy kernel                                  */
    uint32_t reserved;
} psx_timing;
int32_t psx_ctx_set_profiling(psx_ctx *ctx, int32_t on);
/* Synchronises the recorded events, then fills *out (fields of phases not run are 0). */
int32_t psx_ctx_get_timing(psx_ctx *ctx, psx_timing *out);

/* Plain device copy of n_bytes (a multiple of 16, 16-byte aligned pointers), the
 * reference kernel the bandwidth counters and the Adam kernel are scaled against. */
int32_t psx_copy_bytes(psx_ctx *ctx, void *dst, const void *src, uint64_t n_bytes, void *stream);

/* ------------------------------------------------------------------ placement and chunk size
 * Device-aware placement of optimizer-state chunks (Sec. "Device-aware Operator Placement": as many
 * optimizer-state chunks as fit the GPU margin space stay in GPU memory) specialised to the ADAM stage,
 * which scans every chunk once per step.  A resident chunk takes 12*chunk_elems bytes of the budget; a
 * host-resident chunk crosses the link with 12*used[k] bytes in each direction at every step.  The plan
 * keeps the floor(budget / (12*chunk_elems)) fullest chunks in HBM (ties: lower index first), which
 * minimises the link bytes of every step; for a growing budget the resident sets are nested, so a moving
 * budget only moves chunks at the margin.  (On this cyclic scan the farthest-next-use rule of Sec. "Chunk
 * Eviction Strategy" always evicts the chunk just updated, so in steady state a fixed set stays resident
 * and the rest streams; which set is a free choice, taken here to minimise link bytes.)
 * used[n_chunks]  host, in;  loc[n_chunks] host, out: PSX_LOC_HBM / PSX_LOC_HOST;
 * host_elems      host, out, may be NULL: sum of used[] over host-resident chunks.  Pure host code. */
int32_t psx_plan_residency(const uint64_t *used, size_t n_chunks, uint64_t chunk_elems,
                           uint64_t hbm_budget_bytes, uint8_t *loc, uint64_t *host_elems);

/* Chunk-size search (Sec. "Evaluation Methodology", "Chunk Size Searching"): try chunk sizes lo, lo+step,
 * ... <= hi (elements), lay the tensor list out with each (psx_chunk_layout with `flags`), and return the
 * size with the highest utilisation sum(numel) / (n_chunks*chunk_elems); ties go to the smaller size.
 * Sizes for which PSX_LAYOUT_STRICT refuses a tensor, or whose four chunk lists (14 bytes per element of
 * chunk capacity) exceed max_model_data_bytes (0 = no limit), are skipped; PSX_ETOOLARGE if none is left.
 * best_util and best_n_chunks may be NULL.  Pure host code; allocates nothing. */
int32_t psx_chunk_size_search(const uint64_t *numel, size_t n, uint64_t lo, uint64_t hi, uint64_t step,
                              uint32_t flags, uint64_t max_model_data_bytes, uint64_t *best_chunk_elems,
                              double *best_util, size_t *best_n_chunks);

/* Page-locked, device-accessible host memory for host-resident chunks (hipHostMalloc with default
 * flags).  A host-resident chunk needs room for its `used` elements only.  Synchronous. */
int32_t psx_pinned_alloc(uint64_t n_bytes, void **out);
int32_t psx_pinned_free(void *ptr);

/* Pinned-memory copy rates of this machine's host link, measured with hipMemcpyAsync on the
 * context's own two copy streams (the ones host-resident chunks are streamed on): each direction
 * alone, then both directions at once.  GB/s (1e9 bytes) per direction; best of `reps` passes after
 * two warm-up passes.  Allocates and frees two pinned and two device buffers of `mib` MiB.
 * Synchronous.  A measurement aid: the denominator for the host-resident part of the step. */
typedef struct psx_link_rates {
    double h2d_alone, d2h_alone, each_way_both;
} psx_link_rates;
int32_t psx_measure_link(psx_ctx *ctx, uint64_t mib, uint32_t reps, psx_link_rates *out);

#ifdef __cplusplus
}
#endif
#endif /* PSX_H */
