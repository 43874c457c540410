/*
 * psx_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar CPU statement of what the chunked mixed-precision
 * Adam path computes.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fPIC -shared.  With SSE
 * scalar arithmetic every float operation below is rounded to binary32 on
 * its own, no operation is fused, denormals are kept.
 *
 * What the paper fixes (PatrickStar, arXiv 2108.05818):
 *   - tensor set and dtypes: param fp16, grad fp16, and the optimizer states
 *     param fp32 / momentum fp32 / variance fp32  (Sec. "Backgrounds of PTM");
 *   - chunks of equal element count, four chunk lists (param fp16, param fp32,
 *     momentum, variance) built in model-initialisation order with identical
 *     offsets; tensors are not split to fill holes, so a chunk may end in a
 *     fragment (Sec. "Preprocessing Stage");
 *   - the grad fp16 tensor is stored in the slot of its param fp16 tensor
 *     (Sec. "Preprocessing Stage", Sec. "Training Stage", Fig. "Reusing param
 *     fp16 chunk with grad fp16");
 *   - in the ADAM stage grads are converted fp16->fp32 on the fly, the fp32
 *     states are updated, then param fp32 is copied into the param fp16 chunk
 *     (Sec. "Training Stage", last paragraph).
 * What the paper leaves to its citations (Kingma & Ba for Adam, Micikevicius
 * et al. for mixed precision with loss scaling) is written out below in the
 * textbook form; every such reading is listed in the design notes.
 *
 * Pins: see tests/test_oracle_*.py (the placement cost at the end of this file:
 * tests/test_oracle_planner.py with hand-worked cases under tests/golden/).
 * The paper fixes neither a loss-scale schedule nor a decay mode.  The
 * arithmetic of both decay modes is pinned against a library Adam / AdamW, and
 * the schedule (halve on overflow, double after growth_interval good steps,
 * a skipped step does not advance t) against a library mixed-precision loop.
 * What stays a convention of this build, "parity unpinned" by the paper: the
 * floor of the scale at 1, the default growth interval, and which decay mode
 * is the default.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* binary16 <-> binary32, written out on the bit patterns.             */
/* fp16->fp32 is exact (subnormals kept).  fp32->fp16 rounds to        */
/* nearest, ties to even; overflow gives +-inf; fp16 subnormals are    */
/* produced, never flushed; NaN stays NaN (quiet bit forced).          */
/* ------------------------------------------------------------------ */

float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0x1Fu) {                    /* inf / nan */
        bits = sign | 0x7F800000u | (man << 13);
    } else if (exp != 0) {                 /* normal */
        bits = sign | ((exp + 112u) << 23) | (man << 13);
    } else if (man == 0) {                 /* zero */
        bits = sign;
    } else {                               /* subnormal: man * 2^-24 */
        int e = -1;
        do { man <<= 1; e++; } while ((man & 0x400u) == 0);
        bits = sign | ((uint32_t)(112 - e) << 23) | ((man & 0x3FFu) << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

uint16_t orc_f32_to_f16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t a = x & 0x7FFFFFFFu;
    if (a > 0x7F800000u)                   /* nan */
        return (uint16_t)(sign | 0x7E00u | ((a >> 13) & 0x3FFu));
    if (a >= 0x47800000u)                  /* |f| >= 65536 (also inf) */
        return (uint16_t)(sign | 0x7C00u);
    if (a >= 0x38800000u) {                /* fp16 normal range, |f| >= 2^-14 */
        uint32_t r = a - 0x38000000u;      /* rebias exponent 127 -> 15 */
        uint32_t keep = r >> 13;
        uint32_t rem = r & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (keep & 1u)))
            keep++;                        /* carry may reach the exponent, up to inf */
        return (uint16_t)(sign | keep);
    }
    if (a < 0x33000000u)                   /* |f| < 2^-25: rounds to zero */
        return sign;
    /* fp16 subnormal: value = mant24 * 2^(e-150), unit 2^-24 */
    {
        uint32_t e = a >> 23;              /* 102 .. 112 */
        uint32_t mant = (a & 0x7FFFFFu) | 0x800000u;
        uint32_t shift = 126u - e;         /* 14 .. 24 */
        uint32_t keep = mant >> shift;
        uint32_t rem = mant & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1u);
        if (rem > half || (rem == half && (keep & 1u)))
            keep++;
        return (uint16_t)(sign | keep);
    }
}

void orc_f16_to_f32_array(const uint16_t *h, float *f, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++) f[i] = orc_f16_to_f32(h[i]);
}

void orc_f32_to_f16_array(const float *f, uint16_t *h, uint64_t n)
{
    for (uint64_t i = 0; i < n; i++) h[i] = orc_f32_to_f16(f[i]);
}

/* ------------------------------------------------------------------ */
/* Tensor -> chunk mapping (Sec. "Preprocessing Stage").               */
/* Tensors are appended in the given order into chunks of chunk_elems  */
/* elements.  A tensor that does not fit the rest of the current chunk */
/* opens the next one (the rest stays a fragment).  Reading for what   */
/* the paper does not cover: a tensor larger than a whole chunk starts */
/* on a fresh chunk and runs over as many consecutive chunks as it     */
/* needs (strict != 0 refuses it instead, which is the paper's own     */
/* rule of choosing the chunk size above the largest tensor).          */
/* Zero-element tensors take the current position and no space.        */
/* Returns 0, or -1 bad argument, -2 oversized tensor in strict mode,  */
/* -3 used[] too short.  used may be NULL (count only).                */
/* ------------------------------------------------------------------ */

typedef struct {
    uint32_t chunk;
    uint32_t reserved;
    uint64_t offset;
    uint64_t numel;
} orc_slot;

int orc_chunk_layout(const uint64_t *numel, uint64_t n, uint64_t chunk_elems,
                     int strict, orc_slot *slots, uint64_t *used,
                     uint64_t used_cap, uint64_t *n_chunks)
{
    if (chunk_elems == 0 || (n && !numel) || !n_chunks) return -1;
    uint64_t chunk = 0, cur = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint64_t s = numel[i];
        if (s > chunk_elems) {
            if (strict) return -2;
            if (cur > 0) {
                if (used) { if (chunk >= used_cap) return -3; used[chunk] = cur; }
                chunk++;
                cur = 0;
            }
            if (slots) { slots[i].chunk = (uint32_t)chunk; slots[i].reserved = 0;
                         slots[i].offset = 0; slots[i].numel = s; }
            uint64_t left = s;
            while (left > chunk_elems) {
                if (used) { if (chunk >= used_cap) return -3; used[chunk] = chunk_elems; }
                chunk++;
                left -= chunk_elems;
            }
            cur = left;
        } else {
            if (s > chunk_elems - cur) {
                if (used) { if (chunk >= used_cap) return -3; used[chunk] = cur; }
                chunk++;
                cur = 0;
            }
            if (slots) { slots[i].chunk = (uint32_t)chunk; slots[i].reserved = 0;
                         slots[i].offset = cur; slots[i].numel = s; }
            cur += s;
        }
    }
    if (used) { if (chunk >= used_cap) return -3; used[chunk] = cur; }
    *n_chunks = chunk + 1;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Tensor <-> chunk copies (Sec. "Training Stage": a tensor's data is  */
/* the piece of chunk payload its slot names; grads are copied from    */
/* temporary memory into that piece).  Byte copies, elem_size bytes    */
/* per element.  The chunk list is read as one virtual array of        */
/* n_chunks*chunk_elems elements, so an oversized tensor simply runs   */
/* on into the next chunk.  Fragments are never touched.  A NULL entry  */
/* in chunks[] means "this chunk is not materialised here": elements   */
/* that belong to it are skipped (lets a test hold a sample of chunks). */
/* ------------------------------------------------------------------ */

void orc_pack(const void *const *tensors, const orc_slot *slots, uint64_t n,
              void *const *chunks, uint64_t chunk_elems, uint64_t elem_size)
{
    for (uint64_t i = 0; i < n; i++) {
        const unsigned char *src = (const unsigned char *)tensors[i];
        uint64_t lin = (uint64_t)slots[i].chunk * chunk_elems + slots[i].offset;
        for (uint64_t k = 0; k < slots[i].numel; k++, lin++) {
            if (chunks[lin / chunk_elems] == NULL) continue;
            unsigned char *dst = (unsigned char *)chunks[lin / chunk_elems]
                                 + (lin % chunk_elems) * elem_size;
            for (uint64_t b = 0; b < elem_size; b++) dst[b] = src[k * elem_size + b];
        }
    }
}

void orc_unpack(void *const *tensors, const orc_slot *slots, uint64_t n,
                const void *const *chunks, uint64_t chunk_elems, uint64_t elem_size)
{
    for (uint64_t i = 0; i < n; i++) {
        unsigned char *dst = (unsigned char *)tensors[i];
        uint64_t lin = (uint64_t)slots[i].chunk * chunk_elems + slots[i].offset;
        for (uint64_t k = 0; k < slots[i].numel; k++, lin++) {
            if (chunks[lin / chunk_elems] == NULL) continue;
            const unsigned char *src = (const unsigned char *)chunks[lin / chunk_elems]
                                       + (lin % chunk_elems) * elem_size;
            for (uint64_t b = 0; b < elem_size; b++) dst[k * elem_size + b] = src[b];
        }
    }
}

/* ------------------------------------------------------------------ */
/* Overflow flag of mixed-precision training with loss scaling (the    */
/* paper's mixed-precision citation): 1 iff any useful fp16 gradient   */
/* element is inf or nan, i.e. has all five exponent bits set.         */
/* per_chunk (may be NULL) receives the same test per chunk.           */
/* Only [0, used[c]) of each chunk is looked at.                       */
/* ------------------------------------------------------------------ */

uint32_t orc_overflow_check(const uint16_t *const *g16_chunks, const uint64_t *used,
                            uint64_t n_chunks, uint32_t *per_chunk)
{
    uint32_t any = 0;
    for (uint64_t c = 0; c < n_chunks; c++) {
        uint32_t f = 0;
        for (uint64_t k = 0; k < used[c]; k++)
            if ((g16_chunks[c][k] & 0x7C00u) == 0x7C00u) f = 1;
        if (per_chunk) per_chunk[c] = f;
        any |= f;
    }
    return any;
}

/* ------------------------------------------------------------------ */
/* Adam (Kingma & Ba, Algorithm 1, with bias correction; epsilon is    */
/* added to the bias-corrected root, outside the root) on one chunk,   */
/* in fp32 as mixed-precision training prescribes for the update.      */
/*                                                                      */
/* Hyper-parameters arrive as doubles; step-wide scalars are prepared   */
/* in double and rounded to fp32 once:                                  */
/*   b1t = beta1^t, b2t = beta2^t (t-fold product), step_size = lr/(1-b1t), */
/*   c2 = 1/sqrt(1-b2t), inv_scale = 1/loss_scale, beta1, beta2,       */
/*   omb1 = 1-beta1, omb2 = 1-beta2, eps, wd, decay = 1-lr*wd.         */
/* Per element (each operation rounded to fp32, in this order):        */
/*   g = f32(g16) * inv_scale                                          */
/*   L2 decay    (wd != 0, adamw == 0):  g = g + wd*p                  */
/*   decoupled   (wd != 0, adamw != 0):  p = p * decay                 */
/*   m = beta1*m + omb1*g                                              */
/*   v = beta2*v + (omb2*g)*g                                          */
/*   p = p - step_size * (m / (sqrt(v)*c2 + eps))                      */
/*   p16 = f16_rne(p)                                                   */
/* m/(sqrt(v)*c2+eps) * lr/(1-b1t) equals Kingma's                     */
/* lr * mhat/(sqrt(vhat)+eps) with mhat=m/(1-b1t), vhat=v/(1-b2t).     */
/* ------------------------------------------------------------------ */

typedef struct {
    double lr, beta1, beta2, eps, weight_decay, loss_scale;
    uint64_t step;        /* 1-based index t of this step */
    uint32_t adamw_mode;
    uint32_t reserved;
} orc_adam_hyper;

typedef struct {
    float step_size, c2, inv_scale, beta1, beta2, omb1, omb2, eps, wd, decay;
} orc_adam_scalars;

void orc_adam_prepare(const orc_adam_hyper *h, orc_adam_scalars *s)
{
    /* beta^t as its definition: the product of t factors, in double */
    double b1t = 1.0, b2t = 1.0;
    for (uint64_t i = 0; i < h->step; i++) { b1t = b1t * h->beta1; b2t = b2t * h->beta2; }
    s->step_size = (float)(h->lr / (1.0 - b1t));
    s->c2 = (float)(1.0 / sqrt(1.0 - b2t));
    s->inv_scale = (float)(1.0 / h->loss_scale);
    s->beta1 = (float)h->beta1;
    s->beta2 = (float)h->beta2;
    s->omb1 = (float)(1.0 - h->beta1);
    s->omb2 = (float)(1.0 - h->beta2);
    s->eps = (float)h->eps;
    s->wd = (float)h->weight_decay;
    s->decay = (float)(1.0 - h->lr * h->weight_decay);
}

void orc_adam_chunk(const uint16_t *g16, uint16_t *p16, float *p32, float *m32,
                    float *v32, uint64_t used, const orc_adam_hyper *h)
{
    orc_adam_scalars s;
    orc_adam_prepare(h, &s);
    const float beta1 = s.beta1, beta2 = s.beta2, eps = s.eps, wd = s.wd;
    for (uint64_t k = 0; k < used; k++) {
        float g = orc_f16_to_f32(g16[k]) * s.inv_scale;
        float p = p32[k], m = m32[k], v = v32[k];
        if (wd != 0.0f) {
            if (h->adamw_mode) {
                p = p * s.decay;
            } else {
                float t = wd * p;
                g = g + t;
            }
        }
        float a = beta1 * m;
        float b = s.omb1 * g;
        m = a + b;
        float c = beta2 * v;
        float d = s.omb2 * g;
        float e = d * g;
        v = c + e;
        float r = sqrtf(v);
        float den = r * s.c2;
        den = den + eps;
        float q = m / den;
        float u = s.step_size * q;
        p = p - u;
        p32[k] = p; m32[k] = m; v32[k] = v;
        p16[k] = orc_f32_to_f16(p);
    }
}

/* On a skipped (overflow) step the fp32 states stay bit-identical.  When  */
/* the grads were written over the param fp16 chunk (chunk reuse), that    */
/* chunk must hold params again before the next forward pass: it is        */
/* re-derived from the untouched fp32 params.                              */
void orc_recast_chunk(uint16_t *p16, const float *p32, uint64_t used)
{
    for (uint64_t k = 0; k < used; k++) p16[k] = orc_f32_to_f16(p32[k]);
}

/* Whole step over a chunk list: global overflow test, then either skip or */
/* update every chunk.  g16[c] may equal p16[c] (chunk reuse).  Returns    */
/* the overflow flag (1 = skipped).                                        */
uint32_t orc_chunk_adam_step(uint16_t *const *g16, uint16_t *const *p16,
                             float *const *p32, float *const *m32, float *const *v32,
                             const uint64_t *used, uint64_t n_chunks,
                             const orc_adam_hyper *h)
{
    uint32_t flag = orc_overflow_check((const uint16_t *const *)g16, used, n_chunks, NULL);
    for (uint64_t c = 0; c < n_chunks; c++) {
        if (!flag)
            orc_adam_chunk(g16[c], p16[c], p32[c], m32[c], v32[c], used[c], h);
        else if (g16[c] == p16[c])
            orc_recast_chunk(p16[c], p32[c], used[c]);
    }
    return flag;
}

/* ------------------------------------------------------------------ */
/* Dynamic loss scale (convention of mixed-precision training, not in  */
/* the paper): an overflow step halves the scale (floor 1), resets the */
/* run of good steps and does not advance t; growth_interval good      */
/* steps in a row double the scale.                                    */
/* ------------------------------------------------------------------ */

typedef struct {
    float scale;
    uint32_t growth_interval;
    uint32_t good_steps;
    uint32_t reserved;
    uint64_t step;        /* t of the next update to apply (starts at 1) */
} orc_scaler;

void orc_scaler_update(orc_scaler *s, uint32_t overflow)
{
    if (overflow) {
        float half = s->scale * 0.5f;
        s->scale = half < 1.0f ? 1.0f : half;
        s->good_steps = 0;
    } else {
        s->step += 1;
        s->good_steps += 1;
        if (s->good_steps >= s->growth_interval) {
            s->scale = s->scale * 2.0f;
            s->good_steps = 0;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Placement of optimizer-state chunks (Sec. "Device-aware Operator    */
/* Placement") for the ADAM scan, by brute force: over T steps with    */
/* HBM budgets budget[t] (in chunks), every assignment of every chunk  */
/* to HBM or host after each step is tried (n_chunks*T <= 24 bits).    */
/* A chunk that is on the host before a step is read over the link     */
/* (12*used bytes), one that is on the host after it is written over   */
/* the link (12*used bytes).  start[k] = 1 if chunk k starts in HBM.   */
/* Returns the least total link bytes of any valid assignment.         */
/* ------------------------------------------------------------------ */
uint64_t orc_min_link_bytes(const uint64_t *used, uint64_t n_chunks, const uint64_t *budget, uint64_t T,
                            const uint8_t *start)
{
    uint64_t best = UINT64_MAX;
    const uint64_t bits = n_chunks * T;
    for (uint64_t a = 0; a < (1ull << bits); a++) {       /* bit (t*n + k) = chunk k in HBM after step t */
        uint64_t cost = 0;
        int ok = 1;
        for (uint64_t t = 0; t < T && ok; t++) {
            uint64_t resident = 0;
            for (uint64_t k = 0; k < n_chunks; k++) {
                int after = (int)((a >> (t * n_chunks + k)) & 1u);
                int before = t == 0 ? start[k] : (int)((a >> ((t - 1) * n_chunks + k)) & 1u);
                resident += (uint64_t)after;
                if (!before) cost += 12 * used[k];
                if (!after) cost += 12 * used[k];
            }
            if (resident > budget[t]) ok = 0;
        }
        if (ok && cost < best) best = cost;
    }
    return best;
}
