// Host-only parts of the C ABI: error message, tensor->chunk layout, loss scaler.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "psx_internal.h"

namespace psx {

static thread_local char g_err[768] = "";

int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace psx

extern "C" const char *psx_last_error(void) { return psx::g_err; }

// In-order append of tensors into equal-size chunks.  `pos` is the running
// position in the virtual concatenation of chunks; a tensor that would cross a
// chunk boundary is moved to the next boundary unless it is larger than a
// chunk, in which case it starts on a boundary and runs across.
extern "C" int32_t psx_chunk_layout(const uint64_t *numel, size_t n, uint64_t chunk_elems,
                                    uint32_t flags, psx_slot *slots, uint64_t *used, size_t cap,
                                    size_t *n_chunks) {
    if (chunk_elems == 0) return psx::fail(PSX_EINVAL, "psx_chunk_layout: chunk_elems is 0");
    if (n != 0 && numel == nullptr) return psx::fail(PSX_EINVAL, "psx_chunk_layout: numel is NULL");
    if (n_chunks == nullptr) return psx::fail(PSX_EINVAL, "psx_chunk_layout: n_chunks is NULL");
    if (flags & ~PSX_LAYOUT_STRICT) return psx::fail(PSX_EINVAL, "psx_chunk_layout: unknown flags 0x%x", flags);
    const uint64_t C = chunk_elems;

    // first pass: validate and count, so that nothing is written on error
    uint64_t pos = 0;
    for (size_t i = 0; i < n; i++) {
        const uint64_t s = numel[i];
        if (s == 0) continue;
        if (s > C && (flags & PSX_LAYOUT_STRICT))
            return psx::fail(PSX_ETOOLARGE, "psx_chunk_layout: tensor %zu has %llu elements, chunk holds %llu",
                             i, (unsigned long long)s, (unsigned long long)C);
        const uint64_t room = (C - pos % C) % C;      // elements left in a started chunk
        if (s > room) pos += room;                     // skip the fragment (room == 0: on a boundary)
        if (pos + s < pos) return psx::fail(PSX_EINVAL, "psx_chunk_layout: total size overflows 64 bits");
        pos += s;
    }
    const uint64_t count = pos == 0 ? 1 : (pos + C - 1) / C;
    if (count > 0xFFFFFFFFull) return psx::fail(PSX_EINVAL, "psx_chunk_layout: more than 2^32 chunks");
    if (used != nullptr && cap < count)
        return psx::fail(PSX_ECAP, "psx_chunk_layout: used[] holds %zu entries, %llu chunks needed", cap,
                         (unsigned long long)count);

    // second pass: write the slots and the filled prefix of every chunk
    if (used != nullptr)
        for (uint64_t c = 0; c < count; c++) used[c] = 0;
    pos = 0;
    for (size_t i = 0; i < n; i++) {
        const uint64_t s = numel[i];
        if (s != 0) {
            const uint64_t room = (C - pos % C) % C;
            if (s > room) pos += room;
        }
        if (slots != nullptr) {
            // a position on a boundary belongs to the chunk that ends there when nothing follows in it
            uint64_t c = pos / C, off = pos % C;
            if (s == 0 && off == 0 && pos != 0) { c -= 1; off = C; }
            slots[i].chunk = (uint32_t)c;
            slots[i].reserved = 0;
            slots[i].offset = off;
            slots[i].numel = s;
        }
        if (used != nullptr) {
            uint64_t p = pos, left = s;
            while (left != 0) {
                const uint64_t take = left < C - p % C ? left : C - p % C;
                used[p / C] += take;
                p += take;
                left -= take;
            }
        }
        pos += s;
    }
    *n_chunks = (size_t)count;
    return PSX_OK;
}

extern "C" int32_t psx_loss_scale_update(psx_scaler *s, uint32_t overflow) {
    if (s == nullptr) return psx::fail(PSX_EINVAL, "psx_loss_scale_update: scaler is NULL");
    if (overflow) {
        const float half = s->scale * 0.5f;
        s->scale = half < 1.0f ? 1.0f : half;
        s->good_steps = 0;
    } else {
        s->step += 1;
        s->good_steps += 1;
        if (s->good_steps >= s->growth_interval) {
            s->scale *= 2.0f;
            s->good_steps = 0;
        }
    }
    return PSX_OK;
}

// ---------------------------------------------------------------------------
// Placement of optimizer-state chunks for the ADAM stage and chunk-size search.
// ---------------------------------------------------------------------------

// A resident chunk costs 12*chunk_elems bytes of HBM whatever its fill; a
// host-resident chunk costs 12*used bytes on the link in each direction at
// every step.  So the chunks worth keeping are the fullest ones.  The order
// (fill descending, index ascending) does not depend on the budget, which
// makes the resident sets for growing budgets nested: when the budget moves,
// only chunks at the margin change residence.
extern "C" int32_t psx_plan_residency(const uint64_t *used, size_t n_chunks, uint64_t chunk_elems,
                                      uint64_t hbm_budget_bytes, uint8_t *loc, uint64_t *host_elems) {
    if (n_chunks != 0 && (used == nullptr || loc == nullptr)) return psx::fail(PSX_EINVAL, "psx_plan_residency: NULL array");
    if (chunk_elems == 0) return psx::fail(PSX_EINVAL, "psx_plan_residency: chunk_elems is 0");
    for (size_t k = 0; k < n_chunks; k++)
        if (used[k] > chunk_elems) return psx::fail(PSX_EINVAL, "psx_plan_residency: used[%zu] exceeds the chunk", k);
    const uint64_t per_chunk = 12ull * chunk_elems;
    uint64_t room = hbm_budget_bytes / per_chunk;             // chunks that fit
    if (room > n_chunks) room = n_chunks;
    for (size_t k = 0; k < n_chunks; k++) loc[k] = PSX_LOC_HOST;
    uint64_t streamed = 0;
    for (size_t k = 0; k < n_chunks; k++) streamed += used[k];
    // pick the `room` fullest chunks; n_chunks is a few hundred, a selection loop is enough
    for (uint64_t r = 0; r < room; r++) {
        size_t best = n_chunks;
        for (size_t k = 0; k < n_chunks; k++)
            if (loc[k] == PSX_LOC_HOST && (best == n_chunks || used[k] > used[best])) best = k;
        if (best == n_chunks) break;
        loc[best] = PSX_LOC_HBM;
        streamed -= used[best];
    }
    if (host_elems != nullptr) *host_elems = streamed;
    return PSX_OK;
}

extern "C" int32_t psx_chunk_size_search(const uint64_t *numel, size_t n, uint64_t lo, uint64_t hi, uint64_t step,
                                         uint32_t flags, uint64_t max_model_data_bytes, uint64_t *best_chunk_elems,
                                         double *best_util, size_t *best_n_chunks) {
    if (best_chunk_elems == nullptr) return psx::fail(PSX_EINVAL, "psx_chunk_size_search: best_chunk_elems is NULL");
    if (lo == 0 || step == 0 || hi < lo) return psx::fail(PSX_EINVAL, "psx_chunk_size_search: need 0 < lo <= hi and step > 0");
    if (n != 0 && numel == nullptr) return psx::fail(PSX_EINVAL, "psx_chunk_size_search: numel is NULL");
    uint64_t total = 0;
    for (size_t i = 0; i < n; i++) total += numel[i];
    bool found = false;
    double util_best = -1.0;
    uint64_t c_best = 0;
    size_t n_best = 0;
    for (uint64_t c = lo; c <= hi; c += step) {
        size_t nch = 0;
        const int32_t rc = psx_chunk_layout(numel, n, c, flags & PSX_LAYOUT_STRICT, nullptr, nullptr, 0, &nch);
        if (rc == PSX_ETOOLARGE) { if (hi - c < step) break; continue; }   // a tensor does not fit this size
        if (rc != PSX_OK) return rc;
        // the four chunk lists take 14 bytes per element of chunk capacity
        const long double bytes = 14.0L * (long double)nch * (long double)c;
        if (max_model_data_bytes != 0 && bytes > (long double)max_model_data_bytes) { if (hi - c < step) break; continue; }
        const double util = (double)((long double)total / ((long double)nch * (long double)c));
        if (!found || util > util_best) { found = true; util_best = util; c_best = c; n_best = nch; }
        if (hi - c < step) break;                                            // also guards the += against overflow
    }
    if (!found) return psx::fail(PSX_ETOOLARGE, "psx_chunk_size_search: no chunk size in the range holds the model");
    *best_chunk_elems = c_best;
    if (best_util) *best_util = util_best;
    if (best_n_chunks) *best_n_chunks = n_best;
    return PSX_OK;
}
