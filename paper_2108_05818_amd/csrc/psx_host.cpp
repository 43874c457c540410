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
