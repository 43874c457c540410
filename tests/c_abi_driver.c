/*
 * A user of the C ABI written in plain C: no Python, no PyTorch, device memory from hipMalloc.
 * Reads a seeded case from a file, runs the whole path through include/psx.h for a number of
 * steps (layout, fp32 parameter pack, then per step: gradient pack with the overflow test, the
 * Adam step, fp16 parameter unpack, flag read-back, loss-scale update) and writes what it ended
 * up with to a second file.  tests/test_gpu_c_abi.py writes the input, starts this program and
 * compares its output with the oracle's bit for bit.
 *
 *   c_abi_driver IN OUT
 * IN : u64 magic, n, C, steps, adamw, growth_interval, host_from; f64 lr, beta1, beta2, eps, wd, scale0;
 *      (chunks with index >= host_from keep their fp32 states in pinned host memory and are updated over the link)
 *      u64 numel[n]; f32 p32[N]; steps x u16 g16[N]          (N = sum of numel, tensors back to back)
 * OUT: u64 n_chunks; u64 used[n_chunks]; steps x {u32 flag, f32 scale after the step};
 *      per chunk: f32 p32[used], m[used], v[used], u16 p16[used]; u16 unpacked p16 tensors [N]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "psx.h"

#define MAGIC 0x7073785f63616269ull

#define HIP_OK(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            fprintf(stderr, "%s:%d %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            return 2;                                                                              \
        }                                                                                          \
    } while (0)
#define PSX_CALL(call)                                                                                   \
    do {                                                                                                 \
        int32_t r_ = (call);                                                                             \
        if (r_ != PSX_OK) {                                                                              \
            fprintf(stderr, "%s:%d %s -> %d: %s\n", __FILE__, __LINE__, #call, (int)r_, psx_last_error()); \
            return 3;                                                                                    \
        }                                                                                                \
    } while (0)

static int read_exact(FILE *f, void *dst, size_t bytes) { return bytes == 0 || fread(dst, 1, bytes, f) == bytes; }
static int write_exact(FILE *f, const void *src, size_t bytes) { return bytes == 0 || fwrite(src, 1, bytes, f) == bytes; }

int main(int argc, char **argv) {
    if (argc != 3) {
        fprintf(stderr, "usage: %s IN OUT\n", argv[0]);
        return 1;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    uint64_t head[7];
    double hp[6];
    if (!read_exact(in, head, sizeof head) || !read_exact(in, hp, sizeof hp) || head[0] != MAGIC) {
        fprintf(stderr, "bad input header\n");
        return 1;
    }
    const uint64_t n = head[1], C = head[2], steps = head[3], adamw = head[4], growth = head[5], host_from = head[6];
    uint64_t *numel = (uint64_t *)malloc((n ? n : 1) * sizeof(uint64_t));
    if (!numel || !read_exact(in, numel, n * sizeof(uint64_t))) { fprintf(stderr, "bad input: sizes\n"); return 1; }
    uint64_t N = 0;
    for (uint64_t i = 0; i < n; i++) N += numel[i];
    float *h_p32 = (float *)malloc((N ? N : 1) * sizeof(float));
    uint16_t *h_g16 = (uint16_t *)malloc((N ? N : 1) * sizeof(uint16_t));
    uint16_t *h_p16 = (uint16_t *)malloc((N ? N : 1) * sizeof(uint16_t));
    if (!h_p32 || !h_g16 || !h_p16 || !read_exact(in, h_p32, N * sizeof(float))) { fprintf(stderr, "bad input: params\n"); return 1; }

    /* a1: layout, sizing call first */
    size_t n_chunks = 0;
    PSX_CALL(psx_chunk_layout(numel, (size_t)n, C, 0, NULL, NULL, 0, &n_chunks));
    psx_slot *slots = (psx_slot *)malloc((n ? n : 1) * sizeof(psx_slot));
    uint64_t *used = (uint64_t *)malloc(n_chunks * sizeof(uint64_t));
    if (!slots || !used) return 1;
    PSX_CALL(psx_chunk_layout(numel, (size_t)n, C, 0, slots, used, n_chunks, &n_chunks));

    /* device memory: tensors back to back, every chunk list one arena of n_chunks * C elements */
    float *d_p32_t = NULL;
    uint16_t *d_g16_t = NULL, *d_p16_t = NULL;
    HIP_OK(hipMalloc((void **)&d_p32_t, (N ? N : 1) * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_g16_t, (N ? N : 1) * sizeof(uint16_t)));
    HIP_OK(hipMalloc((void **)&d_p16_t, (N ? N : 1) * sizeof(uint16_t)));
    HIP_OK(hipMemset(d_p16_t, 0, (N ? N : 1) * sizeof(uint16_t)));
    const size_t arena_elems = n_chunks * (size_t)C;
    uint16_t *g16 = NULL, *p16 = NULL;
    float *p32 = NULL, *m = NULL, *v = NULL;
    HIP_OK(hipMalloc((void **)&g16, arena_elems * 2)); HIP_OK(hipMemset(g16, 0, arena_elems * 2));
    HIP_OK(hipMalloc((void **)&p16, arena_elems * 2)); HIP_OK(hipMemset(p16, 0, arena_elems * 2));
    HIP_OK(hipMalloc((void **)&p32, arena_elems * 4)); HIP_OK(hipMemset(p32, 0, arena_elems * 4));
    HIP_OK(hipMalloc((void **)&m, arena_elems * 4));   HIP_OK(hipMemset(m, 0, arena_elems * 4));
    HIP_OK(hipMalloc((void **)&v, arena_elems * 4));   HIP_OK(hipMemset(v, 0, arena_elems * 4));
    HIP_OK(hipMemcpy(d_p32_t, h_p32, N * sizeof(float), hipMemcpyHostToDevice));

    const void **t_p32 = (const void **)malloc((n ? n : 1) * sizeof(void *));
    const void **t_g16 = (const void **)malloc((n ? n : 1) * sizeof(void *));
    void **t_p16 = (void **)malloc((n ? n : 1) * sizeof(void *));
    void **c_g16 = (void **)malloc(n_chunks * sizeof(void *)), **c_p16 = (void **)malloc(n_chunks * sizeof(void *));
    void **c_p32 = (void **)malloc(n_chunks * sizeof(void *));
    psx_chunk *chunks = (psx_chunk *)calloc(n_chunks, sizeof(psx_chunk));
    if (!t_p32 || !t_g16 || !t_p16 || !c_g16 || !c_p16 || !c_p32 || !chunks) return 1;
    uint64_t off = 0;
    for (uint64_t i = 0; i < n; i++) {
        t_p32[i] = d_p32_t + off; t_g16[i] = d_g16_t + off; t_p16[i] = d_p16_t + off;
        off += numel[i];
    }
    for (size_t k = 0; k < n_chunks; k++) {
        c_g16[k] = g16 + k * C; c_p16[k] = p16 + k * C; c_p32[k] = p32 + k * C;
        chunks[k].g16 = c_g16[k]; chunks[k].p16 = c_p16[k];
        chunks[k].p32 = c_p32[k]; chunks[k].m = m + k * C; chunks[k].v = v + k * C;
        chunks[k].used = used[k];
        chunks[k].loc_in = chunks[k].loc_out = PSX_LOC_HBM;
        chunks[k].exec = PSX_EXEC_GPU;
    }

    psx_ctx_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.max_chunks = n_chunks; cfg.max_tensors = n ? n : 1;
    psx_ctx *ctx = NULL;
    PSX_CALL(psx_ctx_create(&cfg, &ctx));
    PSX_CALL(psx_pack(ctx, PSX_F32, t_p32, slots, (size_t)n, c_p32, n_chunks, C, 0, NULL));
    HIP_OK(hipDeviceSynchronize());
    /* host-resident chunks: pinned homes for the used prefix; the packed parameters move there, and the
     * device copies are overwritten so that a kernel reading the wrong home would show */
    for (size_t k = (size_t)host_from; k < n_chunks; k++) {
        if (used[k] == 0) continue;
        void *hb[3] = {NULL, NULL, NULL};
        for (int j = 0; j < 3; j++) {
            PSX_CALL(psx_pinned_alloc(used[k] * sizeof(float), &hb[j]));
            memset(hb[j], 0, used[k] * sizeof(float));
        }
        HIP_OK(hipMemcpy(hb[0], p32 + k * C, used[k] * sizeof(float), hipMemcpyDeviceToHost));
        HIP_OK(hipMemset(p32 + k * C, 0x5a, used[k] * sizeof(float)));
        HIP_OK(hipMemset(m + k * C, 0x5a, used[k] * sizeof(float)));
        HIP_OK(hipMemset(v + k * C, 0x5a, used[k] * sizeof(float)));
        chunks[k].p32_host = hb[0]; chunks[k].m_host = hb[1]; chunks[k].v_host = hb[2];
        chunks[k].loc_in = chunks[k].loc_out = PSX_LOC_HOST;
    }

    FILE *out = fopen(argv[2], "wb");
    if (!out) { perror(argv[2]); return 1; }
    uint64_t nc64 = n_chunks;
    if (!write_exact(out, &nc64, 8) || !write_exact(out, used, n_chunks * 8)) return 1;

    psx_scaler sc;
    memset(&sc, 0, sizeof sc);
    sc.scale = (float)hp[5]; sc.growth_interval = (uint32_t)growth; sc.step = 1;
    for (uint64_t s = 0; s < steps; s++) {
        if (!read_exact(in, h_g16, N * sizeof(uint16_t))) { fprintf(stderr, "bad input: gradients of step %llu\n", (unsigned long long)s); return 1; }
        HIP_OK(hipMemcpy(d_g16_t, h_g16, N * sizeof(uint16_t), hipMemcpyHostToDevice));
        psx_adam_hyper h;
        memset(&h, 0, sizeof h);
        h.lr = hp[0]; h.beta1 = hp[1]; h.beta2 = hp[2]; h.eps = hp[3]; h.weight_decay = hp[4];
        h.loss_scale = (double)sc.scale; h.step = sc.step; h.adamw_mode = (uint32_t)adamw;
        uint32_t flag = 0;
        PSX_CALL(psx_overflow_reset(ctx, NULL));
        PSX_CALL(psx_pack(ctx, PSX_F16, t_g16, slots, (size_t)n, c_g16, n_chunks, C, PSX_PACK_CHECK_OVERFLOW, NULL));   /* a2 + a3 */
        PSX_CALL(psx_chunk_adam_step(ctx, chunks, n_chunks, &h, PSX_STEP_USE_FLAG, NULL));                             /* a4, a6 */
        PSX_CALL(psx_unpack(ctx, PSX_F16, t_p16, slots, (size_t)n, (const void *const *)c_p16, n_chunks, C, 0, NULL)); /* a2 */
        PSX_CALL(psx_overflow_read(ctx, NULL, 0, &flag, NULL));
        PSX_CALL(psx_loss_scale_update(&sc, flag));                                                                    /* a7 */
        if (!write_exact(out, &flag, 4) || !write_exact(out, &sc.scale, 4)) return 1;
    }
    HIP_OK(hipDeviceSynchronize());
    float *h_f = (float *)malloc((size_t)(C ? C : 1) * sizeof(float));
    uint16_t *h_h = (uint16_t *)malloc((size_t)(C ? C : 1) * sizeof(uint16_t));
    if (!h_f || !h_h) return 1;
    for (size_t k = 0; k < n_chunks; k++) {
        const float *lists[3] = {p32 + k * C, m + k * C, v + k * C};
        const void *homes[3] = {chunks[k].p32_host, chunks[k].m_host, chunks[k].v_host};
        for (int j = 0; j < 3; j++) {
            if (chunks[k].loc_out == PSX_LOC_HOST && used[k] != 0) memcpy(h_f, homes[j], used[k] * sizeof(float));
            else HIP_OK(hipMemcpy(h_f, lists[j], used[k] * sizeof(float), hipMemcpyDeviceToHost));
            if (!write_exact(out, h_f, used[k] * sizeof(float))) return 1;
        }
        HIP_OK(hipMemcpy(h_h, p16 + k * C, used[k] * sizeof(uint16_t), hipMemcpyDeviceToHost));
        if (!write_exact(out, h_h, used[k] * sizeof(uint16_t))) return 1;
    }
    HIP_OK(hipMemcpy(h_p16, d_p16_t, N * sizeof(uint16_t), hipMemcpyDeviceToHost));
    if (!write_exact(out, h_p16, N * sizeof(uint16_t))) return 1;
    if (fclose(out) != 0) return 1;
    fclose(in);
    PSX_CALL(psx_ctx_destroy(ctx));
    for (size_t k = 0; k < n_chunks; k++) {
        PSX_CALL(psx_pinned_free(chunks[k].p32_host));
        PSX_CALL(psx_pinned_free(chunks[k].m_host));
        PSX_CALL(psx_pinned_free(chunks[k].v_host));
    }
    HIP_OK(hipFree(d_p32_t)); HIP_OK(hipFree(d_g16_t)); HIP_OK(hipFree(d_p16_t));
    HIP_OK(hipFree(g16)); HIP_OK(hipFree(p16)); HIP_OK(hipFree(p32)); HIP_OK(hipFree(m)); HIP_OK(hipFree(v));
    printf("c_abi_driver: %llu tensors, %llu elements, %zu chunks, %llu steps done\n", (unsigned long long)n,
           (unsigned long long)N, n_chunks, (unsigned long long)steps);
    return 0;
}
