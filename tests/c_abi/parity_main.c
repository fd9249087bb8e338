/*
 * The library driven from plain C99 through include/exdyna.h alone: device
 * memory from the HIP runtime, no Python, no torch.  Every step is compared
 * with the CPU oracle (test infrastructure, linked here because this is a
 * test): indices, values, residual, thresholds, counts, bit for bit.
 *
 *   parity_main n_g block_size n_parts density steps
 *
 * Built by __graft_entry__.build():
 *   gcc -std=c99 -O2 -D__HIP_PLATFORM_AMD__ -I include -I oracle -I /opt/rocm/include \
 *       tests/c_abi/parity_main.c -o tests/c_abi/parity_main \
 *       -L paper_2402_13781_amd -lexdyna -L oracle -lexdyna_oracle -L /opt/rocm/lib -lamdhip64 -lm
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "exdyna.h"
#include "exdyna_oracle.h"

#define HIP_OK(call)                                                              \
    do {                                                                          \
        hipError_t e_ = (call);                                                   \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));     \
            return 2;                                                             \
        }                                                                         \
    } while (0)
#define EX_OK(call)                                                               \
    do {                                                                          \
        int r_ = (call);                                                          \
        if (r_ != EXDYNA_OK) {                                                    \
            fprintf(stderr, "%s failed: %s\n", #call, exdyna_strerror(r_));       \
            return 2;                                                             \
        }                                                                         \
    } while (0)

/* input generator only: a counter-based hash turned into a two-sided exponential */
static uint32_t mix(uint64_t x)
{
    x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33;
    return (uint32_t)x;
}
static void fill_gradient(float *g, uint64_t n, uint64_t step, uint64_t hot)
{
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t h = mix((step << 40) ^ i);
        float u = ((h >> 8) + 0.5f) / 16777216.0f;         /* (0, 1) */
        float m = -logf(u) * 1e-3f;
        if (i < hot) m *= 8.0f;                             /* a heavy head: rebalancing has work */
        g[i] = (h & 1u) ? m : -m;
    }
}
static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

int main(int argc, char **argv)
{
    if (argc != 6) {
        fprintf(stderr, "usage: %s n_g block_size n_parts density steps\n", argv[0]);
        return 2;
    }
    const uint64_t n_g = strtoull(argv[1], NULL, 10);
    const uint32_t b = (uint32_t)strtoul(argv[2], NULL, 10), P = (uint32_t)strtoul(argv[3], NULL, 10);
    const double d = atof(argv[4]);
    const int steps = atoi(argv[5]);

    float *g = (float *)malloc(n_g * sizeof(float));
    float *res = (float *)malloc(n_g * sizeof(float));
    float *mag = (float *)malloc(n_g * sizeof(float));
    if (!g || !res || !mag) return 2;
    fill_gradient(g, n_g, 0, n_g / 10);
    for (uint64_t i = 0; i < n_g; ++i) mag[i] = fabsf(g[i]);
    qsort(mag, n_g, sizeof(float), cmp_float);
    uint64_t rank = (uint64_t)ceil((1.0 - d) * (double)n_g);
    const float delta0 = mag[rank ? rank - 1 : 0];
    free(mag);

    exdyna_config cfg;
    EX_OK(exdyna_default_config(&cfg));
    cfg.n_g = n_g; cfg.block_size = b; cfg.n_parts = P; cfg.density = d; cfg.threshold0 = delta0;
    cfg.blk_move = 2;
    size_t ws_bytes = 0;
    EX_OK(exdyna_workspace_bytes(&cfg, &ws_bytes));
    float *d_g = NULL, *d_e = NULL;
    void *d_ws = NULL;
    HIP_OK(hipMalloc((void **)&d_g, n_g * sizeof(float)));
    HIP_OK(hipMalloc((void **)&d_e, n_g * sizeof(float)));
    HIP_OK(hipMalloc(&d_ws, ws_bytes));
    exdyna_ctx *ctx = NULL;
    EX_OK(exdyna_init(&ctx, &cfg, d_e, d_ws, ws_bytes, NULL));
    uint64_t n_b = 0, cap = 0;
    EX_OK(exdyna_get_dims(ctx, &n_b, &cap));

    exo_state *o = exo_create(n_g, b, P, d, delta0, cfg.alpha, cfg.beta, cfg.gamma, cfg.blk_move,
                              cfg.min_blk, cfg.cmp_mode, cfg.max_selected);
    if (!o || exo_capacity(o) != cap || exo_n_blocks(o) != n_b) {
        fprintf(stderr, "oracle and library disagree on the configuration\n");
        return 1;
    }
    uint32_t *idx = (uint32_t *)malloc(cap * sizeof(uint32_t));
    float *val = (float *)malloc(cap * sizeof(float));
    uint32_t *blk = (uint32_t *)malloc(n_b * sizeof(uint32_t));
    if (!idx || !val || !blk) return 2;

    for (int t = 0; t < steps; ++t) {
        if (t) fill_gradient(g, n_g, (uint64_t)t, n_g / 10);
        HIP_OK(hipMemcpy(d_g, g, n_g * sizeof(float), hipMemcpyHostToDevice));
        EX_OK(exdyna_step(ctx, d_g, NULL));
        exo_step(o, g);

        const uint32_t *d_idx; const float *d_val; const uint64_t *d_off;
        uint64_t ka = 0, ke = 0;
        EX_OK(exdyna_get_selected(ctx, &d_idx, &d_val, &d_off, &ka, &ke));
        if (ka != exo_k_actual(o) || ke != exo_k_emitted(o)) {
            fprintf(stderr, "step %d: counts %llu/%llu, oracle %llu/%llu\n", t, (unsigned long long)ka,
                    (unsigned long long)ke, (unsigned long long)exo_k_actual(o),
                    (unsigned long long)exo_k_emitted(o));
            return 1;
        }
        HIP_OK(hipMemcpy(idx, d_idx, ke * sizeof(uint32_t), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(val, d_val, ke * sizeof(float), hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(res, d_e, n_g * sizeof(float), hipMemcpyDeviceToHost));
        EX_OK(exdyna_get_block_counts(ctx, blk));
        exdyna_stats st;
        EX_OK(exdyna_get_stats(ctx, &st));
        float thr = exo_threshold(o);
        if (memcmp(idx, exo_out_idx(o), ke * sizeof(uint32_t)) || memcmp(val, exo_out_val(o), ke * sizeof(float)) ||
            memcmp(res, exo_residual(o), n_g * sizeof(float)) ||
            memcmp(blk, exo_block_count(o), n_b * sizeof(uint32_t)) ||
            memcmp(&st.delta_next, &thr, sizeof(float)) || st.t != (uint64_t)t + 1) {
            fprintf(stderr, "step %d: outputs differ from the oracle\n", t);
            return 1;
        }
        printf("step %d: k'=%llu emitted=%llu delta_next=%g moves=%u ok\n", t, (unsigned long long)ka,
               (unsigned long long)ke, (double)st.delta_next, st.moves);
        fflush(stdout);
    }
    HIP_OK(hipDeviceSynchronize());
    EX_OK(exdyna_destroy(ctx));
    exo_destroy(o);
    HIP_OK(hipFree(d_g)); HIP_OK(hipFree(d_e)); HIP_OK(hipFree(d_ws));
    free(g); free(res); free(idx); free(val); free(blk);
    printf("c-abi parity ok\n");
    return 0;
}
