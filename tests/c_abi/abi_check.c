/*
 * The C ABI used from plain C with nothing but the HIP runtime: device and pinned buffers from hipMalloc /
 * hipHostMalloc, one gradient pass + resident update + direct-mode update of a host-tier subgroup, the result compared
 * bit for bit with the CPU oracle (linked in: this is test code).  Prints "abi_check ok" and exits 0 on success.
 * Built and run by tests/test_gpu_c_abi.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "mlpo.h"

/* the oracle's entry points used here (oracle/mlpo_oracle.c) */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t bias_correction;
    int32_t l2_mode;
} orc_hparams;
typedef struct {
    float* p;
    float* m;
    float* v;
    const uint16_t* g;
    uint16_t* p16;
    uint64_t n;
} orc_subgroup;
int orc_step(const orc_subgroup* sg, int32_t n_sg, const int32_t* order, const orc_hparams* hp, int64_t steps_applied,
             float inv_scale, float max_norm, float* out_norm, uint32_t* out_found_inf, float* out_gmul);

#define CHECK_HIP(x)                                                              \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));               \
            return 2;                                                             \
        }                                                                         \
    } while (0)
#define CHECK_MLPO(x)                                                             \
    do {                                                                          \
        int rc_ = (x);                                                            \
        if (rc_ != MLPO_OK) {                                                     \
            fprintf(stderr, "%s: %d %s\n", #x, rc_, mlpo_last_error());           \
            return 3;                                                             \
        }                                                                         \
    } while (0)

/* a small linear congruential generator: inputs only */
static uint32_t lcg(uint32_t* s) {
    *s = *s * 1664525u + 1013904223u;
    return *s;
}
static float unit(uint32_t* s) { return (float)(lcg(s) >> 8) / 16777216.0f - 0.5f; }

enum { N_SG = 3 };

int main(void) {
    const uint64_t n[N_SG] = {100003, 65536, 40001};
    const int32_t tier[N_SG] = {MLPO_TIER_HBM, MLPO_TIER_HOST, MLPO_TIER_HBM};
    float *hp_[N_SG], *hm[N_SG], *hv[N_SG];       /* host copies for the oracle */
    uint16_t *hg[N_SG], *h16[N_SG];
    float *dp[N_SG], *dm[N_SG], *dv[N_SG];        /* what the library works on */
    uint16_t *dg[N_SG], *d16[N_SG];
    mlpo_subgroup sg[N_SG];
    orc_subgroup osg[N_SG];
    uint32_t seed = 12345u;
    memset(sg, 0, sizeof sg);
    for (int k = 0; k < N_SG; ++k) {
        const size_t fb = n[k] * sizeof(float), hb = n[k] * sizeof(uint16_t);
        hp_[k] = malloc(fb); hm[k] = malloc(fb); hv[k] = malloc(fb); hg[k] = malloc(hb); h16[k] = calloc(n[k], 2);
        for (uint64_t i = 0; i < n[k]; ++i) {
            hp_[k][i] = 0.04f * unit(&seed);
            hm[k][i] = 1e-3f * unit(&seed);
            const float r = 2e-3f * unit(&seed);
            hv[k][i] = r * r;
            float gval = 2.0f * unit(&seed);       /* scaled gradient; its bf16 pattern is the upper half word */
            uint32_t w;
            memcpy(&w, &gval, 4);
            hg[k][i] = (uint16_t)(w >> 16);
        }
        if (tier[k] == MLPO_TIER_HOST) {
            CHECK_HIP(hipHostMalloc((void**)&dp[k], fb, 0));
            CHECK_HIP(hipHostMalloc((void**)&dm[k], fb, 0));
            CHECK_HIP(hipHostMalloc((void**)&dv[k], fb, 0));
            memcpy(dp[k], hp_[k], fb); memcpy(dm[k], hm[k], fb); memcpy(dv[k], hv[k], fb);
        } else {
            CHECK_HIP(hipMalloc((void**)&dp[k], fb));
            CHECK_HIP(hipMalloc((void**)&dm[k], fb));
            CHECK_HIP(hipMalloc((void**)&dv[k], fb));
            CHECK_HIP(hipMemcpy(dp[k], hp_[k], fb, hipMemcpyHostToDevice));
            CHECK_HIP(hipMemcpy(dm[k], hm[k], fb, hipMemcpyHostToDevice));
            CHECK_HIP(hipMemcpy(dv[k], hv[k], fb, hipMemcpyHostToDevice));
        }
        CHECK_HIP(hipMalloc((void**)&dg[k], hb));
        CHECK_HIP(hipMalloc((void**)&d16[k], hb));
        CHECK_HIP(hipMemcpy(dg[k], hg[k], hb, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemset(d16[k], 0, hb));
        sg[k].p = dp[k]; sg[k].m = dm[k]; sg[k].v = dv[k]; sg[k].g = dg[k]; sg[k].p16 = d16[k];
        sg[k].n = n[k]; sg[k].tier = tier[k]; sg[k].tile_elems = 0; sg[k].half_format = MLPO_HALF_BF16;
        osg[k].p = hp_[k]; osg[k].m = hm[k]; osg[k].v = hv[k]; osg[k].g = hg[k]; osg[k].p16 = h16[k]; osg[k].n = n[k];
    }
    void* ws;
    mlpo_step_scalars* scal;
    CHECK_HIP(hipMalloc(&ws, mlpo_norm_workspace_bytes()));
    CHECK_HIP(hipMalloc((void**)&scal, sizeof *scal));
    hipStream_t link, compute;
    CHECK_HIP(hipStreamCreate(&link));
    CHECK_HIP(hipStreamCreate(&compute));

    mlpo_adamw_hparams hp = {1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 0};
    orc_hparams ohp = {1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 0};
    const float inv_scale = 1.0f / 512.0f, max_norm = 0.05f;
    mlpo_stream_cfg cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.mode = MLPO_STREAM_DIRECT;
    cfg.h2d = link;
    cfg.compute = compute;
    cfg.d2h = compute;
    cfg.direct_blocks = 16;

    for (int step = 0; step < 3; ++step) {
        float norm, gmul;
        uint32_t flag;
        const int applied_o = orc_step(osg, N_SG, NULL, &ohp, step, inv_scale, max_norm, &norm, &flag, &gmul);
        int32_t applied = -1;
        CHECK_MLPO(mlpo_grad_unscale_norm(sg, N_SG, inv_scale, max_norm, ws, mlpo_norm_workspace_bytes(), scal, compute));
        CHECK_MLPO(mlpo_stream_update(sg, N_SG, NULL, &hp, step + 1, scal, &cfg, &applied));
        CHECK_HIP(hipStreamSynchronize(compute));
        mlpo_step_scalars got;
        CHECK_HIP(hipMemcpy(&got, scal, sizeof got, hipMemcpyDeviceToHost));
        if (applied != applied_o || got.found_inf != flag || got.gmul != gmul ||
            fabsf(got.norm - norm) > 1e-5f * norm) {
            fprintf(stderr, "step %d: scalars differ (norm %g vs %g, gmul %g vs %g)\n", step, got.norm, norm, got.gmul,
                    gmul);
            return 1;
        }
    }
    for (int k = 0; k < N_SG; ++k) {
        const size_t fb = n[k] * sizeof(float), hb = n[k] * sizeof(uint16_t);
        float* back = malloc(fb);
        uint16_t* back16 = malloc(hb);
        float* src[3] = {dp[k], dm[k], dv[k]};
        float* want[3] = {hp_[k], hm[k], hv[k]};
        for (int a = 0; a < 3; ++a) {
            if (tier[k] == MLPO_TIER_HOST)
                memcpy(back, src[a], fb);
            else
                CHECK_HIP(hipMemcpy(back, src[a], fb, hipMemcpyDeviceToHost));
            if (memcmp(back, want[a], fb) != 0) {
                fprintf(stderr, "subgroup %d array %d differs from the oracle\n", k, a);
                return 1;
            }
        }
        CHECK_HIP(hipMemcpy(back16, d16[k], hb, hipMemcpyDeviceToHost));
        if (memcmp(back16, h16[k], hb) != 0) {
            fprintf(stderr, "subgroup %d: bf16 copy differs from the oracle\n", k);
            return 1;
        }
        free(back);
        free(back16);
    }
    CHECK_MLPO(mlpo_shutdown());
    printf("abi_check ok: %d subgroups (1 host-tier), 3 steps, state and bf16 copies identical to the oracle\n", N_SG);
    return 0;
}
