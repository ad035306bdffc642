/*
 * The C ABI used from plain C, without Python or PyTorch: device memory from the HIP runtime, the
 * update path through include/palsgd.h, and the CPU oracle's element routines linked in as the
 * reference (test infrastructure).  Runs Alg. 1 for a few steps on a small ragged model and compares
 * every element of X, M, V, XG, OM:  |gpu - oracle| <= 1e-5 |oracle| + 1e-7.  Exit code 0 = pass.
 *
 * Built by __graft_entry__.build():
 *   gcc -std=c11 -O2 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude tests/c_abi_parity.c \
 *       oracle/palsgd_oracle.c -o tests/c_abi_parity -Lpaper_2504_18454_amd/csrc -lpalsgd \
 *       -L/opt/rocm/lib -lamdhip64 -lm -Wl,-rpath,...
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "palsgd.h"

/* element routines of oracle/palsgd_oracle.c */
int ora_draw(uint64_t seed, uint64_t t, uint32_t k, uint32_t K, double p);
void ora_mix(float *x, const float *xg, uint64_t n, double beta);
void ora_adamw(float *x, float *m, float *v, const void *g, int g_dtype, uint64_t n, double lr, double beta1,
               double beta2, double eps, double wd, uint64_t tau, double grad_scale);
void ora_outer(float *X, uint64_t row_stride, uint32_t K, float *xg, float *om, uint64_t n, double lr_o,
               double mu_o, int nesterov);

#define HIP(x)                                                                            \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define PAL(x, ctx)                                                                              \
    do {                                                                                         \
        palsgd_status s_ = (x);                                                                  \
        if (s_ != PALSGD_OK) {                                                                   \
            fprintf(stderr, "palsgd status %d at line %d: %s\n", s_, __LINE__, palsgd_last_error(ctx)); \
            return 3;                                                                            \
        }                                                                                        \
    } while (0)

static uint64_t lcg_state = 0x1234567ull;
static double uniform(void) /* in (-1, 1) */
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return ((double)(lcg_state >> 11) / 9007199254740992.0) * 2.0 - 1.0;
}

static int compare(const char *name, const float *got, const float *want, uint64_t n, double *worst)
{
    for (uint64_t i = 0; i < n; ++i) {
        double err = fabs((double)got[i] - (double)want[i]);
        double bound = 1e-5 * fabs((double)want[i]) + 1e-7;
        if (err / bound > *worst) *worst = err / bound;
        if (!(err <= bound)) {
            fprintf(stderr, "%s[%llu]: gpu %.9g oracle %.9g\n", name, (unsigned long long)i, got[i], want[i]);
            return 1;
        }
    }
    return 0;
}

int main(void)
{
    enum { K = 3, NT = 3, STEPS = 11 };
    const uint64_t numel[NT] = {5000, 64, 333};
    const float wd_mult[NT] = {1.0f, 0.0f, 0.5f};
    const float alpha = 1e-3f, eta = 16.0f;
    palsgd_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.K = K; cfg.n_tensors = NT; cfg.tensor_numel = numel; cfg.tensor_wd_mult = wd_mult;
    cfg.inner = PALSGD_INNER_ADAMW; cfg.grad_dtype = PALSGD_GRAD_F32;
    cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.eps = 1e-8f; cfg.weight_decay = 0.01f; cfg.momentum = 0.9f;
    cfg.p = 0.3; cfg.H = 4; cfg.outer_lr = 0.7f; cfg.outer_momentum = 0.9f; cfg.outer_nesterov = 1; cfg.seed = 5;

    uint64_t row = 0, off[NT];
    PAL(palsgd_layout(&cfg, &row, off), NULL);
    const size_t rb = row * sizeof(float);

    /* host copies: the oracle's state */
    float *x0 = calloc(row, 4), *c = calloc(row, 4), *XG = calloc(row, 4), *OM = calloc(row, 4);
    float *X = calloc(K * row, 4), *M = calloc(K * row, 4), *V = calloc(K * row, 4), *G = calloc(K * row, 4);
    float *back = calloc(K * row, 4);
    uint64_t tau[K] = {0};
    for (int j = 0; j < NT; ++j)
        for (uint64_t i = 0; i < numel[j]; ++i) {
            x0[off[j] + i] = (float)(0.02 * uniform());
            c[off[j] + i] = (float)uniform();
        }
    memcpy(XG, x0, rb);
    for (int k = 0; k < K; ++k) memcpy(X + k * row, x0, rb);

    /* device buffers, caller-owned */
    palsgd_buffers buf;
    memset(&buf, 0, sizeof buf);
    float *x0_dev;
    HIP(hipMalloc((void **)&buf.X, K * rb)); HIP(hipMalloc((void **)&buf.M, K * rb)); HIP(hipMalloc((void **)&buf.V, K * rb));
    HIP(hipMalloc(&buf.G, K * rb)); HIP(hipMalloc((void **)&buf.XG, rb)); HIP(hipMalloc((void **)&buf.OM, rb));
    HIP(hipMalloc((void **)&x0_dev, rb));
    buf.row_stride = row;
    HIP(hipMemcpy(x0_dev, x0, rb, hipMemcpyHostToDevice));

    palsgd_ctx *ctx = NULL;
    PAL(palsgd_init(&cfg, &buf, x0_dev, NULL, &ctx), NULL);

    const double b1 = (double)cfg.beta1, b2 = (double)cfg.beta2, eps = (double)cfg.eps, wd = (double)cfg.weight_decay;
    for (uint64_t t = 0; t < STEPS; ++t) {
        for (int k = 0; k < K; ++k)   /* g_k = (x_k - c) + noise at the oracle's x_k, zero on padding */
            for (int j = 0; j < NT; ++j)
                for (uint64_t i = off[j]; i < off[j] + numel[j]; ++i)
                    G[k * row + i] = (float)(((double)X[k * row + i] - (double)c[i]) + 0.05 * uniform());
        HIP(hipMemcpy(buf.G, G, K * rb, hipMemcpyHostToDevice));
        uint8_t mask[K];
        PAL(palsgd_draw(ctx, t, mask), ctx);
        for (int k = 0; k < K; ++k) {
            if (mask[k] != ora_draw(cfg.seed, t, k, K, cfg.p)) {
                fprintf(stderr, "draw differs at t=%llu k=%d\n", (unsigned long long)t, k);
                return 1;
            }
            if (mask[k]) {
                ora_mix(X + k * row, XG, row, (double)alpha * (double)eta / cfg.p);
            } else {
                tau[k] += 1;
                for (int j = 0; j < NT; ++j)
                    ora_adamw(X + k * row + off[j], M + k * row + off[j], V + k * row + off[j], G + k * row + off[j], 0,
                              numel[j], (double)alpha / (1.0 - cfg.p), b1, b2, eps, wd * (double)wd_mult[j], tau[k], 1.0);
            }
        }
        PAL(palsgd_step(ctx, t, alpha, eta, NULL, NULL, NULL), ctx);
        if ((t + 1) % cfg.H == 0) {
            PAL(palsgd_outer_step(ctx, t, NULL), ctx);
            ora_outer(X, row, K, XG, OM, row, (double)cfg.outer_lr, (double)cfg.outer_momentum, 1);
        }
    }
    HIP(hipDeviceSynchronize());

    double worst = 0.0;
    int bad = 0;
    uint64_t tau_dev[K], n_outer = 0;
    PAL(palsgd_get_state(ctx, tau_dev, &n_outer), ctx);
    for (int k = 0; k < K; ++k) bad |= tau_dev[k] != tau[k];
    bad |= n_outer != STEPS / cfg.H;
    HIP(hipMemcpy(back, buf.X, K * rb, hipMemcpyDeviceToHost)); bad |= compare("X", back, X, K * row, &worst);
    HIP(hipMemcpy(back, buf.M, K * rb, hipMemcpyDeviceToHost)); bad |= compare("M", back, M, K * row, &worst);
    HIP(hipMemcpy(back, buf.V, K * rb, hipMemcpyDeviceToHost)); bad |= compare("V", back, V, K * row, &worst);
    HIP(hipMemcpy(back, buf.XG, rb, hipMemcpyDeviceToHost)); bad |= compare("XG", back, XG, row, &worst);
    HIP(hipMemcpy(back, buf.OM, rb, hipMemcpyDeviceToHost)); bad |= compare("OM", back, OM, row, &worst);
    palsgd_destroy(ctx);
    printf("c_abi_parity: %s, %d steps, K=%d, %llu elements per row, worst err/bound %.3f\n", bad ? "FAIL" : "PASS",
           (int)STEPS, (int)K, (unsigned long long)row, worst);
    return bad ? 1 : 0;
}
