/*
 * The CPU checker (oracle/palsgd_oracle.c) driven from plain C on tiny models, for a build with
 * -fsanitize=address,undefined: every buffer is allocated with exactly the bytes the checker may touch
 * (rows of stride > n, so the gap between rows and the end of the last row are guarded), all routines are
 * called (Alg. 1 driver with both inner optimizers and both gradient types, strided outer step, DDP step,
 * norms, clipping scale, diagnostics), and one line of check sums per case is printed for the test that
 * runs this program to compare with the same cases computed through the unsanitized library.  Hyper-parameters
 * are fp32 values widened to double, as the Python wrapper of the checker passes them.
 */
#include <stdio.h>

#include "../oracle/palsgd_oracle.c"

static const uint64_t OFFS[4] = {0, 8, 16, 24}, NUMEL[4] = {1, 3, 5, 17};
static const float WDM[4] = {1.0f, 0.0f, 0.5f, 1.0f};
enum { N = 41, PADROW = 7 };

/* the value pattern both sides generate: multiples of 1/8 in [-0.75, 0.75], exact in bf16 */
static float pattern(uint64_t t, uint32_t k, uint64_t i) { return ((float)((t * 31 + k * 17 + i * 7) % 13) - 6.0f) * 0.125f; }
static int is_real(uint64_t i)
{
    for (int j = 0; j < 4; ++j)
        if (i >= OFFS[j] && i < OFFS[j] + NUMEL[j])
            return 1;
    return 0;
}

static void fill_gradients(void *G, int g_dtype, uint32_t K, uint64_t stride, uint64_t t)
{
    for (uint32_t k = 0; k < K; ++k)
        for (uint64_t i = 0; i < N; ++i) {
            float v = is_real(i) ? pattern(t, k, i) : 0.0f;
            if (g_dtype == 0) {
                ((float *)G)[k * stride + i] = v;
            } else {
                uint32_t bits;
                memcpy(&bits, &v, 4);
                ((uint16_t *)G)[k * stride + i] = (uint16_t)(bits >> 16);
            }
        }
}

static double weighted(const float *a, uint64_t n, double w0)
{
    double s = 0.0;
    for (uint64_t i = 0; i < n; ++i)
        s += (double)a[i] * (w0 + (double)i);
    return s;
}

int main(void)
{
    ora_set_threads(2);
    for (int inner = 0; inner < 2; ++inner)
    for (int g_dtype = 0; g_dtype < 2; ++g_dtype)
    for (uint32_t K = 1; K <= 3; ++K)
    for (uint32_t H = 1; H <= 3; ++H) {
        const uint64_t stride = N + PADROW, rows = (uint64_t)(K - 1) * stride + N;
        float *X = malloc(rows * 4), *M = malloc(rows * 4), *V = malloc(rows * 4);
        float *XG = malloc(N * 4), *OM = malloc(N * 4);
        void *G = malloc(rows * (g_dtype ? 2 : 4));
        uint64_t tau[3] = {0, 0, 0};
        memset(M, 0, rows * 4); memset(V, 0, rows * 4); memset(OM, 0, N * 4); memset(G, 0, rows * (g_dtype ? 2 : 4));
        for (uint64_t i = 0; i < rows; ++i) X[i] = 555.0f;          /* the gaps between rows keep this value */
        for (uint64_t i = 0; i < N; ++i) {
            XG[i] = is_real(i) ? 0.01f * (float)(i + 1) : 0.0f;
            for (uint32_t k = 0; k < K; ++k) X[k * stride + i] = XG[i];
        }
        ora_state s;
        memset(&s, 0, sizeof s);
        s.K = K; s.n = N; s.row_stride = stride; s.n_tensors = 4; s.tensor_offset = OFFS; s.tensor_numel = NUMEL;
        s.tensor_wd_mult = WDM; s.inner = inner; s.g_dtype = g_dtype; s.beta1 = (double)0.9f; s.beta2 = (double)0.999f;
        s.eps = (double)1e-8f; s.weight_decay = (double)0.01f; s.momentum = (double)0.9f; s.inner_nesterov = (int)(H == 2); s.p = 0.4; s.H = H;
        s.outer_lr = (double)0.7f; s.outer_momentum = (double)0.9f; s.outer_nesterov = (int)(K != 2); s.seed = 11 + K;
        s.X = X; s.M = M; s.V = V; s.G = G; s.XG = XG; s.OM = OM; s.tau = tau;
        double gs[3] = {1.0, 0.5, 2.0}, diag[2] = {0, 0}, norms = 0.0;
        uint64_t t = 0;
        for (; t < 2; ++t) {                                       /* DDP warm-up on identical workers */
            fill_gradients(G, g_dtype, K, stride, t);
            double c = ora_clip_scale(ora_mean_grad_norm(G, g_dtype, stride, K, N, gs), 0.5);
            double w[3] = {gs[0] * c, gs[1] * c, gs[2] * c};
            ora_ddp_step(&s, (double)1e-3f, w);
        }
        int syncs = 0;
        for (; t < 14; ++t) {                                      /* Alg. 1 */
            fill_gradients(G, g_dtype, K, stride, t);
            double w[3];
            for (uint32_t k = 0; k < K; ++k) {
                const void *gk = (const char *)G + (uint64_t)k * stride * (g_dtype ? 2 : 4);
                double nk = ora_grad_norm(gk, g_dtype, N);
                norms += nk;
                w[k] = gs[k] * ora_clip_scale(nk, 1.0);
            }
            uint8_t mask[3];
            ora_local_step(&s, t, (double)1e-3f, 16.0, w, NULL, mask);
            if ((t + 1) % H == 0) {
                ora_diagnostics(X, stride, K, XG, N, diag);
                ora_outer_step(&s);
                ++syncs;
            }
        }
        for (uint32_t k = 0; k + 1 < K; ++k)
            for (uint64_t i = N; i < stride; ++i)
                if (X[k * stride + i] != 555.0f) { fprintf(stderr, "gap between rows was written\n"); return 3; }
        double cx = 0.0, cm = 0.0, cv = 0.0;
        for (uint32_t k = 0; k < K; ++k) {
            cx += weighted(X + k * stride, N, 1.0 + 0.5 * k);
            cm += weighted(M + k * stride, N, 1.0 + 0.5 * k);
            cv += weighted(V + k * stride, N, 1.0 + 0.5 * k);
        }
        printf("%d %d %u %u %d %llu %llu %llu %.17g %.17g %.17g %.17g %.17g %.17g %.17g %.17g\n", inner, g_dtype, K, H, syncs,
               (unsigned long long)tau[0], (unsigned long long)tau[K > 1 ? 1 : 0], (unsigned long long)tau[K - 1], cx, cm, cv,
               weighted(XG, N, 1.0), weighted(OM, N, 1.0), diag[0], diag[1], norms);
        free(X); free(M); free(V); free(XG); free(OM); free(G);
    }
    /* the stand-alone kernels on odd sizes, exact-size buffers */
    for (uint64_t n = 1; n <= 9; n += 4) {
        float *x = malloc(n * 4), *xg = malloc(n * 4), *m = calloc(n, 4), *v = calloc(n, 4);
        uint16_t *g = malloc(n * 2);
        for (uint64_t i = 0; i < n; ++i) { x[i] = 0.25f * (float)i; xg[i] = 1.0f; g[i] = 0x3f80; }
        ora_mix(x, xg, n, 0.5);
        ora_adamw(x, m, v, g, 1, n, 1e-3, 0.9, 0.999, 1e-8, 0.01, 1, 1.0);
        ora_sgdm(x, m, g, 1, n, 1e-3, 0.9, 1e-4, 1.0, 1);
        printf("k %llu %.17g %.17g %.17g\n", (unsigned long long)n, weighted(x, n, 1.0), weighted(m, n, 1.0), weighted(v, n, 1.0));
        free(x); free(xg); free(m); free(v); free(g);
    }
    for (uint64_t t = 0; t < 4; ++t)
        printf("d %u %d\n", ora_u24(0xFFFFFFFFFFFFFFFFull, t << 60, 63, 64), ora_draw(7, t, 2, 3, 0.999999));
    return 0;
}
