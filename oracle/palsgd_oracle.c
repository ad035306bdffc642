/*
 * CPU oracle for the PALSGD parameter-update path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It shares no code, header, table or constant with the HIP path and
 * must never be called from it: only the test-suite, the smoke check and the
 * CPU-baseline leg of the benchmark may load it.
 *
 * What it computes: Algorithm 1 of the paper ("Pseudo-Asynchronous Local SGD
 * with Decoupled Optimizers"), executed literally for K worker replicas that
 * live side by side in host memory:
 *
 *   - the Bernoulli(p) branch draw of each worker and step (Alg. 1; App. A.2
 *     basic definitions call it b_k^(t)),
 *   - the pseudo-synchronization step  x_k <- x_k - (alpha_t eta_t / p)(x_k - x)
 *     (Alg. 1; Sec. 4.1, second equation),
 *   - the gradient step  x_k <- InnerOPT(x_k, g_k, alpha_t / (1-p))
 *     (Alg. 1; Sec. 4.1, first equation) for InnerOPT = AdamW or SGD with
 *     momentum (Sec. 4.3; App. B, training configuration),
 *   - every H steps the outer gradient  Delta = mean_k (x - x_k)
 *     (Alg. 1; Sec. 4.2; All-Reduce is the mean, Sec. 3.1) and the
 *     OuterOPT step with Nesterov momentum (Sec. 4.2, Sec. 4.3), after which
 *     every worker restarts from the new global model (Sec. 2.1 states that
 *     the workers share one starting point every H local steps; App. A.5, proof
 *     of Lemma 4: x^(t) = x_k^(t-)).
 *
 * Around Alg. 1, each with its own routine and pins: the DDP step of the
 * warm-up phase (Sec. 3.1, Sec. 4.3), gradient clipping by the global norm of
 * one worker's gradient and of the averaged gradient (App. B), the consensus
 * distance and |Delta|^2 of the analysis (App. A.3), the Nesterov form of the
 * SGD-momentum InnerOPT and AdamW as OuterOPT (the optimizer pairs of App. C).
 *
 * Precision: state (x_k, x, optimizer moments) is stored in fp32, the storage
 * type of the device path.  Every element update reads the stored values,
 * evaluates the whole update in fp64 and rounds to fp32 once per stored value.
 * bf16 gradients are widened exactly.  No blocking, fusion or reordering: each
 * routine is one loop over elements, the K-sum runs over k in ascending order.
 *
 * Parity status: every routine below is pinned by tests/test_oracle_*.py
 * against closed forms, library optimizers in float64, special cases the
 * paper fixes (p=0 => DiLoCo / Local SGD; H=1, outer lr 1, no momentum =>
 * synchronous averaging; K=1 => outer step is the identity) and an
 * independently written brute-force formulation on tiny P.  The numeric
 * defaults of AdamW / SGD-momentum / Nesterov hyper-parameters are inputs, not
 * facts of the paper (it prints none): "parity unpinned" applies to those
 * default VALUES only, never to the arithmetic.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Threads: the element loops are split statically over OpenMP threads when   */
/* the library is built with -fopenmp.  Results do not depend on the count    */
/* (no cross-element arithmetic).                                             */
/* ------------------------------------------------------------------------- */
static int g_threads = 1;

void ora_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int ora_get_threads(void) { return g_threads; }

/* ------------------------------------------------------------------------- */
/* Branch draw b_k^(t)  (Alg. 1: a uniform b is compared with p; App. A.2).  */
/*                                                                           */
/* The paper names no generator.  Both sides of the parity check implement   */
/* the SplitMix64 output function (Steele, Lea, Flood 2014; public domain)   */
/* as a counter hash of idx = t*K + k:                                        */
/*   z = seed + (idx+1) * 0x9E3779B97F4A7C15                                  */
/*   z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9                                 */
/*   z = (z ^ (z >> 27)) * 0x94D049BB133111EB                                 */
/*   z =  z ^ (z >> 31)                                                       */
/* u24 = z >> 40 is a uniform 24-bit integer; the worker mixes iff            */
/* u24 < floor(p * 2^24).  With b = (u24+1)/2^24 in (0,1] this is b <= p on   */
/* the 2^-24 grid; p = 0 never mixes.                                         */
/* ------------------------------------------------------------------------- */
uint32_t ora_u24(uint64_t seed, uint64_t t, uint32_t k, uint32_t K)
{
    uint64_t idx = t * (uint64_t)K + (uint64_t)k;
    uint64_t z = seed + (idx + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z = z ^ (z >> 31);
    return (uint32_t)(z >> 40);
}

int ora_draw(uint64_t seed, uint64_t t, uint32_t k, uint32_t K, double p)
{
    uint32_t threshold = (uint32_t)floor(p * 16777216.0);
    return ora_u24(seed, t, k, K) < threshold ? 1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Gradient element as a double.  dtype 0: fp32; dtype 1: bf16 (upper 16 bits */
/* of an fp32, widened exactly); dtype 2: fp64 (an averaged gradient that     */
/* was never rounded, used by the DDP step).                                  */
/* ------------------------------------------------------------------------- */
static double grad_at(const void *g, int dtype, uint64_t i)
{
    if (dtype == 0)
        return (double)((const float *)g)[i];
    if (dtype == 2)
        return ((const double *)g)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)g)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------------- */
/* Pseudo-synchronization step (Alg. 1; Sec. 4.1 second equation; EMA form    */
/* (1-beta) x_k + beta x with beta = alpha_t eta_t / p).  beta is passed in   */
/* already evaluated in double.                                               */
/* ------------------------------------------------------------------------- */
void ora_mix(float *x, const float *xg, uint64_t n, double beta)
{
    int64_t i;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (i = 0; i < (int64_t)n; ++i) {
        double xk = (double)x[i];
        double xglob = (double)xg[i];
        x[i] = (float)(xk - beta * (xk - xglob));
    }
}

/* ------------------------------------------------------------------------- */
/* InnerOPT = AdamW (Sec. 4.3; Loshchilov & Hutter, "Decoupled Weight Decay   */
/* Regularization", Alg. 2 with the schedule multiplier folded into lr):      */
/*   m <- b1 m + (1-b1) g          v <- b2 v + (1-b2) g^2                     */
/*   mhat = m / (1 - b1^tau)       vhat = v / (1 - b2^tau)                    */
/*   x <- x - lr ( mhat / (sqrt(vhat) + eps) + wd x )                         */
/* tau is the number of gradient steps this replica has taken, this one       */
/* included (a mixing step does not call InnerOPT and does not advance it).   */
/* lr is the value handed to InnerOPT, i.e. alpha_t / (1-p) (Alg. 1).         */
/* ------------------------------------------------------------------------- */
void ora_adamw(float *x, float *m, float *v, const void *g, int g_dtype,
               uint64_t n, double lr, double beta1, double beta2, double eps,
               double wd, uint64_t tau, double grad_scale)
{
    double bc1 = 1.0 - pow(beta1, (double)tau);
    double bc2 = 1.0 - pow(beta2, (double)tau);
    int64_t i;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (i = 0; i < (int64_t)n; ++i) {
        double gi = grad_scale * grad_at(g, g_dtype, (uint64_t)i);
        double xi = (double)x[i];
        double mi = beta1 * (double)m[i] + (1.0 - beta1) * gi;
        double vi = beta2 * (double)v[i] + (1.0 - beta2) * gi * gi;
        double mhat = mi / bc1;
        double vhat = vi / bc2;
        m[i] = (float)mi;
        v[i] = (float)vi;
        x[i] = (float)(xi - lr * (mhat / (sqrt(vhat) + eps) + wd * xi));
    }
}

/* ------------------------------------------------------------------------- */
/* InnerOPT = SGD with momentum (App. B names it for the vision runs, with    */
/* weight decay 1e-4 in the VGG run), heavy-ball form with dampening 0, weight decay coupled    */
/* into the gradient:                                                         */
/*   d = g + wd x      buf <- mu buf + d      x <- x - lr buf                 */
/* (buf starts at 0, so the first step gives buf = d).  mu = 0 is plain SGD,  */
/* the InnerOPT of the paper's Theorem 1.  With nesterov != 0 the step looks  */
/* ahead along the momentum (Sutskever et al. 2013, the form the optimizer    */
/* comparison of App. C varies):   x <- x - lr (d + mu buf).                  */
/* ------------------------------------------------------------------------- */
void ora_sgdm(float *x, float *buf, const void *g, int g_dtype, uint64_t n,
              double lr, double momentum, double wd, double grad_scale, int nesterov)
{
    int64_t i;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (i = 0; i < (int64_t)n; ++i) {
        double xi = (double)x[i];
        double d = grad_scale * grad_at(g, g_dtype, (uint64_t)i) + wd * xi;
        double bi = momentum * (double)buf[i] + d;
        buf[i] = (float)bi;
        x[i] = (float)(xi - lr * (nesterov ? d + momentum * bi : bi));
    }
}

/* ------------------------------------------------------------------------- */
/* Outer step (Alg. 1, the two lines of the synchronisation branch; Sec. 4.2, */
/* both equations; Sec. 3.1 for All-Reduce = mean):                           */
/*   Delta = (1/K) sum_k (x - x_k) = x - (1/K) sum_k x_k     (k ascending)    */
/*   OuterOPT, SGD with (Nesterov) momentum, Sutskever et al. 2013 in the     */
/*   buffer form used by common deep-learning libraries (dampening 0):        */
/*     om <- mu om + Delta                                                    */
/*     x  <- x - lr_o (Delta + mu om)      if nesterov                        */
/*     x  <- x - lr_o om                   otherwise                          */
/*   then every worker restarts from x:  x_k <- x for all k                   */
/*   (Sec. 2.1; App. A.5: x^(t) = xbar^(t-) = x_k^(t-)).                      */
/* X is replica-major: replica k starts at X + k*row_stride.                  */
/* ------------------------------------------------------------------------- */
void ora_outer(float *X, uint64_t row_stride, uint32_t K, float *xg, float *om,
               uint64_t n, double lr_o, double mu_o, int nesterov)
{
    int64_t i;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (i = 0; i < (int64_t)n; ++i) {
        double sum = 0.0;
        for (uint32_t k = 0; k < K; ++k)
            sum += (double)X[(uint64_t)k * row_stride + (uint64_t)i];
        double xi = (double)xg[i];
        double delta = xi - sum / (double)K;
        double omi = mu_o * (double)om[i] + delta;
        double step = nesterov ? delta + mu_o * omi : omi;
        float xnew = (float)(xi - lr_o * step);
        om[i] = (float)omi;
        xg[i] = xnew;
        for (uint32_t k = 0; k < K; ++k)
            X[(uint64_t)k * row_stride + (uint64_t)i] = xnew;
    }
}

/* ------------------------------------------------------------------------- */
/* Outer step with OuterOPT = AdamW, one of the optimizer pairs that App. C   */
/* compares (Alg. 1 leaves OuterOPT open): Delta as above plays the gradient, */
/* om and ov are the two moments, step = number of this outer step (from 1):  */
/*   om <- b1 om + (1-b1) Delta        ov <- b2 ov + (1-b2) Delta^2           */
/*   x  <- x - lr_o ( (om/(1-b1^step)) / (sqrt(ov/(1-b2^step)) + eps) + wd x )*/
/* then every worker restarts from x.                                         */
/* ------------------------------------------------------------------------- */
void ora_outer_adamw(float *X, uint64_t row_stride, uint32_t K, float *xg, float *om,
                     float *ov, uint64_t n, double lr_o, double b1, double b2, double eps,
                     double wd, uint64_t step)
{
    const double bc1 = 1.0 - pow(b1, (double)step);
    const double bc2 = 1.0 - pow(b2, (double)step);
    int64_t i;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (i = 0; i < (int64_t)n; ++i) {
        double sum = 0.0;
        for (uint32_t k = 0; k < K; ++k)
            sum += (double)X[(uint64_t)k * row_stride + (uint64_t)i];
        double xi = (double)xg[i];
        double delta = xi - sum / (double)K;
        double m = b1 * (double)om[i] + (1.0 - b1) * delta;
        double v = b2 * (double)ov[i] + (1.0 - b2) * delta * delta;
        float xnew = (float)(xi - lr_o * ((m / bc1) / (sqrt(v / bc2) + eps) + wd * xi));
        om[i] = (float)m;
        ov[i] = (float)v;
        xg[i] = xnew;
        for (uint32_t k = 0; k < K; ++k)
            X[(uint64_t)k * row_stride + (uint64_t)i] = xnew;
    }
}

/* ------------------------------------------------------------------------- */
/* Whole-algorithm driver: one iteration t of the inner loop of Alg. 1 for    */
/* all K workers, in the order the listing gives: draw, local update (mix or  */
/* gradient step), then the (t+1) mod H test and the outer step.              */
/* ------------------------------------------------------------------------- */
typedef struct {
    uint32_t K;
    uint64_t n;              /* elements per replica row that are updated     */
    uint64_t row_stride;     /* elements between consecutive replica rows     */
    uint32_t n_tensors;      /* tensors tile [0,n) in order; see offsets      */
    const uint64_t *tensor_offset; /* start element of each tensor            */
    const uint64_t *tensor_numel;  /* element count of each tensor            */
    const float *tensor_wd_mult;   /* per-tensor multiplier on weight decay,  */
                                   /* NULL = 1 everywhere                     */
    int inner;               /* 0 AdamW, 1 SGD-momentum                       */
    int g_dtype;             /* 0 fp32, 1 bf16                                */
    double beta1, beta2, eps, weight_decay; /* AdamW (weight_decay also SGDM) */
    double momentum;         /* SGDM                                          */
    int inner_nesterov;      /* SGDM: Nesterov form of the momentum step      */
    double p;                /* mixing probability                            */
    uint32_t H;              /* sync interval                                 */
    double outer_lr, outer_momentum;
    int outer_nesterov;
    uint64_t seed;
    /* state */
    float *X, *M, *V;        /* [K][row_stride]; V unused by SGDM             */
    const void *G;           /* [K][row_stride] gradients in g_dtype          */
    float *XG, *OM;          /* [row_stride]                                  */
    uint64_t *tau;           /* [K] gradient steps taken per replica          */
    uint64_t n_outer;        /* outer steps taken                             */
    /* OuterOPT = AdamW instead of the SGD family (outer_opt != 0)             */
    int outer_opt;
    double outer_beta1, outer_beta2, outer_eps, outer_weight_decay;
    float *OV;               /* [row_stride] second moment of the outer AdamW */
} ora_state;

/* Local update of step t for every replica.  mask_out (nullable) receives    */
/* the K branch decisions actually used (1 = mixed).  mask_override           */
/* (nullable) replaces the drawn decisions.  grad_scale (nullable) holds one  */
/* multiplier per replica applied to its gradient before InnerOPT (hook for   */
/* gradient clipping, App. B).                                                */
void ora_local_step(ora_state *s, uint64_t t, double alpha_t, double eta_t,
                    const double *grad_scale, const uint8_t *mask_override,
                    uint8_t *mask_out)
{
    for (uint32_t k = 0; k < s->K; ++k) {
        int b = mask_override ? (mask_override[k] != 0)
                              : ora_draw(s->seed, t, k, s->K, s->p);
        if (mask_out)
            mask_out[k] = (uint8_t)b;
        float *xk = s->X + (uint64_t)k * s->row_stride;
        if (b) {
            /* pseudo-synchronization step */
            double beta = alpha_t * eta_t / s->p;
            ora_mix(xk, s->XG, s->n, beta);
        } else {
            /* gradient step with the rescaled learning rate */
            double lr = alpha_t / (1.0 - s->p);
            double gs = grad_scale ? grad_scale[k] : 1.0;
            s->tau[k] += 1;
            for (uint32_t j = 0; j < s->n_tensors; ++j) {
                uint64_t off = s->tensor_offset[j];
                uint64_t len = s->tensor_numel[j];
                double wd = s->weight_decay *
                            (s->tensor_wd_mult ? (double)s->tensor_wd_mult[j] : 1.0);
                size_t gbytes = s->g_dtype == 0 ? 4 : 2;
                const void *gk = (const char *)s->G +
                                 ((uint64_t)k * s->row_stride + off) * gbytes;
                if (s->inner == 0) {
                    float *mk = s->M + (uint64_t)k * s->row_stride;
                    float *vk = s->V + (uint64_t)k * s->row_stride;
                    ora_adamw(xk + off, mk + off, vk + off, gk, s->g_dtype, len,
                              lr, s->beta1, s->beta2, s->eps, wd, s->tau[k], gs);
                } else {
                    float *bk = s->M + (uint64_t)k * s->row_stride;
                    ora_sgdm(xk + off, bk + off, gk, s->g_dtype, len, lr,
                             s->momentum, wd, gs, s->inner_nesterov);
                }
            }
        }
    }
}

void ora_outer_step(ora_state *s)
{
    if (s->outer_opt)
        ora_outer_adamw(s->X, s->row_stride, s->K, s->XG, s->OM, s->OV, s->n, s->outer_lr,
                        s->outer_beta1, s->outer_beta2, s->outer_eps, s->outer_weight_decay,
                        s->n_outer + 1);
    else
        ora_outer(s->X, s->row_stride, s->K, s->XG, s->OM, s->n, s->outer_lr,
                  s->outer_momentum, s->outer_nesterov);
    s->n_outer += 1;
}

/* One full iteration of Alg. 1's inner loop; returns 1 if it synchronised.   */
int ora_iteration(ora_state *s, uint64_t t, double alpha_t, double eta_t,
                  const double *grad_scale, const uint8_t *mask_override,
                  uint8_t *mask_out)
{
    ora_local_step(s, t, alpha_t, eta_t, grad_scale, mask_override, mask_out);
    if ((t + 1) % s->H == 0) {
        ora_outer_step(s);
        return 1;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* DDP step (Sec. 3.1: an All-Reduce of the gradient at every step before the */
/* optimizer update, so that all workers apply the same update; Sec. 4.3 and  */
/* Sec. 5.1: the warm-up phase that precedes PALSGD):                         */
/*   gbar = (1/K) sum_k grad_scale_k g_k           (k ascending, never rounded)*/
/*   x <- InnerOPT(x, gbar, alpha_t)               (no 1/(1-p) rescale: there  */
/*                                                  is no mixing branch here)  */
/*   every worker holds the result: x_k <- x, and every worker's InnerOPT      */
/*   state is the common one.                                                  */
/* Precondition (true from initialisation through the warm-up): all workers    */
/* are identical; the common model is read from XG, the common InnerOPT state  */
/* from worker 0.                                                              */
/* ------------------------------------------------------------------------- */
void ora_ddp_step(ora_state *s, double alpha_t, const double *grad_scale)
{
    const uint64_t n = s->n;
    double *gbar = (double *)malloc(sizeof(double) * (n ? n : 1));
    size_t gbytes = s->g_dtype == 0 ? 4 : 2;
    for (uint64_t i = 0; i < n; ++i) {
        double sum = 0.0;
        for (uint32_t k = 0; k < s->K; ++k) {
            const void *gk = (const char *)s->G + (uint64_t)k * s->row_stride * gbytes;
            sum += (grad_scale ? grad_scale[k] : 1.0) * grad_at(gk, s->g_dtype, i);
        }
        gbar[i] = sum / (double)s->K;
    }
    s->tau[0] += 1;
    for (uint32_t j = 0; j < s->n_tensors; ++j) {
        uint64_t off = s->tensor_offset[j];
        uint64_t len = s->tensor_numel[j];
        double wd = s->weight_decay * (s->tensor_wd_mult ? (double)s->tensor_wd_mult[j] : 1.0);
        if (s->inner == 0)
            ora_adamw(s->XG + off, s->M + off, s->V + off, gbar + off, 2, len, alpha_t, s->beta1,
                      s->beta2, s->eps, wd, s->tau[0], 1.0);
        else
            ora_sgdm(s->XG + off, s->M + off, gbar + off, 2, len, alpha_t, s->momentum, wd, 1.0,
                     s->inner_nesterov);
    }
    for (uint32_t k = 0; k < s->K; ++k) {
        memcpy(s->X + (uint64_t)k * s->row_stride, s->XG, sizeof(float) * n);
        if (k > 0) {
            s->tau[k] = s->tau[0];
            memcpy(s->M + (uint64_t)k * s->row_stride, s->M, sizeof(float) * n);
            if (s->inner == 0)
                memcpy(s->V + (uint64_t)k * s->row_stride, s->V, sizeof(float) * n);
        }
    }
    free(gbar);
}

/* ------------------------------------------------------------------------- */
/* Gradient clipping (App. B says the GPT-Neo runs clip gradients; neither    */
/* threshold nor norm is printed).  Reading: clipping by the global L2 norm of */
/* one worker's gradient, the common deep-learning convention:                */
/*   norm_k = sqrt(sum_i g_k[i]^2)       scale_k = min(1, c / (norm_k + 1e-6)) */
/* The scale is what the local update takes as grad_scale[k].                 */
/* ------------------------------------------------------------------------- */
double ora_grad_norm(const void *g, int g_dtype, uint64_t n)
{
    double sum = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double gi = grad_at(g, g_dtype, i);
        sum += gi * gi;
    }
    return sqrt(sum);
}

/* Norm of the averaged gradient, for clipping in the DDP phase (there the     */
/* gradients are averaged before the optimizer sees them, Sec. 3.1, so the    */
/* norm that is clipped is that of gbar = (1/K) sum_k grad_scale_k g_k).       */
double ora_mean_grad_norm(const void *G, int g_dtype, uint64_t row_stride, uint32_t K, uint64_t n,
                          const double *grad_scale)
{
    size_t gbytes = g_dtype == 0 ? 4 : 2;
    double sum = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double gbar = 0.0;
        for (uint32_t k = 0; k < K; ++k) {
            const void *gk = (const char *)G + (uint64_t)k * row_stride * gbytes;
            gbar += (grad_scale ? grad_scale[k] : 1.0) * grad_at(gk, g_dtype, i);
        }
        gbar /= (double)K;
        sum += gbar * gbar;
    }
    return sqrt(sum);
}

double ora_clip_scale(double norm, double max_norm)
{
    double c = max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ------------------------------------------------------------------------- */
/* Diagnostics of the theory (App. A.3, the consensus-distance lemma):        */
/*   Xi = (1/K) sum_k |x_k - x|^2   (zero right after a synchronisation)       */
/*   |Delta|^2 with Delta = x - (1/K) sum_k x_k  (the outer gradient, Sec 4.2) */
/* out[0] = Xi, out[1] = |Delta|^2.  Nothing is modified.                      */
/* ------------------------------------------------------------------------- */
void ora_diagnostics(const float *X, uint64_t row_stride, uint32_t K, const float *xg, uint64_t n,
                     double *out)
{
    double xi = 0.0, d2 = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        double sum = 0.0;
        for (uint32_t k = 0; k < K; ++k) {
            double d = (double)X[(uint64_t)k * row_stride + i] - (double)xg[i];
            xi += d * d;
            sum += (double)X[(uint64_t)k * row_stride + i];
        }
        double delta = (double)xg[i] - sum / (double)K;
        d2 += delta * delta;
    }
    out[0] = xi / (double)K;
    out[1] = d2;
}
