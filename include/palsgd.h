/*
 * palsgd.h - C ABI of the PALSGD parameter-update path for AMD MI355X (gfx950).
 *
 * The library updates K worker replicas of a model that live side by side in one
 * GPU's memory, following Algorithm 1 of "Pseudo-Asynchronous Local SGD" (PALSGD):
 * per step either a pseudo-synchronization (mixing) step toward the stale global
 * model or an InnerOPT gradient step, and every H steps the outer step.
 *
 * Data layout (all device memory, caller-owned, fp32 unless noted):
 *   X [K][row_stride]  local models x_k                      (Sec. 4.1)
 *   M [K][row_stride]  InnerOPT first moment / momentum buffer
 *   V [K][row_stride]  InnerOPT second moment (AdamW only; may be NULL for SGDM)
 *   G [K][row_stride]  gradients g_k, fp32 or bf16, written by the caller before
 *                      each step                             (Sec. 3, WorkerOPT eq.)
 *   XG[row_stride]     global model copy x                   (Sec. 4.1)
 *   OM[row_stride]     OuterOPT momentum buffer              (Sec. 4.3)
 *   OV[row_stride]     OuterOPT second moment (only with OuterOPT = AdamW, else NULL)
 * A row is the flat concatenation of the model's tensors; every tensor starts at a
 * multiple of 64 elements and the padded row length P_padded is a multiple of 256
 * (palsgd_layout).  Padding elements must be zero in x0 and in G; the update keeps them
 * zero.  row_stride >= P_padded, a multiple of 64; a multiple of 256 (such as P_padded
 * itself) keeps every wavefront's 1 KiB access 1 KiB-aligned in every row, which is
 * about 3 % faster than rows shifted against each other by 256 B.
 * Every base pointer must be 16-byte aligned; 1 KiB alignment is recommended for the
 * same reason (large allocations of the HIP runtime and of PyTorch have it).
 *
 * Ownership: the library borrows the buffer pointers from palsgd_init until
 * palsgd_destroy and owns only its context, a device-side table of weight-decay
 * values (4 bytes per 64 elements of a row, only when tensor_wd_mult is not
 * uniform), the scratch of the scalar reductions (P_padded/32 bytes, or
 * K * P_padded/1024 if that is more) and the 2.3 KB device schedule of the capturable
 * mode.  palsgd_init allocates all of it; no other entry point allocates or frees
 * device memory, so every one of them may be the first call inside a stream capture.
 * Streams: `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 * device work is enqueued on it; calls return without waiting.
 * Errors: every entry point returns a palsgd_status and never aborts; argument
 * errors are found before any launch and leave all state untouched.  The text of
 * the last error of a context is available through palsgd_last_error.  The library
 * gets plain pointers: it checks alignment and NULLs, not sizes; every row buffer must
 * hold (K-1) * row_stride + P_padded elements, every single-row buffer P_padded.
 * palsgd_destroy frees the library's device memory: the caller waits for the streams
 * it used first.
 * Threads: a context must not be used from two threads at once.
 */
#ifndef PALSGD_H
#define PALSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PALSGD_MAX_K 64u /* largest worker count the paper runs (App. B, CIFAR-10 simulation) */

typedef struct palsgd_ctx palsgd_ctx; /* opaque */

typedef enum {
    PALSGD_OK = 0,
    PALSGD_EINVAL = 1, /* bad argument; nothing was launched            */
    PALSGD_ENOMEM = 2, /* host or device allocation of library state    */
    PALSGD_EHIP = 3,   /* a HIP call failed; see palsgd_last_error       */
    PALSGD_ESTATE = 4  /* call not valid in the context's current state */
} palsgd_status;

typedef enum { PALSGD_INNER_ADAMW = 0, PALSGD_INNER_SGDM = 1 } palsgd_inner_opt;
typedef enum { PALSGD_GRAD_F32 = 0, PALSGD_GRAD_BF16 = 1 } palsgd_grad_dtype;
typedef enum { PALSGD_OUTER_SGD = 0, PALSGD_OUTER_ADAMW = 1 } palsgd_outer_opt;

/* Inputs of Algorithm 1 plus the constants of the two optimizers (Sec. 4.3). */
typedef struct {
    uint32_t K;                   /* workers, 1..PALSGD_MAX_K                               */
    uint32_t n_tensors;           /* >= 1                                                   */
    uint64_t P;                   /* logical parameter count: 0 = not stated, else it must
                                     equal the sum of tensor_numel (checked: EINVAL)         */
    const uint64_t *tensor_numel; /* host array [n_tensors], each >= 1; copied at init      */
    const float *tensor_wd_mult;  /* host array [n_tensors] or NULL (= 1): per-tensor
                                     multiplier on weight_decay                             */
    int32_t inner;                /* palsgd_inner_opt                                       */
    int32_t grad_dtype;           /* palsgd_grad_dtype                                      */
    float beta1, beta2, eps;      /* AdamW moments and epsilon (eps > 0: zero padding stays zero) */
    float weight_decay;           /* AdamW: decoupled; SGDM: added to the gradient          */
    float momentum;               /* SGDM momentum (dampening 0)                            */
    int32_t inner_nesterov;       /* SGDM: 1 = Nesterov form x -= lr (d + mu buf), 0 = heavy
                                     ball x -= lr buf (the optimizer comparison of App. C);
                                     ignored by AdamW                                       */
    double p;                     /* mixing probability, 0 <= p < 1 (Alg. 1 input)          */
    uint32_t H;                   /* synchronization interval, >= 1 (Alg. 1 input)          */
    float outer_lr;               /* OuterOPT learning rate                                 */
    float outer_momentum;         /* OuterOPT momentum, 0 = plain SGD                       */
    int32_t outer_nesterov;       /* 1: Nesterov momentum (Sec. 4.3), 0: heavy ball         */
    uint64_t seed;                /* seed of the branch draws                               */
    int32_t outer_opt;            /* palsgd_outer_opt: SGD family above (Sec. 4.3), or AdamW
                                     with Delta as its gradient (the optimizer pairs of App. C) */
    float outer_beta1, outer_beta2, outer_eps; /* OuterOPT = AdamW: moments and epsilon     */
    float outer_weight_decay;     /* OuterOPT = AdamW: decoupled weight decay               */
} palsgd_config;

typedef struct {
    float *X, *M, *V; /* device */
    void *G;          /* device, float or bf16 according to grad_dtype */
    float *XG, *OM;   /* device; OM: OuterOPT momentum buffer, or first moment with AdamW */
    uint64_t row_stride;
    float *OV;        /* device [row_stride]: second moment of OuterOPT = AdamW, else NULL */
} palsgd_buffers;

/* Flat layout of a row: tensor_offset[j] (host array [n_tensors], may be NULL) is the
 * start element of tensor j, each start rounded up to a multiple of 64; *P_padded is
 * the padded row length, rounded up to a multiple of 256.  Only K-independent fields of the config are read
 * (n_tensors, tensor_numel, P).  EINVAL on NULL pointers, n_tensors == 0, a zero numel, or
 * a non-zero P that is not the sum of tensor_numel. */
palsgd_status palsgd_layout(const palsgd_config *cfg, uint64_t *P_padded, uint64_t *tensor_offset);

/* Alg. 1, initialisation x_k^(0) <- x^(0): creates a context over the caller's buffers.  If x0_dev
 * (device, P_padded floats, padding zero) is not NULL, it is copied into XG and every
 * row of X, and M, V, OM are cleared, on `stream`; if NULL the buffers are taken as
 * they are (resume).  EINVAL: K outside 1..64, H == 0, p outside [0,1), NULL or
 * misaligned buffers, row_stride < P_padded or not a multiple of 64, P_padded > 2^33,
 * beta/eps/momentum outside their ranges, V == NULL with AdamW.  When the weight-decay
 * multipliers differ between tensors (and weight_decay != 0) a device table of one float
 * per 64 row elements is allocated and filled here, and so are the reduction scratch and
 * the device schedule (ENOMEM / EHIP if that fails): no later call allocates.  On failure
 * *out is NULL.  With no GPU visible the context is still created, for palsgd_draw and the
 * scalar state calls (host-side checks); every call of it that would launch returns EHIP. */
palsgd_status palsgd_init(const palsgd_config *cfg, const palsgd_buffers *buf, const float *x0_dev,
                          void *stream, palsgd_ctx **out);

/* Branch draws b_k^(t) of step t for all K workers (Alg. 1: a uniform b compared with p;
 * App. A.2): mask_out (host, K bytes) gets 1 where worker k takes the mixing step.
 * Pure function of (seed, t, k): SplitMix64 output function of the counter t*K+k,
 * top 24 bits compared with floor(p * 2^24).  Host only, no device work. */
palsgd_status palsgd_draw(const palsgd_ctx *ctx, uint64_t t, uint8_t *mask_out);

/* Gradient step of step t (Alg. 1, the branch b > p; Sec. 4.1 first equation):
 * x_k <- InnerOPT(x_k, grad_scale[k] * G[k], alpha_t / (1-p)) for every worker whose
 * draw is 0, and advances that worker's InnerOPT step count.  grad_scale: host array
 * [K] or NULL (= 1).  mask_override: host array [K] or NULL; if given it replaces the
 * draws (1 = this worker mixes, so it is skipped here).  One launch; no launch if no
 * worker takes the branch. */
palsgd_status palsgd_inner_step(palsgd_ctx *ctx, uint64_t t, float alpha_t, const float *grad_scale,
                                const uint8_t *mask_override, void *stream);

/* Pseudo-synchronization step of step t (Alg. 1, the branch b <= p;
 * Sec. 4.1 second equation): x_k <- x_k - (alpha_t * eta_t / p) (x_k - XG) for every
 * worker whose draw is 1.  InnerOPT state is not touched.  EINVAL if a worker is to
 * mix while p == 0 (the coefficient is undefined).  No launch if no worker mixes. */
palsgd_status palsgd_pseudo_sync(palsgd_ctx *ctx, uint64_t t, float alpha_t, float eta_t,
                                 const uint8_t *mask_override, void *stream);

/* Both branches of step t in ONE launch: equal to palsgd_inner_step followed by
 * palsgd_pseudo_sync for the same t (they touch disjoint workers). */
palsgd_status palsgd_step(palsgd_ctx *ctx, uint64_t t, float alpha_t, float eta_t,
                          const float *grad_scale, const uint8_t *mask_override, void *stream);

/* Step t of Alg. 1 when (t+1) mod H == 0, whole: palsgd_step followed by
 * palsgd_outer_step fused into ONE launch (followed by the launch that restarts the
 * workers' rows where palsgd_outer_step uses one), with identical results.  The local update's new x_k
 * stay in registers and go straight into the outer gradient, which saves one write and
 * one read of the K rows of X (8K of 34K+16 bytes per element with AdamW).  Arguments as
 * palsgd_step. */
palsgd_status palsgd_step_sync(palsgd_ctx *ctx, uint64_t t, float alpha_t, float eta_t,
                               const float *grad_scale, const uint8_t *mask_override, void *stream);

/* Outer step (Alg. 1, the two lines of the synchronisation branch; Sec. 4.2):
 * Delta = XG - (1/K) sum_k X[k];  OM <- mu OM + Delta;
 * XG <- XG - outer_lr (Delta + mu OM) (Nesterov) or XG - outer_lr OM;  X[k] <- XG for
 * all k (Sec. 2.1: workers restart from the global model).  One launch; with K >= 24 and
 * rows of at most 192 MiB (the global model then stays in the memory-side cache) the restart
 * of the K rows is a second launch on the same stream: short wavefronts that store eight
 * rows each fill them 5-20 % faster than the reducing wavefronts can.  With outer_opt = AdamW:
 * OM <- b1 OM + (1-b1) Delta, OV <- b2 OV + (1-b2) Delta^2,
 * XG <- XG - outer_lr ((OM/(1-b1^n)) / (sqrt(OV/(1-b2^n)) + eps) + wd XG), n = number of
 * this outer step (from 1; part of palsgd_get_state / palsgd_set_state).  The bias
 * corrections are launch arguments computed from n on the host, so with AdamW this call
 * (and palsgd_step_sync, palsgd_outer_step_diag) returns ESTATE while `stream` is being
 * captured into a HIP graph.  The caller decides when
 * ((t+1) mod H == 0 in Alg. 1); t is recorded for diagnostics only. */
palsgd_status palsgd_outer_step(palsgd_ctx *ctx, uint64_t t, void *stream);

/* palsgd_outer_step that also reports, at no extra memory traffic, the diagnostics of
 * App. A.3 taken just before the update: diag_out_dev[0] = consensus distance
 * Xi = (1/K) sum_k |x_k - XG|^2, diag_out_dev[1] = |Delta|^2 (device array of 2 floats;
 * EINVAL if NULL).  Uses the library's reduction scratch (see palsgd_clip_grad_norm). */
palsgd_status palsgd_outer_step_diag(palsgd_ctx *ctx, uint64_t t, float *diag_out_dev, void *stream);

/* DDP step of the warm-up phase that precedes PALSGD (Sec. 3.1: an All-Reduce of the
 * gradient at every step before the optimizer update; Sec. 4.3, Sec. 5.1):
 * gbar = (1/K) sum_k grad_scale[k] G[k];  x <- InnerOPT(x, gbar, alpha_t) (no 1/(1-p)
 * rescale: there is no mixing branch);  the result is stored to XG and to every row of X
 * (by a second launch under the same condition as in palsgd_outer_step), and every worker's
 * step count advances.  The InnerOPT state of the identical workers
 * is kept once, in worker 0's rows of M, V; rows 1..K-1 are stale during the warm-up and
 * are filled from row 0 by the first palsgd_inner_step / palsgd_pseudo_sync / palsgd_step /
 * palsgd_step_sync / palsgd_outer_step / palsgd_diagnostics / palsgd_capturable_begin that
 * follows, or by palsgd_ddp_finish.
 * Precondition: all workers are identical (true from palsgd_init through the warm-up);
 * the common model is read from XG, the common InnerOPT state from worker 0.  ESTATE if
 * the workers' step counts differ.  OM is not touched.  The per-worker clipping scales of
 * palsgd_clip_grad_norm are not consumed here; the scale of palsgd_clip_mean_grad_norm is. */
palsgd_status palsgd_ddp_step(palsgd_ctx *ctx, uint64_t t, float alpha_t, const float *grad_scale, void *stream);

/* The same DDP step with the model kept once as well (Sec. 3.1: in DDP every worker holds
 * the same model): the new model is stored to XG only, which saves the K row stores of
 * palsgd_ddp_step (4K of 4K + 24 + K*sizeof(g) bytes per element with AdamW).  During such
 * a warm-up the workers' model IS XG: the caller computes every worker's gradient at XG,
 * and the K rows of X are stale.  They are filled from XG, together with the InnerOPT
 * state, by palsgd_ddp_finish or by the first later call of this context that reads or
 * updates them (palsgd_inner_step, palsgd_pseudo_sync, palsgd_step, palsgd_step_sync,
 * palsgd_outer_step, palsgd_outer_step_diag, palsgd_diagnostics, palsgd_capturable_begin);
 * a palsgd_ddp_step stores all rows itself.  Arguments, preconditions and errors as
 * palsgd_ddp_step. */
palsgd_status palsgd_ddp_step_shared(palsgd_ctx *ctx, uint64_t t, float alpha_t, const float *grad_scale,
                                     void *stream);

/* End of the warm-up made explicit: copies worker 0's InnerOPT state into rows 1..K-1 of
 * M, V, and XG into the K rows of X, where DDP steps left them stale (one launch); no
 * launch otherwise.  Call it before capturing PALSGD steps into a HIP graph: left to the
 * first captured call, the broadcast would be part of the graph and every replay would
 * hand the workers the common state again. */
palsgd_status palsgd_ddp_finish(palsgd_ctx *ctx, void *stream);

/* Gradient clipping by the global L2 norm of each worker's gradient (App. B says the GPT-Neo runs
 * clip gradients; the paper prints no threshold): norm_k = |G[k]|_2 and
 * scale_k = min(1, max_norm / (norm_k + 1e-6)) are computed on the device, without a host
 * round trip.  The next palsgd_inner_step / palsgd_step / palsgd_step_sync /
 * palsgd_step_capturable of this context multiplies worker k's gradient by scale_k (on top
 * of grad_scale[k]) and forgets the scales, whether or not worker k (or any worker) takes
 * the gradient branch in that step: they belong to that step's gradients.
 * norms_out_dev: device array of K floats that receives the norms, or NULL.
 * palsgd_clip_grad_norm, palsgd_clip_mean_grad_norm, palsgd_diagnostics and
 * palsgd_outer_step_diag share the context's reduction scratch and must be issued on one
 * stream.
 * EINVAL unless max_norm is finite and > 0. */
palsgd_status palsgd_clip_grad_norm(palsgd_ctx *ctx, float max_norm, float *norms_out_dev, void *stream);

/* palsgd_clip_grad_norm for callers that cannot allocate or may not touch allocated scratch: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results (the
 * same kernels, bit for bit) and the same arming of the next gradient step; the partial sums go through a
 * fixed array that is part of the library's code object (16.1 MiB on every GPU the library runs on, held
 * until the process ends) instead of the context's reduction scratch, and the call allocates and frees
 * nothing, on the host or on the device.  palsgd_init looks the array's device address up once per device.
 * Limit: K * ceil(P_padded / 4096) <= 2^22 partial sums (K * P_padded up to 1.7e10 elements); EINVAL with
 * the two numbers in the error text beyond that, before any launch.
 * All contexts on one GPU share the array and it keeps the last call's contents (none of which a later call
 * reads before writing): two calls that overlap in time on one GPU, from different streams or contexts,
 * race on it and may both return wrong norms.  The scales themselves land in the context's own memory. */
palsgd_status palsgd_clip_grad_norm_noalloc(palsgd_ctx *ctx, float max_norm, float *norms_out_dev, void *stream);

/* Clipping in the DDP phase, where the optimizer sees the averaged gradient (Sec. 3.1):
 * norm = |(1/K) sum_k grad_scale[k] G[k]|_2 and scale = min(1, max_norm / (norm + 1e-6))
 * stay on the device; the next palsgd_ddp_step multiplies the averaged gradient by scale
 * and forgets it.  Pass the same grad_scale (host, K floats, or NULL) to both calls.
 * norm_out_dev: device float that receives the norm, or NULL.  Shares the reduction
 * scratch and the one-stream rule of palsgd_clip_grad_norm. */
palsgd_status palsgd_clip_mean_grad_norm(palsgd_ctx *ctx, float max_norm, const float *grad_scale,
                                         float *norm_out_dev, void *stream);

/* Diagnostics of the paper's analysis (App. A.3): out_dev[0] = consensus distance
 * Xi = (1/K) sum_k |x_k - XG|^2 (zero right after an outer step), out_dev[1] = |Delta|^2
 * with Delta = XG - (1/K) sum_k x_k, the outer gradient of Sec. 4.2.  out_dev: device
 * array of 2 floats.  Nothing else is modified.  Sums are formed in a fixed order. */
palsgd_status palsgd_diagnostics(palsgd_ctx *ctx, float *out_dev, void *stream);

/* Device-resident schedule, for callers that capture their training step in a HIP graph
 * (a captured launch keeps its arguments, so nothing that changes per step may be one).
 * Between palsgd_capturable_begin and palsgd_capturable_end the step index t, the branch
 * draws b_k^(t) (same hash as palsgd_draw), each worker's InnerOPT step count and AdamW
 * bias corrections live in library-owned device memory and are advanced on the device.
 *
 * palsgd_capturable_begin: uploads t0 (index of the next step) and the current step counts
 *   (one small launch on `stream`).  ESTATE if the schedule is already device-resident.
 * palsgd_step_capturable: step t of Alg. 1 for all K workers, as palsgd_step with
 *   grad_scale == NULL and no mask override, then t <- t+1, in two launches.  alpha_eta_dev:
 *   device array {alpha_t, eta_t}, read when the step runs (the caller may update it between
 *   replays: learning-rate schedules).  Clipping scales armed at the time of the call are
 *   applied.  Safe to capture; palsgd_outer_step, palsgd_outer_step_diag,
 *   palsgd_clip_grad_norm and palsgd_diagnostics are capturable as they are, with no call
 *   needed before the capture.  The host-side count of outer steps (palsgd_get_state) advances
 *   when palsgd_outer_step is called, not when a graph that holds it is replayed: a caller that
 *   replays outer steps keeps that count itself.
 * palsgd_capturable_end: waits for `stream`, reads t and the step counts back (t_out may be
 *   NULL) and returns the context to host-driven calls.
 * While the schedule is device-resident, palsgd_inner_step, palsgd_pseudo_sync, palsgd_step,
 * palsgd_step_sync, palsgd_ddp_step, palsgd_ddp_step_shared, palsgd_get_state and
 * palsgd_set_state return ESTATE. */
palsgd_status palsgd_capturable_begin(palsgd_ctx *ctx, uint64_t t0, void *stream);
palsgd_status palsgd_step_capturable(palsgd_ctx *ctx, const float *alpha_eta_dev, void *stream);
palsgd_status palsgd_capturable_end(palsgd_ctx *ctx, uint64_t *t_out, void *stream);

/* Host-side scalar state for checkpoint / resume: tau[k] = gradient steps worker k
 * has taken (drives AdamW's bias correction), n_outer = outer steps taken.  Together with
 * the caller's buffers this is the whole state of a run.  After DDP warm-up steps the
 * buffers are not yet complete (rows 1..K-1 of M, V, and after palsgd_ddp_step_shared the
 * rows of X, are filled by the broadcast that ends the warm-up): palsgd_get_state returns
 * ESTATE until palsgd_ddp_finish or the first PALSGD call has run that broadcast, so call
 * palsgd_ddp_finish before saving a checkpoint in the warm-up phase. */
palsgd_status palsgd_get_state(const palsgd_ctx *ctx, uint64_t *tau, uint64_t *n_outer);
palsgd_status palsgd_set_state(palsgd_ctx *ctx, const uint64_t *tau, uint64_t n_outer);

/* Text of the last error recorded in ctx ("" if none).  With ctx == NULL: the text of
 * the last error of a call that had no context (palsgd_layout, palsgd_init). */
const char *palsgd_last_error(const palsgd_ctx *ctx);

/* Frees the context and the library's device table (waits for nothing: the caller
 * must have synchronised work that still uses the table).  NULL is accepted. */
void palsgd_destroy(palsgd_ctx *ctx);

/* OuterOPT learning rate for the outer steps that follow (App. B: the ImageNet runs schedule
 * the outer learning rate, warm-up then cosine decay), replacing the value given at
 * palsgd_init.  Host state only: a launch that was captured into a HIP graph keeps the
 * value it was captured with.  EINVAL unless finite and >= 0. */
palsgd_status palsgd_set_outer_lr(palsgd_ctx *ctx, float outer_lr);

/* Launch-shape knobs for tuning and tests.  The kernels are throttled to a number of
 * resident wavefronts per compute unit (fewer than the hardware allows streams better);
 * step_waves_per_cu / outer_waves_per_cu override the built-in choice (0 = built-in,
 * else 3..32; 32 = no throttle).  outer_variant: 0 = default choice (3 for K >= 24 with rows
 * of at most 192 MiB, else 1), 1 = per-lane walk over k in one launch, 2 = replicas split over the
 * workgroup's wavefronts with partial sums staged through LDS, 3 = the walk without the K
 * row stores, followed by a second launch that restarts the workers' rows from the new
 * global model (also used by palsgd_step_sync).  Results do not depend on the wave caps;
 * variants 1 and 3 are bit-identical, variant 2 differs in the order of the K-sum only.
 * EINVAL on other values. */
palsgd_status palsgd_set_tuning(palsgd_ctx *ctx, uint32_t step_waves_per_cu, uint32_t outer_waves_per_cu,
                                uint32_t outer_variant);

#ifdef __cplusplus
}
#endif
#endif /* PALSGD_H */
