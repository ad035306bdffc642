// Branch draws (counter hash) and the device-resident schedule of the graph-capturable mode.
#pragma once

#include "device_common.h"

namespace palsgd_dev {

// ---------------------------------------------------------------------------------------
// Device-resident schedule, for callers that capture their training step in a HIP graph: a
// captured launch keeps its arguments, so everything that changes from step to step (the
// step index t, the branch draws, each worker's InnerOPT step count and bias corrections,
// alpha_t and eta_t) lives in device memory and is advanced by plan_kernel, one lane per
// worker, right before each local update.
struct DevSchedule {
    uint64_t t;                  // index of the next step
    uint64_t tau[PALSGD_MAX_K];  // gradient steps taken per worker
    Slot slot[PALSGD_MAX_K];     // scalars of the step about to run
};

struct PlanArgs {
    uint64_t seed;
    double p, beta1, beta2;
    uint32_t K, threshold, adamw;
};

// SplitMix64 output function as a counter hash (Steele, Lea, Flood 2014), top 24 bits.
__host__ __device__ inline uint32_t draw_u24(uint64_t seed, uint64_t t, uint32_t k, uint32_t K) {
    uint64_t z = seed + (t * (uint64_t)K + k + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z >> 40);
}

__global__ __launch_bounds__(kWave) void plan_kernel(DevSchedule* __restrict__ s, const float* __restrict__ alpha_eta,
                                                     PlanArgs a) {
    const uint32_t k = threadIdx.x;
    const uint64_t t = s->t;
    const double alpha = (double)alpha_eta[0], eta = (double)alpha_eta[1];
    if (k < a.K) {
        Slot sl;
        sl.replica = k;
        sl.gscale = 1.0f;
        sl.lr = sl.c1 = sl.c2 = sl.beta_mix = 0.0f;
        sl.mix = draw_u24(a.seed, t, k, a.K) < a.threshold ? 1u : 0u;
        if (sl.mix) {
            sl.beta_mix = (float)(alpha * eta / a.p);        // a.p > 0 whenever a draw can fire
        } else {
            const uint64_t tau = s->tau[k] + 1;
            s->tau[k] = tau;
            const double lr = alpha / (1.0 - a.p);
            sl.lr = (float)lr;
            if (a.adamw) {
                sl.c1 = (float)(lr / (1.0 - pow(a.beta1, (double)tau)));
                sl.c2 = (float)(1.0 / sqrt(1.0 - pow(a.beta2, (double)tau)));
            }
        }
        s->slot[k] = sl;
    }
    __syncthreads();  // every lane has read t
    if (k == 0) s->t = t + 1;
}

struct TauArgs {
    uint64_t tau[PALSGD_MAX_K];
};

__global__ void schedule_set_kernel(DevSchedule* __restrict__ s, uint64_t t0, TauArgs a) {
    const uint32_t k = threadIdx.x;
    if (k < PALSGD_MAX_K) s->tau[k] = a.tau[k];
    if (k == 0) s->t = t0;
}

}  // namespace palsgd_dev
