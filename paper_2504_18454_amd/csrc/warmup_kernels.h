// DDP step of the warm-up phase and the broadcast that ends it.
#pragma once

#include "device_common.h"
#include "step_kernel.h"

namespace palsgd_dev {

// ---------------------------------------------------------------------------------------
// DDP step of the warm-up phase (Sec. 3.1: All-Reduce of the gradient, then the optimizer
// update, identical on every worker; Sec. 4.3).  One wavefront per tile: weighted mean of the
// K gradient rows (k ascending, eight loads in flight), InnerOPT on the common model (read
// from XG) with the common state (replica 0's), model stored to XG and to the first x_rows
// rows of X (K, or 0 when the rows are left to the end of the warm-up), state to replica 0
// only: the other replicas' copies are made once, when the warm-up ends.
struct DdpArgs {
    float w[PALSGD_MAX_K];  // grad_scale[k]
    float inv_k, lr, c1, c2;
};

template <int INNER, int GDT, bool TAB>
__global__ __launch_bounds__(kWave) void ddp_kernel(const DdpArgs a, const float* __restrict__ wd_tab,
                                                    float* __restrict__ X, float* __restrict__ M,
                                                    float* __restrict__ V, const void* __restrict__ G,
                                                    float* __restrict__ XG,
                                                    const float* __restrict__ clip_scale, uint64_t n,
                                                    uint64_t row_stride, uint32_t K, uint32_t x_rows, Hyper h) {
    const uint64_t e = (uint64_t)blockIdx.x * kTile + threadIdx.x * 4;
    if (e >= n) return;
    typedef GradLoad<GDT> GL;
    f4 xv = ld4(XG + e), mv = ld4(M + e), vv;
    if (INNER == PALSGD_INNER_ADAMW) vv = ld4(V + e);
    f4 sum = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t k0 = 0; k0 < K; k0 += 8) {
        typename GL::raw t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < K) t[u] = GL::load(G, (uint64_t)(k0 + u) * row_stride + e);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < K) sum += GL::widen(t[u]) * a.w[k0 + u];
    }
    // averaged gradient, times the clipping scale of its norm if one was left on the device
    const f4 g = sum * (clip_scale ? a.inv_k * clip_scale[0] : a.inv_k);
    const float wd = TAB ? wd_tab[e >> 6] : h.wd;
    if (INNER == PALSGD_INNER_ADAMW)
        adamw4(xv, mv, vv, g, h, a.c1, a.c2, a.lr * wd);
    else
        sgdm4(xv, mv, g, h, a.lr, wd);
    st4(XG + e, xv);
    st4(M + e, mv);  // the common InnerOPT state lives in replica 0 during the warm-up
    if (INNER == PALSGD_INNER_ADAMW) st4(V + e, vv);
    for (uint32_t k = 0; k < x_rows; ++k) st4(X + (uint64_t)k * row_stride + e, xv);
}

// End of the warm-up: replicas 1..K-1 take over the common InnerOPT state of replica 0
// (M, and V unless NULL), and all K rows of X take the common model from XG (unless X is
// NULL: the DDP steps kept the rows current themselves).
__global__ __launch_bounds__(kWave) void warmup_broadcast_kernel(float* __restrict__ M, float* __restrict__ V,
                                                                 float* __restrict__ X, const float* __restrict__ XG,
                                                                 uint64_t n, uint64_t row_stride, uint32_t K) {
    const uint64_t e = (uint64_t)blockIdx.x * kTile + threadIdx.x * 4;
    if (e >= n) return;
    f4 mv, vv, xv;
    if (M) mv = ld4(M + e);
    if (V) vv = ld4(V + e);
    if (X) {
        xv = ld4(XG + e);
        st4(X + e, xv);
    }
    for (uint32_t k = 1; k < K; ++k) {
        const uint64_t o = (uint64_t)k * row_stride + e;
        if (M) st4(M + o, mv);
        if (V) st4(V + o, vv);
        if (X) st4(X + o, xv);
    }
}

}  // namespace palsgd_dev
