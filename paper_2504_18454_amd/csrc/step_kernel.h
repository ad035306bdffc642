// Local update of Alg. 1 for all K workers in one launch: InnerOPT arithmetic (AdamW, SGD with
// momentum) and the pseudo-synchronization step, one wavefront per (tile of a row, worker).
#pragma once

#include "device_common.h"

namespace palsgd_dev {

// AdamW on four elements (Loshchilov & Hutter Alg. 2; Sec. 4.3 of the paper names it as
// InnerOPT).  c1 = lr/(1-b1^tau), c2 = 1/sqrt(1-b2^tau), decay = lr*wd.
__device__ __forceinline__ void adamw4(f4& x, f4& m, f4& v, f4 g, const Hyper& h, float c1, float c2,
                                       float decay) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float mi = fmaf(h.beta1, m[i], (1.0f - h.beta1) * g[i]);
        float vi = fmaf(h.beta2, v[i], (1.0f - h.beta2) * g[i] * g[i]);
        float denom = fmaf(sqrtf(vi), c2, h.eps);
        // the whole step first (small, so its rounding is far below an ulp of x), then ONE rounding of x
        x[i] = x[i] - fmaf(c1, mi / denom, decay * x[i]);
        m[i] = mi;
        v[i] = vi;
    }
}

// SGD with momentum on four elements: d = g + wd x; buf = mu buf + d; x -= lr buf, or in the
// Nesterov form x -= lr (d + mu buf).
__device__ __forceinline__ void sgdm4(f4& x, f4& b, f4 g, const Hyper& h, float lr, float wd) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float d = fmaf(wd, x[i], g[i]);
        float bi = fmaf(h.momentum, b[i], d);
        float dir = h.nesterov ? fmaf(h.momentum, bi, d) : bi;
        x[i] = fmaf(-lr, dir, x[i]);
        b[i] = bi;
    }
}

// Local update of step t.  Grid: x = tile of the row, y = slot.  A gradient-step wavefront
// takes one tile (256 elements: 6.5-7 KiB of traffic); a mixing wavefront takes two (6 KiB),
// so that both kinds keep about the same number of bytes in flight.
// TAB: weight decay comes from a table with one entry per 64 elements of a row.
// DEV: the per-slot scalars come from device memory (dev_slots, written by plan_kernel for
// this step) instead of the kernel arguments.  A compile-time switch: selecting the source
// at run time turns the scalar loads and the uniform branch into vector ones (-10 %).
template <int INNER, int GDT, bool TAB, bool DEV>
__global__ __launch_bounds__(kWave) void step_kernel(const StepArgs args, const Slot* __restrict__ dev_slots,
                                                     const float* __restrict__ wd_tab, float* __restrict__ X, float* __restrict__ M,
                                                     float* __restrict__ V, const void* __restrict__ G,
                                                     const float* __restrict__ XG,
                                                     const float* __restrict__ clip_scale, uint64_t n,
                                                     uint64_t row_stride, Hyper h) {
    const Slot sl = DEV ? dev_slots[blockIdx.y] : args.s[blockIdx.y];
    const uint64_t row = (uint64_t)sl.replica * row_stride;
    const uint32_t lane4 = threadIdx.x * 4;

    if (sl.mix) {
        // pseudo-synchronization step: x_k <- x_k - beta (x_k - x)     (Sec. 4.1, second equation)
        const uint64_t e0 = (uint64_t)blockIdx.x * (2 * kTile) + lane4;
        if (e0 >= n) return;
        const uint64_t e1 = e0 + kTile;
        const bool two = e1 < n;
        float* __restrict__ x = X + row;
        f4 x0 = ld4(x + e0), g0 = ld4_cached(XG + e0), x1, g1;
        if (two) {
            x1 = ld4(x + e1);
            g1 = ld4_cached(XG + e1);
        }
        st4(x + e0, x0 - sl.beta_mix * (x0 - g0));
        if (two) st4(x + e1, x1 - sl.beta_mix * (x1 - g1));
        return;
    }

    // gradient step: x_k <- InnerOPT(x_k, g_k, alpha/(1-p))             (Sec. 4.1, first equation)
    const uint64_t e = (uint64_t)blockIdx.x * kTile + lane4;
    if (e >= n) return;
    const uint64_t o = row + e;
    typedef GradLoad<GDT> GL;
    typename GL::raw gr = GL::load(G, o);
    f4 xv = ld4(X + o), mv = ld4(M + o);
    const float wd = TAB ? wd_tab[e >> 6] : h.wd;
    // per-replica gradient multiplier: the caller's, times the clipping scale left on the device
    const float gs = clip_scale ? sl.gscale * clip_scale[sl.replica] : sl.gscale;
    if (INNER == PALSGD_INNER_ADAMW) {
        f4 vv = ld4(V + o);
        f4 g = GL::widen(gr) * gs;
        adamw4(xv, mv, vv, g, h, sl.c1, sl.c2, sl.lr * wd);
        st4(X + o, xv);
        st4(M + o, mv);
        st4(V + o, vv);
    } else {
        f4 g = GL::widen(gr) * gs;
        sgdm4(xv, mv, g, h, sl.lr, wd);
        st4(X + o, xv);
        st4(M + o, mv);
    }
}

}  // namespace palsgd_dev
