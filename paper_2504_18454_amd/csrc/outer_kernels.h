// Outer step of Alg. 1 (K-way mean of x - x_k, OuterOPT, restart of the workers), its fusion with the
// last local update of a window, the LDS-staged split-K variant, and the initialisation kernel.
#pragma once

#include "device_common.h"
#include "step_kernel.h"

namespace palsgd_dev {

struct OuterArgs {
    float inv_k, lr, mu;
    int nesterov;
    // OuterOPT = AdamW with Delta as its gradient, instead of the SGD family:
    float b1, b2, eps;     // its decay rates and epsilon
    float c1, c2, decay;   // for this outer step n: lr/(1-b1^n), 1/sqrt(1-b2^n), lr*wd
};

// OuterOPT on four elements given dsum = sum_k (x - x_k) (Sec. 4.2; Sec. 4.3).  Summing the
// differences instead of the models keeps Delta accurate to fp32 relative to its own size
// and makes it exactly zero when the workers equal the global model.  om is the momentum
// buffer of the SGD family or the first moment of AdamW; ov (AdamW only) the second moment.
template <bool OADAM>
__device__ __forceinline__ f4 outer4(f4 dsum, f4 xg, f4& om, f4& ov, const OuterArgs& a) {
    f4 delta = dsum * a.inv_k;                     // Delta = mean_k (x - x_k)
    if (OADAM) {
        const Hyper h{a.b1, a.b2, a.eps, 0.f, 0.f, 0};
        adamw4(xg, om, ov, delta, h, a.c1, a.c2, a.decay);
        return xg;
    }
    om = a.mu * om + delta;
    f4 dir = a.nesterov ? delta + a.mu * om : om;
    return xg - a.lr * dir;
}

// Variant 1: one wavefront per tile; each lane owns four consecutive elements and walks the
// K rows in ascending order, eight independent loads in flight at a time.
// ROWS: the wavefront also stores the new model to the K rows of X (the restart of the workers).  With
// ROWS = false that is left to restart_rows_kernel in a second launch: with many workers a wavefront that has
// to issue K stores in a row holds the chip at 5.6 TB/s, while short wavefronts that store a few rows each
// run the restart alone at the speed of a plain fill (as long as the model they re-read comes from the caches).
// DIAG: also leaves, per wavefront, the partial sums of sum_k |x - x_k|^2 and |Delta|^2
// (App. A.3) taken from the values already in registers: no extra HBM reads.
// OADAM: OuterOPT = AdamW (a compile-time switch: as a run-time one it slowed the SGD-family
// outer step by a quarter).
template <bool DIAG, bool OADAM, bool ROWS>
__global__ __launch_bounds__(kWave) void outer_kernel_walk(float* __restrict__ X, float* __restrict__ XG,
                                                           float* __restrict__ OM, float* __restrict__ OV, uint64_t n,
                                                           uint64_t row_stride, uint32_t K, OuterArgs a,
                                                           float* __restrict__ partial, uint32_t n_part) {
    const uint64_t e = (uint64_t)blockIdx.x * kTile + threadIdx.x * 4;
    const bool active = e < n;  // no early exit: every lane takes part in the shuffles
    f4 sum = {0.f, 0.f, 0.f, 0.f}, sq = {0.f, 0.f, 0.f, 0.f};
    if (active) {
        f4 xg = ld4(XG + e);
        f4 om = ld4(OM + e), ov;
        if (OADAM) ov = ld4(OV + e);
        for (uint32_t k0 = 0; k0 < K; k0 += 8) {
            f4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (k0 + u < K) t[u] = ld4(X + (uint64_t)(k0 + u) * row_stride + e);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (k0 + u < K) {
                    f4 d = xg - t[u];
                    sum += d;
                    if (DIAG) sq += d * d;
                }
        }
        f4 xn = outer4<OADAM>(sum, xg, om, ov, a);
        st4(XG + e, xn);
        st4(OM + e, om);
        if (OADAM) st4(OV + e, ov);
        if (ROWS)
            for (uint32_t k = 0; k < K; ++k) st4(X + (uint64_t)k * row_stride + e, xn);
    }
    if (DIAG) {
        const f4 delta = sum * a.inv_k;
        const f4 dd = delta * delta;
        float xi = wave_sum((sq.x + sq.y) + (sq.z + sq.w));
        float d2 = wave_sum((dd.x + dd.y) + (dd.z + dd.w));
        if (threadIdx.x == 0) {
            partial[blockIdx.x] = xi;
            partial[n_part + blockIdx.x] = d2;
        }
    }
}

// Restart of the workers as a launch of its own (Sec. 2.1: every worker continues from the new global model):
// grid x = tile, y = group of kRestartRows rows, so the chip fills one group of rows after the other and a
// wavefront lives for one load and kRestartRows stores.  The global model is re-read once per group; it was
// written by the launch before and is served by the caches while it fits them.
constexpr int kRestartRows = 8;

__global__ __launch_bounds__(kWave) void restart_rows_kernel(float* __restrict__ X, const float* __restrict__ XG,
                                                             uint64_t n, uint64_t row_stride, uint32_t K) {
    const uint64_t e = (uint64_t)blockIdx.x * kTile + threadIdx.x * 4;
    if (e >= n) return;
    const f4 v = ld4_cached(XG + e);
    const uint32_t k0 = blockIdx.y * kRestartRows;
#pragma unroll
    for (int u = 0; u < kRestartRows; ++u)
        if (k0 + u < K) st4(X + (uint64_t)(k0 + u) * row_stride + e, v);
}

// Last local update of a window fused with the outer step (Alg. 1, step t with (t+1) mod H = 0):
// a wavefront owns a tile of ALL K rows.  It takes the replicas in ascending order, four at a
// time (their loads in flight together), applies each replica's branch, stores the InnerOPT
// state, keeps the new x_k in registers only and adds x - x_k to the outer gradient; then
// OuterOPT and the restart stores.  Against the two separate launches this saves writing the
// K rows of X in the local update and reading them back in the outer step (8K of 34K+16 bytes
// per element with AdamW).  Slot s of `args` is replica s.  The arithmetic, its order and its
// roundings are those of step_kernel followed by outer_kernel_walk: results are bit-identical.
constexpr int kSyncBatch = 4;

template <int INNER, int GDT, bool TAB, bool OADAM, bool ROWS>
__global__ __launch_bounds__(kWave) void sync_step_kernel(const StepArgs args, const float* __restrict__ wd_tab,
                                                          float* __restrict__ X, float* __restrict__ M,
                                                          float* __restrict__ V, const void* __restrict__ G,
                                                          float* __restrict__ XG, float* __restrict__ OM,
                                                          float* __restrict__ OV,
                                                          const float* __restrict__ clip_scale, uint64_t n,
                                                          uint64_t row_stride, uint32_t K, Hyper h, OuterArgs a) {
    const uint64_t e = (uint64_t)blockIdx.x * kTile + threadIdx.x * 4;
    if (e >= n) return;
    typedef GradLoad<GDT> GL;
    const f4 xg = ld4(XG + e);
    f4 om = ld4(OM + e), ov;
    if (OADAM) ov = ld4(OV + e);
    const float wd = TAB ? wd_tab[e >> 6] : h.wd;
    f4 dsum = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t k0 = 0; k0 < K; k0 += kSyncBatch) {
        typename GL::raw gr[kSyncBatch];
        f4 xv[kSyncBatch], mv[kSyncBatch], vv[kSyncBatch];
#pragma unroll
        for (int u = 0; u < kSyncBatch; ++u) {
            if (k0 + u < K) {
                const uint64_t o = (uint64_t)(k0 + u) * row_stride + e;
                xv[u] = ld4(X + o);
                if (!args.s[k0 + u].mix) {
                    gr[u] = GL::load(G, o);
                    mv[u] = ld4(M + o);
                    if (INNER == PALSGD_INNER_ADAMW) vv[u] = ld4(V + o);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kSyncBatch; ++u) {
            if (k0 + u < K) {
                const Slot sl = args.s[k0 + u];
                const uint64_t o = (uint64_t)(k0 + u) * row_stride + e;
                if (sl.mix) {
                    xv[u] = xv[u] - sl.beta_mix * (xv[u] - xg);
                } else {
                    const float gs = clip_scale ? sl.gscale * clip_scale[sl.replica] : sl.gscale;
                    const f4 g = GL::widen(gr[u]) * gs;
                    if (INNER == PALSGD_INNER_ADAMW) {
                        adamw4(xv[u], mv[u], vv[u], g, h, sl.c1, sl.c2, sl.lr * wd);
                        st4(V + o, vv[u]);
                    } else {
                        sgdm4(xv[u], mv[u], g, h, sl.lr, wd);
                    }
                    st4(M + o, mv[u]);
                }
                dsum += xg - xv[u];
            }
        }
    }
    const f4 xn = outer4<OADAM>(dsum, xg, om, ov, a);
    st4(XG + e, xn);
    st4(OM + e, om);
    if (OADAM) st4(OV + e, ov);
    if (ROWS)  // else restart_rows_kernel follows
        for (uint32_t k = 0; k < K; ++k) st4(X + (uint64_t)k * row_stride + e, xn);
}

// Variant 2: a workgroup owns a tile of 4 x 256 elements.  Wave w sums the replicas
// k = w, w+4, ... for the whole tile, the four partial sums per element meet in LDS,
// and wave w finishes sub-tile w: fixed-order combine, OuterOPT, stores.  Puts 4*ceil(K/4)
// row loads in flight per lane before the first add.
template <bool OADAM>
__global__ __launch_bounds__(kThreads) void outer_kernel_lds(float* __restrict__ X, float* __restrict__ XG,
                                                             float* __restrict__ OM, float* __restrict__ OV, uint64_t n4,
                                                             uint64_t row_stride, uint32_t K, OuterArgs a) {
    __shared__ f4 part[4][4][64];  // [wave][sub-tile][lane], 16 KiB
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint64_t tile4 = (uint64_t)blockIdx.x * 256;  // first float4 of the tile
    f4 acc[4], xgt[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        acc[s] = (f4){0.f, 0.f, 0.f, 0.f};
        uint64_t i = tile4 + s * 64 + lane;
        xgt[s] = i < n4 ? ld4_cached(XG + i * 4) : (f4){0.f, 0.f, 0.f, 0.f};
    }
    for (uint32_t k = w; k < K; k += 4) {
        const float* row = X + (uint64_t)k * row_stride;
        f4 t[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint64_t i = tile4 + s * 64 + lane;
            t[s] = i < n4 ? ld4(row + i * 4) : (f4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[s] += xgt[s] - t[s];
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) part[w][s][lane] = acc[s];
    __syncthreads();
    const uint64_t i = tile4 + w * 64 + lane;
    if (i < n4) {
        const uint64_t e = i * 4;
        f4 sum = ((part[0][w][lane] + part[1][w][lane]) + part[2][w][lane]) + part[3][w][lane];
        f4 xg = w == 0 ? xgt[0] : (w == 1 ? xgt[1] : (w == 2 ? xgt[2] : xgt[3]));
        f4 om = ld4(OM + e), ov;
        if (OADAM) ov = ld4(OV + e);
        f4 xn = outer4<OADAM>(sum, xg, om, ov, a);
        st4(XG + e, xn);
        st4(OM + e, om);
        if (OADAM) st4(OV + e, ov);
        for (uint32_t k = 0; k < K; ++k) st4(X + (uint64_t)k * row_stride + e, xn);
    }
}

// x_k^(0) <- x^(0) for all k, XG <- x^(0), cleared moments (Alg. 1, first line of the worker loop).
__global__ __launch_bounds__(kThreads) void init_kernel(const float* __restrict__ x0, float* __restrict__ X,
                                                        float* __restrict__ M, float* __restrict__ V,
                                                        float* __restrict__ XG, float* __restrict__ OM,
                                                        float* __restrict__ OV, uint64_t n4, uint64_t row_stride,
                                                        uint32_t K) {
    uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n4) return;
    uint64_t e = i * 4;
    f4 v = *(const f4*)(x0 + e);
    f4 z = {0.f, 0.f, 0.f, 0.f};
    st4(XG + e, v);
    st4(OM + e, z);
    if (OV) st4(OV + e, z);
    for (uint32_t k = 0; k < K; ++k) {
        uint64_t r = (uint64_t)k * row_stride + e;
        st4(X + r, v);
        st4(M + r, z);
        if (V) st4(V + r, z);
    }
}

}  // namespace palsgd_dev
