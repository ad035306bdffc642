// Reductions to scalars: gradient norms for clipping, consensus-distance diagnostics.
#pragma once

#include "device_common.h"
#include "warmup_kernels.h"

namespace palsgd_dev {

// ---------------------------------------------------------------------------------------
// Reductions to scalars: lane-local accumulation, a shuffle tree inside the wavefront, one
// partial per wavefront in device scratch, and a second single-workgroup pass that adds the
// partials in double in a fixed order (deterministic run to run).
constexpr int kNormTiles = 16;  // tiles a wavefront of the norm kernel walks: one partial per 4096 elements
constexpr int kDiagTiles = 8;   // same for the diagnostics kernel: one partial pair per 2048 elements

// Sum of squares of one replica's gradient row, per wavefront (App. B: gradient clipping).
template <int GDT>
__global__ __launch_bounds__(kWave) void sumsq_kernel(const void* __restrict__ G, float* __restrict__ partial,
                                                      uint64_t n, uint64_t row_stride, uint32_t per_row) {
    typedef GradLoad<GDT> GL;
    const uint64_t base = (uint64_t)blockIdx.x * (kTile * kNormTiles) + threadIdx.x * 4;
    const uint64_t row = (uint64_t)blockIdx.y * row_stride;
    float acc = 0.f;
    typename GL::raw r[kNormTiles];  // all loads of the wavefront are issued before the first use
#pragma unroll
    for (int u = 0; u < kNormTiles; ++u) {
        const uint64_t e = base + (uint64_t)u * kTile;
        if (e < n) r[u] = GL::load(G, row + e);
    }
#pragma unroll
    for (int u = 0; u < kNormTiles; ++u) {
        const uint64_t e = base + (uint64_t)u * kTile;
        if (e < n) {
            f4 g = GL::widen(r[u]);
            acc += (g.x * g.x + g.y * g.y) + (g.z * g.z + g.w * g.w);
        }
    }
    acc = wave_sum(acc);
    if (threadIdx.x == 0) partial[(uint64_t)blockIdx.y * per_row + blockIdx.x] = acc;
}

// Sum of squares of the averaged gradient (1/K) sum_k w_k g_k, per wavefront of two tiles
// (clipping in the DDP phase, where the optimizer sees the averaged gradient, Sec. 3.1).
constexpr int kMeanTiles = 2;
template <int GDT>
__global__ __launch_bounds__(kWave) void sumsq_mean_kernel(const void* __restrict__ G, const DdpArgs a,
                                                           float* __restrict__ partial, uint64_t n,
                                                           uint64_t row_stride, uint32_t K) {
    typedef GradLoad<GDT> GL;
    const uint64_t base = (uint64_t)blockIdx.x * (kTile * kMeanTiles) + threadIdx.x * 4;
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kMeanTiles; ++u) {
        const uint64_t e = base + (uint64_t)u * kTile;
        if (e < n) {
            f4 sum = {0.f, 0.f, 0.f, 0.f};
            for (uint32_t k0 = 0; k0 < K; k0 += 8) {
                typename GL::raw t[8];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (k0 + q < K) t[q] = GL::load(G, (uint64_t)(k0 + q) * row_stride + e);
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (k0 + q < K) sum += GL::widen(t[q]) * a.w[k0 + q];
            }
            const f4 g = sum * a.inv_k;
            acc += (g.x * g.x + g.y * g.y) + (g.z * g.z + g.w * g.w);
        }
    }
    acc = wave_sum(acc);
    if (threadIdx.x == 0) partial[blockIdx.x] = acc;
}

// Fixed-order sum of `count` values in double by one workgroup; every thread returns the total.
template <typename T>
__device__ double block_sum(const T* __restrict__ v, uint32_t count, double* lds) {
    double acc = 0.0;
    for (uint32_t j = threadIdx.x; j < count; j += 4 * kThreads) {  // four independent loads in flight
        T t[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = j + q * kThreads < count ? v[j + q * kThreads] : (T)0;
#pragma unroll
        for (int q = 0; q < 4; ++q) acc += (double)t[q];
    }
    lds[threadIdx.x] = acc;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) lds[threadIdx.x] += lds[threadIdx.x + s];
        __syncthreads();
    }
    double total = lds[0];
    __syncthreads();
    return total;
}

constexpr uint32_t kFold = 128;  // second-stage workgroups per series of partial sums

// Second stage: series y has `count` float partials; workgroup x adds its contiguous slice in double.
__global__ __launch_bounds__(kThreads) void fold_kernel(const float* __restrict__ partial, uint32_t count,
                                                        double* __restrict__ fold) {
    __shared__ double lds[kThreads];
    const uint32_t slice = (count + kFold - 1) / kFold;
    const uint32_t begin = blockIdx.x * slice;
    const uint32_t len = begin >= count ? 0u : (count - begin < slice ? count - begin : slice);
    double total = block_sum(partial + (uint64_t)blockIdx.y * count + begin, len, lds);
    if (threadIdx.x == 0) fold[blockIdx.y * kFold + blockIdx.x] = total;
}

// norm_k = sqrt(sum of squares); scale_k = min(1, max_norm / (norm_k + 1e-6)).  One workgroup per replica.
__global__ __launch_bounds__(kThreads) void clip_finish_kernel(const double* __restrict__ fold, float max_norm,
                                                               float* __restrict__ scale,
                                                               float* __restrict__ norms_out) {
    __shared__ double lds[kThreads];
    const uint32_t k = blockIdx.x;
    double total = block_sum(fold + k * kFold, kFold, lds);
    if (threadIdx.x == 0) {
        double norm = sqrt(total);
        double c = (double)max_norm / (norm + 1e-6);
        scale[k] = (float)(c < 1.0 ? c : 1.0);
        if (norms_out) norms_out[k] = (float)norm;
    }
}

// Consensus distance and outer-gradient norm (App. A.3): per wavefront, partial sums of
// sum_k |x_k - x|^2 and of |x - mean_k x_k|^2.
__global__ __launch_bounds__(kWave) void diag_kernel(const float* __restrict__ X, const float* __restrict__ XG,
                                                     float* __restrict__ partial, uint64_t n, uint64_t row_stride,
                                                     uint32_t K, float inv_k, uint32_t n_part) {
    const uint64_t base = (uint64_t)blockIdx.x * (kTile * kDiagTiles) + threadIdx.x * 4;
    float xi = 0.f, d2 = 0.f;
    for (int u = 0; u < kDiagTiles; ++u) {
        const uint64_t e = base + (uint64_t)u * kTile;
        if (e >= n) break;
        const f4 xg = ld4(XG + e);
        f4 sum = {0.f, 0.f, 0.f, 0.f}, sq = {0.f, 0.f, 0.f, 0.f};
        for (uint32_t k0 = 0; k0 < K; k0 += 8) {
            f4 t[8];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (k0 + q < K) t[q] = ld4(X + (uint64_t)(k0 + q) * row_stride + e);
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (k0 + q < K) {
                    f4 d = xg - t[q];
                    sq += d * d;
                    sum += d;
                }
        }
        const f4 delta = sum * inv_k;
        const f4 dd = delta * delta;
        xi += (sq.x + sq.y) + (sq.z + sq.w);
        d2 += (dd.x + dd.y) + (dd.z + dd.w);
    }
    xi = wave_sum(xi);
    d2 = wave_sum(d2);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = xi;
        partial[n_part + blockIdx.x] = d2;
    }
}

__global__ __launch_bounds__(kThreads) void diag_finish_kernel(const double* __restrict__ fold, float inv_k,
                                                               float* __restrict__ out) {
    __shared__ double lds[kThreads];
    double xi = block_sum(fold, kFold, lds);
    double d2 = block_sum(fold + kFold, kFold, lds);
    if (threadIdx.x == 0) {
        out[0] = (float)(xi * (double)inv_k);
        out[1] = (float)d2;
    }
}

}  // namespace palsgd_dev
