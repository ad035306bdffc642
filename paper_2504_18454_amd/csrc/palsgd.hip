// PALSGD parameter-update path for MI355X (gfx950, CDNA4): HIP kernels and the C ABI
// declared in include/palsgd.h.
//
// Three kernels, all bound by HBM bandwidth (about one flop per byte moved, far below
// the vector-ALU ridge), so the design rules are: every access a full-width coalesced
// vector load/store (each wavefront instruction touches one contiguous 1 KiB / 512 B
// span), every byte of state read once and written once per step, many independent
// loads in flight per lane, one launch per step whatever the number of tensors.
//
//   step_kernel   Alg. 1 local update of all K workers in one launch: a workgroup
//                 owns (chunk, worker); the worker's branch (gradient step / mixing
//                 step) is uniform over the workgroup, so there is no divergence.
//   outer_kernel  Alg. 1 outer step: K-way mean over the replica rows, Delta,
//                 OuterOPT with (Nesterov) momentum, restart of the K workers.
//   init_kernel   x_k^(0) <- x^(0), cleared optimizer state.
//
// No matrix cores: nothing here is a contraction.  No LDS in the step kernel: there is
// no reuse to stage.  Each XCD's private L2 is irrelevant to pure streaming, so the
// blockIdx -> (chunk, worker) map is a plain row-major one.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/palsgd.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;          // 4 wavefronts of 64 lanes
constexpr int kGroup = kThreads * 4;   // elements one workgroup instruction covers
constexpr uint32_t kDefaultChunk = 8192;
constexpr uint32_t kMaxChunk = 65536;

// One entry per contiguous range of a row that shares a weight-decay multiplier.
struct Chunk {
    uint64_t off;   // first element (multiple of 64)
    uint32_t len;   // elements (multiple of 64, <= chunk size)
    float wd;       // weight_decay * multiplier of the tensors inside
};

// Per-launch, per-slot scalars; slot s of the grid's y dimension works on row `replica`.
struct Slot {
    float lr;        // alpha_t / (1-p), the learning rate handed to InnerOPT
    float c1;        // AdamW: lr / (1 - beta1^tau)
    float c2;        // AdamW: 1 / sqrt(1 - beta2^tau)
    float beta_mix;  // alpha_t * eta_t / p
    float gscale;    // multiplier on the gradient
    uint32_t replica;
    uint32_t mix;    // 1: pseudo-synchronization step, 0: gradient step
};
struct StepArgs {
    Slot s[PALSGD_MAX_K];
};

struct Hyper {
    float beta1, beta2, eps, momentum;
};

__device__ __forceinline__ f4 ld4(const float* p) { return __builtin_nontemporal_load((const f4*)p); }
__device__ __forceinline__ void st4(float* p, f4 v) { __builtin_nontemporal_store(v, (f4*)p); }
// read that other workgroups will want again soon (the global model during mixing)
__device__ __forceinline__ f4 ld4_cached(const float* p) { return *(const f4*)p; }

template <int GDT>
struct GradLoad;
template <>
struct GradLoad<PALSGD_GRAD_F32> {
    typedef f4 raw;
    static __device__ __forceinline__ raw load(const void* g, uint64_t e) {
        return __builtin_nontemporal_load((const f4*)((const float*)g + e));
    }
    static __device__ __forceinline__ f4 widen(raw r) { return r; }
};
template <>
struct GradLoad<PALSGD_GRAD_BF16> {
    typedef u2 raw;  // four bf16 values
    static __device__ __forceinline__ raw load(const void* g, uint64_t e) {
        return __builtin_nontemporal_load((const u2*)((const uint16_t*)g + e));
    }
    // bf16 is the upper half of an fp32: widening is a shift, exact
    static __device__ __forceinline__ f4 widen(raw r) {
        f4 o;
        o.x = __uint_as_float(r.x << 16);
        o.y = __uint_as_float(r.x & 0xFFFF0000u);
        o.z = __uint_as_float(r.y << 16);
        o.w = __uint_as_float(r.y & 0xFFFF0000u);
        return o;
    }
};

// AdamW on four elements (Loshchilov & Hutter Alg. 2; Sec. 4.3 of the paper names it as
// InnerOPT).  c1 = lr/(1-b1^tau), c2 = 1/sqrt(1-b2^tau), decay = lr*wd.
__device__ __forceinline__ void adamw4(f4& x, f4& m, f4& v, f4 g, const Hyper& h, float c1, float c2,
                                       float decay) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float mi = fmaf(h.beta1, m[i], (1.0f - h.beta1) * g[i]);
        float vi = fmaf(h.beta2, v[i], (1.0f - h.beta2) * g[i] * g[i]);
        float denom = fmaf(sqrtf(vi), c2, h.eps);
        x[i] = fmaf(-c1, mi / denom, fmaf(-decay, x[i], x[i]));
        m[i] = mi;
        v[i] = vi;
    }
}

// SGD with momentum on four elements: d = g + wd x; buf = mu buf + d; x -= lr buf.
__device__ __forceinline__ void sgdm4(f4& x, f4& b, f4 g, float mu, float lr, float wd) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float d = fmaf(wd, x[i], g[i]);
        float bi = fmaf(mu, b[i], d);
        x[i] = fmaf(-lr, bi, x[i]);
        b[i] = bi;
    }
}

// Local update of step t for every (chunk, slot).  U = independent 4-element groups a
// lane keeps in flight per loop trip.
template <int INNER, int GDT, int U>
__global__ __launch_bounds__(kThreads) void step_kernel(const StepArgs args, const Chunk* __restrict__ chunks,
                                                        float* __restrict__ X, float* __restrict__ M,
                                                        float* __restrict__ V, const void* __restrict__ G,
                                                        const float* __restrict__ XG, uint64_t row_stride,
                                                        Hyper h) {
    const Slot sl = args.s[blockIdx.y];
    const Chunk ch = chunks[blockIdx.x];
    const uint64_t row = (uint64_t)sl.replica * row_stride;
    const uint32_t len = ch.len;
    float* __restrict__ x = X + row + ch.off;
    const uint32_t lane0 = threadIdx.x * 4;

    if (sl.mix) {
        // pseudo-synchronization step: x_k <- x_k - beta (x_k - x)     (Sec. 4.1, second equation)
        const float* __restrict__ xg = XG + ch.off;
        const float beta = sl.beta_mix;
        for (uint32_t base = 0; base < len; base += kGroup * U) {
            f4 xv[U], gv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    xv[u] = ld4(x + e);
                    gv[u] = ld4_cached(xg + e);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    f4 r = xv[u] - beta * (xv[u] - gv[u]);
                    st4(x + e, r);
                }
            }
        }
        return;
    }

    // gradient step: x_k <- InnerOPT(x_k, g_k, alpha/(1-p))             (Sec. 4.1, first equation)
    float* __restrict__ m = M + row + ch.off;
    const uint64_t gbase = row + ch.off;
    typedef GradLoad<GDT> GL;
    if (INNER == PALSGD_INNER_ADAMW) {
        float* __restrict__ v = V + row + ch.off;
        const float decay = sl.lr * ch.wd;
        for (uint32_t base = 0; base < len; base += kGroup * U) {
            f4 xv[U], mv[U], vv[U];
            typename GL::raw gr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    gr[u] = GL::load(G, gbase + e);
                    xv[u] = ld4(x + e);
                    mv[u] = ld4(m + e);
                    vv[u] = ld4(v + e);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    f4 g = GL::widen(gr[u]) * sl.gscale;
                    adamw4(xv[u], mv[u], vv[u], g, h, sl.c1, sl.c2, decay);
                    st4(x + e, xv[u]);
                    st4(m + e, mv[u]);
                    st4(v + e, vv[u]);
                }
            }
        }
    } else {
        for (uint32_t base = 0; base < len; base += kGroup * U) {
            f4 xv[U], mv[U];
            typename GL::raw gr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    gr[u] = GL::load(G, gbase + e);
                    xv[u] = ld4(x + e);
                    mv[u] = ld4(m + e);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t e = base + u * kGroup + lane0;
                if (e < len) {
                    f4 g = GL::widen(gr[u]) * sl.gscale;
                    sgdm4(xv[u], mv[u], g, h.momentum, sl.lr, ch.wd);
                    st4(x + e, xv[u]);
                    st4(m + e, mv[u]);
                }
            }
        }
    }
}

struct OuterArgs {
    float inv_k, lr, mu;
    int nesterov;
};

// OuterOPT on four elements given the replica sum (Sec. 4.2; Sec. 4.3).
__device__ __forceinline__ f4 outer4(f4 sum, f4 xg, f4& om, const OuterArgs& a) {
    f4 delta = xg - sum * a.inv_k;                 // Delta = x - mean_k x_k
    om = a.mu * om + delta;
    f4 dir = a.nesterov ? delta + a.mu * om : om;
    return xg - a.lr * dir;
}

// Variant 1: each lane owns four consecutive elements and walks the K rows in ascending
// order, eight independent loads in flight at a time.
__global__ __launch_bounds__(kThreads) void outer_kernel_walk(float* __restrict__ X, float* __restrict__ XG,
                                                              float* __restrict__ OM, uint64_t n4,
                                                              uint64_t row_stride, uint32_t K, OuterArgs a) {
    uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n4) return;
    uint64_t e = i * 4;
    f4 xg = ld4(XG + e);
    f4 om = ld4(OM + e);
    f4 sum = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t k0 = 0; k0 < K; k0 += 8) {
        f4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < K) t[u] = ld4(X + (uint64_t)(k0 + u) * row_stride + e);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < K) sum += t[u];
    }
    f4 xn = outer4(sum, xg, om, a);
    st4(XG + e, xn);
    st4(OM + e, om);
    for (uint32_t k = 0; k < K; ++k) st4(X + (uint64_t)k * row_stride + e, xn);
}

// Variant 2: a workgroup owns a tile of 4 x 256 elements.  Wave w sums the replicas
// k = w, w+4, ... for the whole tile, the four partial sums per element meet in LDS,
// and wave w finishes sub-tile w: fixed-order combine, OuterOPT, stores.  Puts 4*ceil(K/4)
// row loads in flight per lane before the first add.
__global__ __launch_bounds__(kThreads) void outer_kernel_lds(float* __restrict__ X, float* __restrict__ XG,
                                                             float* __restrict__ OM, uint64_t n4,
                                                             uint64_t row_stride, uint32_t K, OuterArgs a) {
    __shared__ f4 part[4][4][64];  // [wave][sub-tile][lane], 16 KiB
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint64_t tile4 = (uint64_t)blockIdx.x * 256;  // first float4 of the tile
    f4 acc[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[s] = (f4){0.f, 0.f, 0.f, 0.f};
    for (uint32_t k = w; k < K; k += 4) {
        const float* row = X + (uint64_t)k * row_stride;
        f4 t[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint64_t i = tile4 + s * 64 + lane;
            t[s] = i < n4 ? ld4(row + i * 4) : (f4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[s] += t[s];
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) part[w][s][lane] = acc[s];
    __syncthreads();
    const uint64_t i = tile4 + w * 64 + lane;
    if (i < n4) {
        const uint64_t e = i * 4;
        f4 sum = ((part[0][w][lane] + part[1][w][lane]) + part[2][w][lane]) + part[3][w][lane];
        f4 xg = ld4(XG + e);
        f4 om = ld4(OM + e);
        f4 xn = outer4(sum, xg, om, a);
        st4(XG + e, xn);
        st4(OM + e, om);
        for (uint32_t k = 0; k < K; ++k) st4(X + (uint64_t)k * row_stride + e, xn);
    }
}

// x_k^(0) <- x^(0) for all k, XG <- x^(0), cleared moments (Alg. 1, first line of the worker loop).
__global__ __launch_bounds__(kThreads) void init_kernel(const float* __restrict__ x0, float* __restrict__ X,
                                                        float* __restrict__ M, float* __restrict__ V,
                                                        float* __restrict__ XG, float* __restrict__ OM,
                                                        uint64_t n4, uint64_t row_stride, uint32_t K) {
    uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n4) return;
    uint64_t e = i * 4;
    f4 v = *(const f4*)(x0 + e);
    f4 z = {0.f, 0.f, 0.f, 0.f};
    st4(XG + e, v);
    st4(OM + e, z);
    for (uint32_t k = 0; k < K; ++k) {
        uint64_t r = (uint64_t)k * row_stride + e;
        st4(X + r, v);
        st4(M + r, z);
        if (V) st4(V + r, z);
    }
}

thread_local char g_error[256] = "";

void set_error(char* dst, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
}

// SplitMix64 output function as a counter hash (Steele, Lea, Flood 2014), top 24 bits.
uint32_t draw_u24(uint64_t seed, uint64_t t, uint32_t k, uint32_t K) {
    uint64_t z = seed + (t * (uint64_t)K + k + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z >> 40);
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

struct palsgd_ctx {
    palsgd_config cfg;
    palsgd_buffers buf;
    std::vector<uint64_t> numel, offset;
    std::vector<float> wd_mult;
    uint64_t P_padded = 0;
    uint32_t draw_threshold = 0;
    uint32_t chunk_elems = kDefaultChunk;
    uint32_t outer_variant = 0;
    Chunk* d_chunks = nullptr;
    uint32_t n_chunks = 0;
    uint64_t tau[PALSGD_MAX_K] = {0};
    uint64_t n_outer = 0;
    uint64_t last_outer_t = 0;
    char error[256] = "";
};

namespace {

palsgd_status layout_impl(uint32_t n_tensors, const uint64_t* numel, uint64_t* P_padded, uint64_t* offs,
                          char* err) {
    if (!numel || !P_padded || n_tensors == 0) {
        set_error(err, "palsgd_layout: NULL argument or n_tensors == 0");
        return PALSGD_EINVAL;
    }
    uint64_t cur = 0;
    for (uint32_t j = 0; j < n_tensors; ++j) {
        if (numel[j] == 0) {
            set_error(err, "palsgd_layout: tensor %u has zero elements", j);
            return PALSGD_EINVAL;
        }
        if (offs) offs[j] = cur;
        cur = (cur + numel[j] + 63u) / 64u * 64u;
    }
    *P_padded = cur;
    return PALSGD_OK;
}

// Cut the row into chunks: neighbouring tensors with the same multiplier form one range
// (rows are flat, padding included), each range is cut every chunk_elems elements.
palsgd_status build_chunks(palsgd_ctx* c) {
    std::vector<Chunk> host;
    const size_t nt = c->numel.size();
    size_t j = 0;
    while (j < nt) {
        size_t j2 = j + 1;
        while (j2 < nt && c->wd_mult[j2] == c->wd_mult[j]) ++j2;
        uint64_t begin = c->offset[j];
        uint64_t end = j2 < nt ? c->offset[j2] : c->P_padded;
        float wd = (float)((double)c->cfg.weight_decay * (double)c->wd_mult[j]);
        for (uint64_t o = begin; o < end; o += c->chunk_elems) {
            uint64_t l = end - o < c->chunk_elems ? end - o : c->chunk_elems;
            host.push_back(Chunk{o, (uint32_t)l, wd});
        }
        j = j2;
    }
    Chunk* d = nullptr;
    hipError_t e = hipMalloc(&d, host.size() * sizeof(Chunk));
    if (e != hipSuccess) {
        set_error(c->error, "hipMalloc(chunk table): %s", hipGetErrorString(e));
        return PALSGD_ENOMEM;
    }
    e = hipMemcpy(d, host.data(), host.size() * sizeof(Chunk), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        set_error(c->error, "hipMemcpy(chunk table): %s", hipGetErrorString(e));
        (void)hipFree(d);
        return PALSGD_EHIP;
    }
    if (c->d_chunks) (void)hipFree(c->d_chunks);
    c->d_chunks = d;
    c->n_chunks = (uint32_t)host.size();
    return PALSGD_OK;
}

palsgd_status check_launch(palsgd_ctx* c, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(c->error, "%s: %s", what, hipGetErrorString(e));
        return PALSGD_EHIP;
    }
    return PALSGD_OK;
}

template <int INNER, int GDT>
void launch_step(palsgd_ctx* c, const StepArgs& args, uint32_t n_slots, hipStream_t st) {
    dim3 grid(c->n_chunks, n_slots), block(kThreads);
    Hyper h{c->cfg.beta1, c->cfg.beta2, c->cfg.eps, c->cfg.momentum};
    step_kernel<INNER, GDT, 2><<<grid, block, 0, st>>>(args, c->d_chunks, c->buf.X, c->buf.M, c->buf.V, c->buf.G,
                                                       c->buf.XG, c->buf.row_stride, h);
}

// Shared body of palsgd_inner_step / palsgd_pseudo_sync / palsgd_step.
palsgd_status local_update(palsgd_ctx* c, const char* who, uint64_t t, float alpha, float eta,
                           const float* grad_scale, const uint8_t* mask_override, bool do_grad, bool do_mix,
                           void* stream) {
    if (!c) {
        set_error(g_error, "%s: NULL context", who);
        return PALSGD_EINVAL;
    }
    if (!(alpha >= 0.0f) || !std::isfinite(alpha)) {
        set_error(c->error, "%s: alpha_t must be finite and >= 0", who);
        return PALSGD_EINVAL;
    }
    if (do_mix && (!std::isfinite(eta) || !(eta >= 0.0f))) {
        set_error(c->error, "%s: eta_t must be finite and >= 0", who);
        return PALSGD_EINVAL;
    }
    const uint32_t K = c->cfg.K;
    const double p = c->cfg.p;
    StepArgs args;
    uint32_t n = 0;
    bool stepped[PALSGD_MAX_K] = {false};
    for (uint32_t k = 0; k < K; ++k) {
        bool mix = mask_override ? mask_override[k] != 0 : draw_u24(c->cfg.seed, t, k, K) < c->draw_threshold;
        if (mix ? !do_mix : !do_grad) continue;
        Slot& s = args.s[n++];
        s.replica = k;
        s.mix = mix ? 1u : 0u;
        s.lr = s.c1 = s.c2 = s.beta_mix = 0.0f;
        s.gscale = 1.0f;
        if (mix) {
            if (p <= 0.0) {
                set_error(c->error, "%s: worker %u is to mix but p == 0 (alpha*eta/p undefined)", who, k);
                return PALSGD_EINVAL;
            }
            s.beta_mix = (float)((double)alpha * (double)eta / p);
        } else {
            double lr = (double)alpha / (1.0 - p);
            double tau = (double)(c->tau[k] + 1);
            s.lr = (float)lr;
            if (c->cfg.inner == PALSGD_INNER_ADAMW) {
                s.c1 = (float)(lr / (1.0 - std::pow((double)c->cfg.beta1, tau)));
                s.c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.beta2, tau)));
            }
            if (grad_scale) {
                if (!std::isfinite(grad_scale[k])) {
                    set_error(c->error, "%s: grad_scale[%u] is not finite", who, k);
                    return PALSGD_EINVAL;
                }
                s.gscale = grad_scale[k];
            }
            stepped[k] = true;
        }
    }
    if (n == 0) return PALSGD_OK;
    if (!c->d_chunks) {  // the device table is made on the first launch that needs it
        palsgd_status rc = build_chunks(c);
        if (rc != PALSGD_OK) return rc;
    }
    hipStream_t st = (hipStream_t)stream;
    const bool adamw = c->cfg.inner == PALSGD_INNER_ADAMW, bf16 = c->cfg.grad_dtype == PALSGD_GRAD_BF16;
    if (adamw && bf16) launch_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_BF16>(c, args, n, st);
    else if (adamw) launch_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_F32>(c, args, n, st);
    else if (bf16) launch_step<PALSGD_INNER_SGDM, PALSGD_GRAD_BF16>(c, args, n, st);
    else launch_step<PALSGD_INNER_SGDM, PALSGD_GRAD_F32>(c, args, n, st);
    palsgd_status rc = check_launch(c, who);
    if (rc != PALSGD_OK) return rc;
    for (uint32_t k = 0; k < K; ++k)
        if (stepped[k]) c->tau[k] += 1;
    return PALSGD_OK;
}

}  // namespace

extern "C" {

palsgd_status palsgd_layout(const palsgd_config* cfg, uint64_t* P_padded, uint64_t* tensor_offset) {
    if (!cfg) {
        set_error(g_error, "palsgd_layout: NULL config");
        return PALSGD_EINVAL;
    }
    return layout_impl(cfg->n_tensors, cfg->tensor_numel, P_padded, tensor_offset, g_error);
}

palsgd_status palsgd_init(const palsgd_config* cfg, const palsgd_buffers* buf, const float* x0_dev, void* stream,
                          palsgd_ctx** out) {
    if (out) *out = nullptr;
    if (!cfg || !buf || !out) {
        set_error(g_error, "palsgd_init: NULL argument");
        return PALSGD_EINVAL;
    }
    uint64_t P_padded = 0;
    std::vector<uint64_t> offs(cfg->n_tensors ? cfg->n_tensors : 1);
    palsgd_status rc = layout_impl(cfg->n_tensors, cfg->tensor_numel, &P_padded, offs.data(), g_error);
    if (rc != PALSGD_OK) return rc;
#define PALSGD_REQUIRE(cond, msg)                          \
    if (!(cond)) {                                         \
        set_error(g_error, "palsgd_init: %s", msg);        \
        return PALSGD_EINVAL;                              \
    }
    PALSGD_REQUIRE(cfg->K >= 1 && cfg->K <= PALSGD_MAX_K, "K must be in 1..64");
    PALSGD_REQUIRE(cfg->H >= 1, "H must be >= 1");
    PALSGD_REQUIRE(cfg->p >= 0.0 && cfg->p < 1.0, "p must satisfy 0 <= p < 1");
    PALSGD_REQUIRE(cfg->inner == PALSGD_INNER_ADAMW || cfg->inner == PALSGD_INNER_SGDM, "unknown inner optimizer");
    PALSGD_REQUIRE(cfg->grad_dtype == PALSGD_GRAD_F32 || cfg->grad_dtype == PALSGD_GRAD_BF16, "unknown gradient dtype");
    PALSGD_REQUIRE(std::isfinite(cfg->weight_decay) && cfg->weight_decay >= 0.0f, "weight_decay must be finite, >= 0");
    if (cfg->inner == PALSGD_INNER_ADAMW) {
        PALSGD_REQUIRE(cfg->beta1 >= 0.0f && cfg->beta1 < 1.0f, "beta1 must satisfy 0 <= beta1 < 1");
        PALSGD_REQUIRE(cfg->beta2 >= 0.0f && cfg->beta2 < 1.0f, "beta2 must satisfy 0 <= beta2 < 1");
        PALSGD_REQUIRE(std::isfinite(cfg->eps) && cfg->eps >= 0.0f, "eps must be finite, >= 0");
        PALSGD_REQUIRE(buf->V != nullptr, "V buffer is required by AdamW");
    } else {
        PALSGD_REQUIRE(std::isfinite(cfg->momentum) && cfg->momentum >= 0.0f && cfg->momentum < 1.0f,
                       "momentum must satisfy 0 <= momentum < 1");
    }
    PALSGD_REQUIRE(std::isfinite(cfg->outer_lr) && cfg->outer_lr >= 0.0f, "outer_lr must be finite, >= 0");
    PALSGD_REQUIRE(std::isfinite(cfg->outer_momentum) && cfg->outer_momentum >= 0.0f && cfg->outer_momentum < 1.0f,
                   "outer_momentum must satisfy 0 <= outer_momentum < 1");
    PALSGD_REQUIRE(buf->X && buf->M && buf->G && buf->XG && buf->OM, "NULL device buffer");
    PALSGD_REQUIRE(aligned16(buf->X) && aligned16(buf->M) && aligned16(buf->V) && aligned16(buf->G) &&
                       aligned16(buf->XG) && aligned16(buf->OM) && aligned16(x0_dev),
                   "device buffers must be 16-byte aligned");
    PALSGD_REQUIRE(buf->row_stride >= P_padded && buf->row_stride % 64 == 0,
                   "row_stride must be a multiple of 64 and >= the padded row length");
    if (cfg->tensor_wd_mult)
        for (uint32_t j = 0; j < cfg->n_tensors; ++j)
            PALSGD_REQUIRE(std::isfinite(cfg->tensor_wd_mult[j]) && cfg->tensor_wd_mult[j] >= 0.0f,
                           "tensor_wd_mult entries must be finite, >= 0");
#undef PALSGD_REQUIRE

    palsgd_ctx* c = new (std::nothrow) palsgd_ctx;
    if (!c) {
        set_error(g_error, "palsgd_init: out of host memory");
        return PALSGD_ENOMEM;
    }
    c->cfg = *cfg;
    c->buf = *buf;
    c->numel.assign(cfg->tensor_numel, cfg->tensor_numel + cfg->n_tensors);
    c->offset = offs;
    c->wd_mult.assign(cfg->n_tensors, 1.0f);
    if (cfg->tensor_wd_mult) c->wd_mult.assign(cfg->tensor_wd_mult, cfg->tensor_wd_mult + cfg->n_tensors);
    c->cfg.tensor_numel = nullptr;  // the caller's arrays are not kept
    c->cfg.tensor_wd_mult = nullptr;
    c->P_padded = P_padded;
    c->draw_threshold = (uint32_t)std::floor(cfg->p * 16777216.0);
    if (x0_dev) {
        uint64_t n4 = P_padded / 4;
        uint32_t blocks = (uint32_t)((n4 + kThreads - 1) / kThreads);
        init_kernel<<<blocks, kThreads, 0, (hipStream_t)stream>>>(x0_dev, buf->X, buf->M, buf->V, buf->XG, buf->OM,
                                                                  n4, buf->row_stride, cfg->K);
        rc = check_launch(c, "palsgd_init");
        if (rc != PALSGD_OK) {
            memcpy(g_error, c->error, sizeof g_error);
            palsgd_destroy(c);
            return rc;
        }
    }
    *out = c;
    return PALSGD_OK;
}

palsgd_status palsgd_draw(const palsgd_ctx* ctx, uint64_t t, uint8_t* mask_out) {
    if (!ctx || !mask_out) {
        set_error(g_error, "palsgd_draw: NULL argument");
        return PALSGD_EINVAL;
    }
    for (uint32_t k = 0; k < ctx->cfg.K; ++k)
        mask_out[k] = draw_u24(ctx->cfg.seed, t, k, ctx->cfg.K) < ctx->draw_threshold ? 1 : 0;
    return PALSGD_OK;
}

palsgd_status palsgd_inner_step(palsgd_ctx* ctx, uint64_t t, float alpha_t, const float* grad_scale,
                                const uint8_t* mask_override, void* stream) {
    return local_update(ctx, "palsgd_inner_step", t, alpha_t, 0.0f, grad_scale, mask_override, true, false, stream);
}

palsgd_status palsgd_pseudo_sync(palsgd_ctx* ctx, uint64_t t, float alpha_t, float eta_t,
                                 const uint8_t* mask_override, void* stream) {
    return local_update(ctx, "palsgd_pseudo_sync", t, alpha_t, eta_t, nullptr, mask_override, false, true, stream);
}

palsgd_status palsgd_step(palsgd_ctx* ctx, uint64_t t, float alpha_t, float eta_t, const float* grad_scale,
                          const uint8_t* mask_override, void* stream) {
    return local_update(ctx, "palsgd_step", t, alpha_t, eta_t, grad_scale, mask_override, true, true, stream);
}

palsgd_status palsgd_outer_step(palsgd_ctx* ctx, uint64_t t, void* stream) {
    if (!ctx) {
        set_error(g_error, "palsgd_outer_step: NULL context");
        return PALSGD_EINVAL;
    }
    const uint32_t K = ctx->cfg.K;
    OuterArgs a{(float)(1.0 / (double)K), ctx->cfg.outer_lr, ctx->cfg.outer_momentum, ctx->cfg.outer_nesterov ? 1 : 0};
    const uint64_t n4 = ctx->P_padded / 4;
    hipStream_t st = (hipStream_t)stream;
    uint32_t variant = ctx->outer_variant ? ctx->outer_variant : 1u;
    if (variant == 2) {
        uint32_t blocks = (uint32_t)((n4 + 255) / 256);
        outer_kernel_lds<<<blocks, kThreads, 0, st>>>(ctx->buf.X, ctx->buf.XG, ctx->buf.OM, n4, ctx->buf.row_stride, K, a);
    } else {
        uint32_t blocks = (uint32_t)((n4 + kThreads - 1) / kThreads);
        outer_kernel_walk<<<blocks, kThreads, 0, st>>>(ctx->buf.X, ctx->buf.XG, ctx->buf.OM, n4, ctx->buf.row_stride, K, a);
    }
    palsgd_status rc = check_launch(ctx, "palsgd_outer_step");
    if (rc != PALSGD_OK) return rc;
    ctx->n_outer += 1;
    ctx->last_outer_t = t;
    return PALSGD_OK;
}

palsgd_status palsgd_get_state(const palsgd_ctx* ctx, uint64_t* tau, uint64_t* n_outer) {
    if (!ctx) {
        set_error(g_error, "palsgd_get_state: NULL context");
        return PALSGD_EINVAL;
    }
    if (tau) memcpy(tau, ctx->tau, ctx->cfg.K * sizeof(uint64_t));
    if (n_outer) *n_outer = ctx->n_outer;
    return PALSGD_OK;
}

palsgd_status palsgd_set_state(palsgd_ctx* ctx, const uint64_t* tau, uint64_t n_outer) {
    if (!ctx || !tau) {
        set_error(ctx ? ctx->error : g_error, "palsgd_set_state: NULL argument");
        return PALSGD_EINVAL;
    }
    memcpy(ctx->tau, tau, ctx->cfg.K * sizeof(uint64_t));
    ctx->n_outer = n_outer;
    return PALSGD_OK;
}

const char* palsgd_last_error(const palsgd_ctx* ctx) { return ctx ? ctx->error : g_error; }

void palsgd_destroy(palsgd_ctx* ctx) {
    if (!ctx) return;
    if (ctx->d_chunks) (void)hipFree(ctx->d_chunks);
    delete ctx;
}

palsgd_status palsgd_set_tuning(palsgd_ctx* ctx, uint32_t chunk_elems, uint32_t outer_variant) {
    if (!ctx) {
        set_error(g_error, "palsgd_set_tuning: NULL context");
        return PALSGD_EINVAL;
    }
    if (chunk_elems == 0) chunk_elems = kDefaultChunk;
    if (chunk_elems % 2048 != 0 || chunk_elems > kMaxChunk || outer_variant > 2) {
        set_error(ctx->error, "palsgd_set_tuning: chunk_elems must be a multiple of 2048 <= 65536, outer_variant 0..2");
        return PALSGD_EINVAL;
    }
    ctx->outer_variant = outer_variant;
    if (chunk_elems != ctx->chunk_elems) {
        ctx->chunk_elems = chunk_elems;
        if (ctx->d_chunks) {  // hipFree waits for the device, so no launch still reads the old table
            (void)hipFree(ctx->d_chunks);
            ctx->d_chunks = nullptr;
        }
    }
    return PALSGD_OK;
}

}  // extern "C"
