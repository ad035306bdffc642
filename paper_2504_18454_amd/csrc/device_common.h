// Types, constants and memory-access helpers shared by every kernel of the PALSGD update path
// (gfx950): the 16-byte vector type, the tile a wavefront covers, the per-slot scalars of a
// launch, streaming loads and stores, gradient widening, the wavefront sum.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/palsgd.h"

namespace palsgd_dev {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;            // lanes of a wavefront = threads of a streaming workgroup
constexpr int kTile = kWave * 4;     // elements a wavefront covers with one 16-byte group per lane
constexpr int kThreads = 256;        // workgroup of the LDS-staged outer variant and of init
constexpr uint32_t kLdsPerCUDefault = 160u * 1024u;  // gfx950; the device is asked at the first launch
constexpr uint32_t kInflightDefault = 72u * 1024u;  // bytes of loads+stores in flight per CU

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
    float wd;        // weight decay when every tensor has the same multiplier
    int nesterov;    // SGD-momentum: step along d + mu * buf instead of buf
};

__device__ __forceinline__ f4 ld4(const float* p) { return __builtin_nontemporal_load((const f4*)p); }
// Streaming store: non-temporal and agent scope ("sc1 nt").  The compiler's non-temporal
// store builtin emits "nt" alone; the agent-scope variant measured 2 % faster on the 7-stream
// update and is what every write-once store of this file uses.
__device__ __forceinline__ void st4(float* p, f4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}
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

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;  // lane 0 holds the sum
}

}  // namespace palsgd_dev
