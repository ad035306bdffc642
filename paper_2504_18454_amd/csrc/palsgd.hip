// PALSGD parameter-update path for MI355X (gfx950, CDNA4): the C ABI declared in
// include/palsgd.h (context, argument checks, launches) over the HIP kernels of this
// directory, which this one translation unit includes:
//   device_common.h     vector type, tile, per-slot scalars, streaming loads/stores
//   step_kernel.h       local update of all K workers (both branches) in one launch
//   outer_kernels.h     outer step, its fusion with the last local update, init
//   warmup_kernels.h    DDP warm-up step and the broadcast that ends the warm-up
//   reduce_kernels.h    gradient norms, consensus-distance diagnostics
//   schedule_kernels.h  branch draws, device-resident schedule for HIP graphs
//
// All kernels are bound by HBM bandwidth (about one flop per byte moved; the correctly
// rounded divide and the square root cost nothing measurable), so the design rules are:
//   * every access a full-width coalesced vector load/store: one wavefront instruction
//     touches one contiguous 1 KiB span (512 B for bf16 gradients);
//   * every byte of state read once and written once per step, non-temporal both ways;
//   * one launch per step whatever the number of tensors: rows are flat, a per-64-element
//     table carries the weight-decay multiplier only when tensors differ in it;
//   * ONE wavefront per workgroup, one 16-byte group per lane and stream, no loop: the
//     dispatcher streams tiles through the chip in address order, which keeps the DRAM
//     pages of the 7 streams open;
//   * a cap on the wavefronts resident per CU (through the workgroup's LDS allocation, of
//     which nothing is used): about 72 KiB of loads+stores in flight per CU is the
//     measured optimum; full occupancy loses 10-15 % to DRAM page conflicts.
//
//   step_kernel    Alg. 1 local update of all K workers in one launch: a wavefront owns
//                  (tile of a row, worker); the worker's branch (gradient step / mixing
//                  step) is uniform over the wavefront, so there is no divergence.
//   outer_kernel_* Alg. 1 outer step: K-way mean of the differences x - x_k, OuterOPT with
//                  (Nesterov) momentum, restart of the K workers; optionally the
//                  consensus-distance diagnostics from the values already in registers.
//   restart_rows_kernel
//                  the restart of the K workers as a launch of its own, used from K = 24 up
//                  while the global model fits the memory-side cache: short store-only
//                  wavefronts fill the rows faster than a reducing wavefront that has K
//                  stores to issue.
//   init_kernel    x_k^(0) <- x^(0), cleared optimizer state.
//   ddp_kernel     DDP step of the warm-up phase: K-way gradient mean + one InnerOPT step.
//   plan_kernel    device-resident schedule (draws, step counts, bias corrections) for
//                  callers that replay the step from a HIP graph.
//   sumsq_kernel, diag_kernel, fold_kernel, *_finish_kernel
//                  scalar reductions (gradient norms for clipping, consensus distance):
//                  lane-local sums, a shuffle tree per wavefront, fixed-order folds in double.
//
// All device memory of the library (weight-decay table, reduction scratch, device schedule) is
// allocated by palsgd_init; no other entry point allocates, so each may be captured in a HIP graph.
//
// No matrix cores: nothing here is a contraction.  No data goes through LDS in the step
// kernel: there is no reuse to stage.  Each XCD's private L2 is irrelevant to pure
// streaming; remapping tiles so that an XCD walks a contiguous range measured slower
// than the plain blockIdx order, so the map is the plain row-major one.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/palsgd.h"
#include "device_common.h"
#include "outer_kernels.h"
#include "reduce_kernels.h"
#include "schedule_kernels.h"
#include "step_kernel.h"
#include "warmup_kernels.h"

using namespace palsgd_dev;

// Scratch of palsgd_clip_grad_norm_noalloc, the entry point for callers that cannot allocate: part of the
// library's code object, so every GPU the library runs on holds its own copy (16.1 MiB) until the process
// ends.  Layout: 2 * PALSGD_MAX_K * kFold floats that hold the second-stage sums (as PALSGD_MAX_K * kFold
// doubles), then up to kStaticMaxParts first-stage partial sums.  In host code this name is only a handle
// for hipGetSymbolAddress: the device address it yields (per device, kept in g_static_scratch) is what the
// launches get.
constexpr uint32_t kStaticFoldFloats = 2u * PALSGD_MAX_K * kFold;
constexpr uint32_t kStaticMaxParts = 1u << 22;
static __device__ __align__(256) float scratch[kStaticFoldFloats + kStaticMaxParts];

namespace {

// ======== host side: context, argument checks, launches ========

thread_local char g_error[256] = "";

void set_error(char* dst, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Device address of `scratch` on the current device, looked up once per device (with that device current)
// and kept: each GPU has its own copy of the array at its own address.
constexpr int kMaxDevices = 64;
float* g_static_scratch[kMaxDevices] = {nullptr};
std::mutex g_static_scratch_mutex;

palsgd_status static_scratch(char* err, float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error(err, "static scratch: hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
        return PALSGD_EHIP;
    }
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error(err, "static scratch: hipGetSymbolAddress on device %d: %s", dev, hipGetErrorString(e));
            return PALSGD_EHIP;
        }
        g_static_scratch[dev] = (float*)p;
    }
    if (out) *out = g_static_scratch[dev];
    return PALSGD_OK;
}

}  // namespace

struct palsgd_ctx {
    palsgd_config cfg;
    palsgd_buffers buf;
    std::vector<uint64_t> numel, offset;
    std::vector<float> wd_mult;
    uint64_t P_padded = 0;
    uint32_t draw_threshold = 0;
    bool wd_uniform = true;        // every tensor has the same weight-decay multiplier
    float wd_eff0 = 0.0f;          // weight_decay * that multiplier
    float* d_wd_tab = nullptr;     // else: weight_decay * multiplier per 64 elements of a row
    float* d_scratch = nullptr;    // partial sums of the scalar reductions + their K+2 results
    bool clip_armed = false;       // d_scratch holds clipping scales for the next gradient step
    bool clip_mean_armed = false;  // ... and the scale of the averaged gradient for the next DDP step
    bool moments_shared = false;   // after DDP steps: only replica 0's M, V are current
    bool model_shared = false;     // after palsgd_ddp_step_shared: the rows of X are stale, the model is XG
    void* d_schedule = nullptr;    // DevSchedule of the graph-capturable mode
    bool capturable = false;       // between palsgd_capturable_begin and palsgd_capturable_end
    bool host_only = false;        // created with no GPU visible: draws and scalar state only, every launch is refused
    uint32_t step_waves = 0;       // cap on resident wavefronts per CU, 0 = derive from bytes per wavefront
    uint32_t outer_waves = 0;
    uint32_t outer_variant = 0;
    uint64_t tau[PALSGD_MAX_K] = {0};
    uint64_t n_outer = 0;
    uint64_t last_outer_t = 0;
    mutable char error[256] = "";  // written by const entry points too
};

namespace {

// One lane per four elements and fewer than 2^32 work-items per launch dimension: rows below 2^34 elements.
constexpr uint64_t kMaxRow = 1ull << 33;

palsgd_status layout_impl(uint32_t n_tensors, const uint64_t* numel, uint64_t P_stated, uint64_t* P_padded,
                          uint64_t* offs, char* err) {
    if (!numel || !P_padded || n_tensors == 0) {
        set_error(err, "palsgd_layout: NULL argument or n_tensors == 0");
        return PALSGD_EINVAL;
    }
    uint64_t cur = 0, total = 0;
    for (uint32_t j = 0; j < n_tensors; ++j) {
        if (numel[j] == 0) {
            set_error(err, "palsgd_layout: tensor %u has zero elements", j);
            return PALSGD_EINVAL;
        }
        if (offs) offs[j] = cur;
        cur = (cur + numel[j] + 63u) / 64u * 64u;
        total += numel[j];
    }
    if (P_stated != 0 && P_stated != total) {
        set_error(err, "palsgd_layout: P = %llu but the tensors hold %llu elements", (unsigned long long)P_stated,
                  (unsigned long long)total);
        return PALSGD_EINVAL;
    }
    // rows end on a tile boundary: with row_stride = P_padded every wavefront's 1 KiB access is 1 KiB-aligned
    // in every row (rows shifted against each other by 256 B measured 3 % slower)
    *P_padded = (cur + kTile - 1) / kTile * kTile;
    return PALSGD_OK;
}

// Device table with weight_decay * multiplier for every 64 elements of a row (a tensor's
// tail padding takes the tensor's value).  Only needed when the multipliers differ.
palsgd_status build_wd_table(palsgd_ctx* c) {
    const uint64_t blocks = c->P_padded / 64;
    std::vector<float> host(blocks);
    const size_t nt = c->numel.size();
    for (size_t j = 0; j < nt; ++j) {
        uint64_t begin = c->offset[j] / 64;
        uint64_t end = (j + 1 < nt ? c->offset[j + 1] : c->P_padded) / 64;
        float wd = (float)((double)c->cfg.weight_decay * (double)c->wd_mult[j]);
        for (uint64_t q = begin; q < end; ++q) host[q] = wd;
    }
    float* d = nullptr;
    hipError_t e = hipMalloc(&d, blocks * sizeof(float));
    if (e != hipSuccess) {
        set_error(c->error, "hipMalloc(weight-decay table): %s", hipGetErrorString(e));
        return PALSGD_ENOMEM;
    }
    e = hipMemcpy(d, host.data(), blocks * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        set_error(c->error, "hipMemcpy(weight-decay table): %s", hipGetErrorString(e));
        (void)hipFree(d);
        return PALSGD_EHIP;
    }
    c->d_wd_tab = d;
    return PALSGD_OK;
}

// LDS bytes to request per workgroup so that at most `groups` workgroups are resident on a
// CU (0 = no cap).  The kernels use none of it: the allocation is the occupancy throttle.
uint32_t g_lds_per_cu = 0;

uint32_t lds_per_cu() {
    if (g_lds_per_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) == hipSuccess &&
            v >= 65536)
            g_lds_per_cu = (uint32_t)v;
        else
            g_lds_per_cu = kLdsPerCUDefault;
        (void)hipGetLastError();
    }
    return g_lds_per_cu;
}

uint32_t lds_cap(uint32_t groups, uint32_t static_lds) {
    if (groups == 0 || groups >= 32) return 0;
    uint32_t l = lds_per_cu() / groups / 512u * 512u;
    if (l > 65536u) l = 65536u;
    return l > static_lds ? l - static_lds : 0;
}

// Wavefronts per CU that keep about kInflightDefault bytes of loads+stores in flight.
uint32_t auto_waves(uint32_t bytes_per_wave, uint32_t floor_waves = 3) {
    uint32_t w = (kInflightDefault + bytes_per_wave / 2) / bytes_per_wave;
    return w < floor_waves ? floor_waves : (w > 32 ? 32 : w);
}

// Scalars of the outer step that comes next (its number, from 1, sets AdamW's bias corrections).
OuterArgs outer_args_of(const palsgd_ctx* c) {
    OuterArgs a{};
    a.inv_k = (float)(1.0 / (double)c->cfg.K);
    a.lr = c->cfg.outer_lr;
    a.mu = c->cfg.outer_momentum;
    a.nesterov = c->cfg.outer_nesterov ? 1 : 0;
    if (c->cfg.outer_opt == PALSGD_OUTER_ADAMW) {
        const double n = (double)(c->n_outer + 1);
        a.b1 = c->cfg.outer_beta1;
        a.b2 = c->cfg.outer_beta2;
        a.eps = c->cfg.outer_eps;
        a.c1 = (float)((double)c->cfg.outer_lr / (1.0 - std::pow((double)c->cfg.outer_beta1, n)));
        a.c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)c->cfg.outer_beta2, n)));
        a.decay = c->cfg.outer_lr * c->cfg.outer_weight_decay;
    }
    return a;
}

// True while `st` records a stream capture (a query that fails, as on the null stream next to another
// stream's capture, counts as not capturing).
bool stream_is_capturing(hipStream_t st) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status != hipStreamCaptureStatusNone;
}

// OuterOPT = AdamW takes its bias corrections from the host-side outer-step count as launch arguments: a
// captured launch would replay the first one's corrections for ever.
palsgd_status refuse_captured_outer_adamw(palsgd_ctx* c, const char* who, hipStream_t st) {
    if (c->cfg.outer_opt == PALSGD_OUTER_ADAMW && stream_is_capturing(st)) {
        set_error(c->error, "%s: an outer step with OuterOPT = AdamW cannot be captured into a HIP graph "
                            "(its bias corrections are launch arguments)", who);
        return PALSGD_ESTATE;
    }
    return PALSGD_OK;
}

Hyper hyper_of(const palsgd_ctx* c) {
    return Hyper{c->cfg.beta1, c->cfg.beta2, c->cfg.eps, c->cfg.momentum, c->wd_eff0, c->cfg.inner_nesterov != 0};
}

// Every entry point calls this before its first launch: it refuses a context that was created without a
// GPU, and it drops an error that another library may have left in the runtime, so that what check_launch
// reads afterwards is the status of this entry point's own launches.
palsgd_status begin_launches(palsgd_ctx* c, const char* who) {
    if (c->host_only) {
        set_error(c->error, "%s: no GPU was visible when this context was created; it serves palsgd_draw and "
                            "the scalar state calls only", who);
        return PALSGD_EHIP;
    }
    (void)hipGetLastError();
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

// Scratch layout (floats): [0, 64) per-worker clipping scales | [64] clipping scale of the averaged
// gradient | from 128: 64 * kFold doubles of second-stage sums | first-stage partial sums (one per
// wavefront of the producing kernel).
uint32_t norm_parts(const palsgd_ctx* c) {
    return (uint32_t)((c->P_padded + (uint64_t)kTile * kNormTiles - 1) / ((uint64_t)kTile * kNormTiles));
}
uint32_t diag_parts(const palsgd_ctx* c) {
    return (uint32_t)((c->P_padded + (uint64_t)kTile * kDiagTiles - 1) / ((uint64_t)kTile * kDiagTiles));
}
uint32_t tile_count(const palsgd_ctx* c) { return (uint32_t)((c->P_padded + kTile - 1) / kTile); }
float* clip_scales(palsgd_ctx* c) { return c->d_scratch; }
float* mean_clip_scale(palsgd_ctx* c) { return c->d_scratch + PALSGD_MAX_K; }
double* scratch_fold(palsgd_ctx* c) { return (double*)(c->d_scratch + 2 * PALSGD_MAX_K); }
float* scratch_partials(palsgd_ctx* c) { return c->d_scratch + 2 * PALSGD_MAX_K + 2 * PALSGD_MAX_K * kFold; }

// The library's device memory beyond the weight-decay table, all of it allocated by palsgd_init so that no
// later call allocates: the reduction scratch (sized for the largest producer: K rows of norm partials, or two
// partials per tile for the diagnostics fused into the outer step) and the device-resident schedule.
palsgd_status alloc_device_state(palsgd_ctx* c) {
    uint64_t parts = (uint64_t)c->cfg.K * norm_parts(c);
    if (parts < 2ull * tile_count(c)) parts = 2ull * tile_count(c);
    uint64_t floats = 2ull * PALSGD_MAX_K + 2ull * PALSGD_MAX_K * kFold + parts;
    float* d = nullptr;
    hipError_t e = hipMalloc(&d, floats * sizeof(float));
    if (e != hipSuccess) {
        set_error(c->error, "hipMalloc(reduction scratch): %s", hipGetErrorString(e));
        return PALSGD_ENOMEM;
    }
    c->d_scratch = d;
    e = hipMalloc(&c->d_schedule, sizeof(DevSchedule));
    if (e != hipSuccess) {
        c->d_schedule = nullptr;
        set_error(c->error, "hipMalloc(device schedule): %s", hipGetErrorString(e));
        return PALSGD_ENOMEM;
    }
    return PALSGD_OK;
}

// When the outer step, the fused synchronisation step and the DDP step leave the K row stores to a second launch:
// from 24 workers on, and only while the global model, which that launch re-reads once per group of rows, is
// served by the 256 MB memory-side cache (rows up to 192 MiB).  Measured through the library: at 16-192 MiB rows the
// two launches are ahead by 4-8 % at K = 24, 8-10 % at K = 32 and 12-18 % at K = 48-64, level at K = 20; at 256 MiB rows
// and beyond the re-reads come from DRAM and one launch is ahead by 2-10 % for every K up to 64.
constexpr uint32_t kSplitOuterFromK = 24;
constexpr uint64_t kSplitOuterMaxRowBytes = 192ull << 20;

bool restart_apart(const palsgd_ctx* c) {
    if (c->outer_variant == 3) return true;
    return c->outer_variant == 0 && c->cfg.K >= kSplitOuterFromK && c->P_padded * sizeof(float) <= kSplitOuterMaxRowBytes;
}

// X[k] <- XG for all k as short wavefronts, one group of rows after the other, 16 resident per CU.
void launch_restart_rows(palsgd_ctx* c, hipStream_t st) {
    dim3 grid(tile_count(c), (c->cfg.K + kRestartRows - 1) / kRestartRows);
    restart_rows_kernel<<<grid, kWave, lds_cap(16, 0), st>>>(c->buf.X, c->buf.XG, c->P_padded, c->buf.row_stride, c->cfg.K);
}

template <int INNER, int GDT>
void launch_step(palsgd_ctx* c, const StepArgs& args, const Slot* dev_slots, uint32_t n_slots, bool any_grad,
                 const float* clip, hipStream_t st) {
    const uint64_t n = c->P_padded;
    // mixing wavefronts take two tiles each, so a mixing-only launch needs half the grid
    const uint32_t tiles = (uint32_t)(any_grad ? (n + kTile - 1) / kTile : (n + 2 * kTile - 1) / (2 * kTile));
    const uint32_t per_elem = any_grad ? (INNER == PALSGD_INNER_ADAMW ? 24u : 16u) + (GDT == PALSGD_GRAD_F32 ? 4u : 2u)
                                       : 24u;
    const uint32_t waves = c->step_waves ? c->step_waves : auto_waves(per_elem * kTile);
    dim3 grid(tiles, n_slots), block(kWave);
    Hyper h = hyper_of(c);
    const uint32_t lds = lds_cap(waves, 0);
    const palsgd_buffers& b = c->buf;
#define PALSGD_STEP(TAB, DEV, tab)                                                                              \
    step_kernel<INNER, GDT, TAB, DEV><<<grid, block, lds, st>>>(args, dev_slots, tab, b.X, b.M, b.V, b.G, b.XG, clip, n, \
                                                                b.row_stride, h)
    if (c->wd_uniform && !dev_slots) PALSGD_STEP(false, false, nullptr);
    else if (c->wd_uniform) PALSGD_STEP(false, true, nullptr);
    else if (!dev_slots) PALSGD_STEP(true, false, c->d_wd_tab);
    else PALSGD_STEP(true, true, c->d_wd_tab);
#undef PALSGD_STEP
}

// What the DDP steps of the warm-up kept once for the identical workers goes to every worker:
// replica 0's InnerOPT state to replicas 1..K-1, the common model XG to the K rows of X.
palsgd_status end_warmup_sharing(palsgd_ctx* c, const char* who, hipStream_t st) {
    if (!c->moments_shared && !c->model_shared) return PALSGD_OK;
    const uint32_t K = c->cfg.K;
    const bool adamw = c->cfg.inner == PALSGD_INNER_ADAMW;
    float* m = c->moments_shared && K > 1 ? c->buf.M : nullptr;
    float* v = m && adamw ? c->buf.V : nullptr;
    float* x = c->model_shared ? c->buf.X : nullptr;
    if (m || x) {
        const uint32_t bytes = ((m ? (adamw ? 8u : 4u) : 0u) + (x ? 4u : 0u)) * K * kTile;
        warmup_broadcast_kernel<<<tile_count(c), kWave, lds_cap(auto_waves(bytes, 4), 0), st>>>(
            m, v, x, c->buf.XG, c->P_padded, c->buf.row_stride, K);
        palsgd_status rc = check_launch(c, who);
        if (rc != PALSGD_OK) return rc;
    }
    c->moments_shared = false;
    c->model_shared = false;
    return PALSGD_OK;
}

void dispatch_step(palsgd_ctx* c, const StepArgs& args, const Slot* dev_slots, uint32_t n_slots, bool any_grad,
                   const float* clip, hipStream_t st) {
    const bool adamw = c->cfg.inner == PALSGD_INNER_ADAMW, bf16 = c->cfg.grad_dtype == PALSGD_GRAD_BF16;
    if (adamw && bf16) launch_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_BF16>(c, args, dev_slots, n_slots, any_grad, clip, st);
    else if (adamw) launch_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_F32>(c, args, dev_slots, n_slots, any_grad, clip, st);
    else if (bf16) launch_step<PALSGD_INNER_SGDM, PALSGD_GRAD_BF16>(c, args, dev_slots, n_slots, any_grad, clip, st);
    else launch_step<PALSGD_INNER_SGDM, PALSGD_GRAD_F32>(c, args, dev_slots, n_slots, any_grad, clip, st);
}

// Argument checks and per-slot scalars of step t for the replicas that take a requested branch.
// Nothing is launched and no state is changed here.
palsgd_status plan_slots(palsgd_ctx* c, const char* who, uint64_t t, float alpha, float eta, const float* grad_scale,
                         const uint8_t* mask_override, bool do_grad, bool do_mix, StepArgs& args, uint32_t& n,
                         bool stepped[PALSGD_MAX_K]) {
    if (!c) {
        set_error(g_error, "%s: NULL context", who);
        return PALSGD_EINVAL;
    }
    if (c->capturable) {
        set_error(c->error, "%s: the schedule is device-resident (palsgd_capturable_begin); use "
                            "palsgd_step_capturable or call palsgd_capturable_end first", who);
        return PALSGD_ESTATE;
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
    n = 0;
    for (uint32_t k = 0; k < PALSGD_MAX_K; ++k) stepped[k] = false;
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
    return PALSGD_OK;
}

// Shared body of palsgd_inner_step / palsgd_pseudo_sync / palsgd_step.
palsgd_status local_update(palsgd_ctx* c, const char* who, uint64_t t, float alpha, float eta,
                           const float* grad_scale, const uint8_t* mask_override, bool do_grad, bool do_mix,
                           void* stream) {
    StepArgs args;
    uint32_t n = 0;
    bool stepped[PALSGD_MAX_K];
    palsgd_status rc = plan_slots(c, who, t, alpha, eta, grad_scale, mask_override, do_grad, do_mix, args, n, stepped);
    if (rc != PALSGD_OK) return rc;
    if (n == 0) {
        if (do_grad) c->clip_armed = false;  // the scales belonged to this step's gradients, which nobody used
        return PALSGD_OK;
    }
    const uint32_t K = c->cfg.K;
    bool any_grad = false;
    for (uint32_t k = 0; k < K; ++k) any_grad = any_grad || stepped[k];
    hipStream_t st = (hipStream_t)stream;
    rc = begin_launches(c, who);
    if (rc != PALSGD_OK) return rc;
    rc = end_warmup_sharing(c, who, st);  // every worker needs its own model row and InnerOPT state from here on
    if (rc != PALSGD_OK) return rc;
    // clipping scales computed by palsgd_clip_grad_norm are consumed by the first gradient step after it
    const float* clip = any_grad && c->clip_armed ? clip_scales(c) : nullptr;
    dispatch_step(c, args, nullptr, n, any_grad, clip, st);
    rc = check_launch(c, who);
    if (rc != PALSGD_OK) return rc;
    if (do_grad) c->clip_armed = false;  // also when every worker mixed: the scales are this step's, not the next one's
    for (uint32_t k = 0; k < K; ++k)
        if (stepped[k]) c->tau[k] += 1;
    return PALSGD_OK;
}

template <int INNER, int GDT>
void launch_sync_step(palsgd_ctx* c, const StepArgs& args, const float* clip, const OuterArgs& a, hipStream_t st) {
    const uint32_t K = c->cfg.K;
    // Resident wavefronts per CU, from sweeps of this kernel: 4-6 for AdamW at K <= 8 (two batches of four
    // replicas per wavefront), 8-10 from K = 16 up, 8-12 for SGD-momentum.
    (void)GDT;
    const uint32_t best = INNER == PALSGD_INNER_ADAMW ? (K <= 8 ? 6u : 8u) : 10u;
    const uint32_t waves = c->outer_waves ? c->outer_waves : best;
    Hyper h = hyper_of(c);
    const palsgd_buffers& b = c->buf;
    const uint32_t lds = lds_cap(waves, 0);
    const bool oadam = c->cfg.outer_opt == PALSGD_OUTER_ADAMW;
    const bool split = restart_apart(c);
#define PALSGD_SYNC(TAB, OADAM, tab)                                                                               \
    if (split)                                                                                                     \
        sync_step_kernel<INNER, GDT, TAB, OADAM, false><<<tile_count(c), kWave, lds, st>>>(                        \
            args, tab, b.X, b.M, b.V, b.G, b.XG, b.OM, b.OV, clip, c->P_padded, b.row_stride, K, h, a);            \
    else                                                                                                           \
        sync_step_kernel<INNER, GDT, TAB, OADAM, true><<<tile_count(c), kWave, lds, st>>>(                         \
            args, tab, b.X, b.M, b.V, b.G, b.XG, b.OM, b.OV, clip, c->P_padded, b.row_stride, K, h, a)
    if (c->wd_uniform && !oadam) { PALSGD_SYNC(false, false, nullptr); }
    else if (c->wd_uniform) { PALSGD_SYNC(false, true, nullptr); }
    else if (!oadam) { PALSGD_SYNC(true, false, c->d_wd_tab); }
    else { PALSGD_SYNC(true, true, c->d_wd_tab); }
#undef PALSGD_SYNC
    if (split) launch_restart_rows(c, st);
}

}  // namespace

extern "C" {

palsgd_status palsgd_layout(const palsgd_config* cfg, uint64_t* P_padded, uint64_t* tensor_offset) {
    if (!cfg) {
        set_error(g_error, "palsgd_layout: NULL config");
        return PALSGD_EINVAL;
    }
    return layout_impl(cfg->n_tensors, cfg->tensor_numel, cfg->P, P_padded, tensor_offset, g_error);
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
    palsgd_status rc = layout_impl(cfg->n_tensors, cfg->tensor_numel, cfg->P, &P_padded, offs.data(), g_error);
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
        // > 0: the padding between tensors holds g = m = v = 0 and must stay 0, not become 0/0
        PALSGD_REQUIRE(std::isfinite(cfg->eps) && cfg->eps > 0.0f, "eps must be finite, > 0");
        PALSGD_REQUIRE(buf->V != nullptr, "V buffer is required by AdamW");
    } else {
        PALSGD_REQUIRE(std::isfinite(cfg->momentum) && cfg->momentum >= 0.0f && cfg->momentum < 1.0f,
                       "momentum must satisfy 0 <= momentum < 1");
    }
    PALSGD_REQUIRE(std::isfinite(cfg->outer_lr) && cfg->outer_lr >= 0.0f, "outer_lr must be finite, >= 0");
    PALSGD_REQUIRE(std::isfinite(cfg->outer_momentum) && cfg->outer_momentum >= 0.0f && cfg->outer_momentum < 1.0f,
                   "outer_momentum must satisfy 0 <= outer_momentum < 1");
    PALSGD_REQUIRE(cfg->outer_opt == PALSGD_OUTER_SGD || cfg->outer_opt == PALSGD_OUTER_ADAMW, "unknown outer optimizer");
    if (cfg->outer_opt == PALSGD_OUTER_ADAMW) {
        PALSGD_REQUIRE(cfg->outer_beta1 >= 0.0f && cfg->outer_beta1 < 1.0f, "outer_beta1 must satisfy 0 <= outer_beta1 < 1");
        PALSGD_REQUIRE(cfg->outer_beta2 >= 0.0f && cfg->outer_beta2 < 1.0f, "outer_beta2 must satisfy 0 <= outer_beta2 < 1");
        PALSGD_REQUIRE(std::isfinite(cfg->outer_eps) && cfg->outer_eps > 0.0f, "outer_eps must be finite, > 0");
        PALSGD_REQUIRE(std::isfinite(cfg->outer_weight_decay) && cfg->outer_weight_decay >= 0.0f,
                       "outer_weight_decay must be finite, >= 0");
        PALSGD_REQUIRE(buf->OV != nullptr && aligned16(buf->OV), "OV buffer (16-byte aligned) is required by OuterOPT = AdamW");
    }
    PALSGD_REQUIRE(buf->X && buf->M && buf->G && buf->XG && buf->OM, "NULL device buffer");
    PALSGD_REQUIRE(aligned16(buf->X) && aligned16(buf->M) && aligned16(buf->V) && aligned16(buf->G) &&
                       aligned16(buf->XG) && aligned16(buf->OM) && aligned16(x0_dev),
                   "device buffers must be 16-byte aligned");
    PALSGD_REQUIRE(buf->row_stride >= P_padded && buf->row_stride % 64 == 0,
                   "row_stride must be a multiple of 64 and >= the padded row length");
    PALSGD_REQUIRE(P_padded <= kMaxRow, "a row may hold at most 2^33 elements (one lane per four elements in one launch dimension)");
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
    for (float m : c->wd_mult) c->wd_uniform = c->wd_uniform && m == c->wd_mult[0];
    if (cfg->weight_decay == 0.0f) c->wd_uniform = true;  // the multipliers multiply zero
    c->wd_eff0 = (float)((double)cfg->weight_decay * (double)c->wd_mult[0]);
    c->draw_threshold = (uint32_t)std::floor(cfg->p * 16777216.0);
    // all device memory of the library is allocated here, never at first use: any later call may be the
    // first one inside a stream capture, or come from a caller that must not allocate
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) {
        // no GPU: the context still answers palsgd_draw and the scalar state calls (what the host-side
        // checks of this library use); every call that would launch returns PALSGD_EHIP
        (void)hipGetLastError();
        c->host_only = true;
    } else {
        rc = c->wd_uniform ? PALSGD_OK : build_wd_table(c);
        if (rc == PALSGD_OK) rc = alloc_device_state(c);
        if (rc == PALSGD_OK) rc = static_scratch(c->error, nullptr);  // set-up of palsgd_clip_grad_norm_noalloc
        if (rc != PALSGD_OK) {
            memcpy(g_error, c->error, sizeof g_error);
            palsgd_destroy(c);
            return rc;
        }
        (void)lds_per_cu();  // the device attribute query happens here as well
    }
    if (x0_dev) {
        uint64_t n4 = P_padded / 4;
        uint32_t blocks = (uint32_t)((n4 + kThreads - 1) / kThreads);
        rc = begin_launches(c, "palsgd_init");
        if (rc == PALSGD_OK)
            init_kernel<<<blocks, kThreads, 0, (hipStream_t)stream>>>(x0_dev, buf->X, buf->M, buf->V, buf->XG, buf->OM,
                                                                  cfg->outer_opt == PALSGD_OUTER_ADAMW ? buf->OV : nullptr, n4,
                                                                  buf->row_stride, cfg->K);
        if (rc == PALSGD_OK) rc = check_launch(c, "palsgd_init");
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

palsgd_status palsgd_step_sync(palsgd_ctx* ctx, uint64_t t, float alpha_t, float eta_t, const float* grad_scale,
                               const uint8_t* mask_override, void* stream) {
    StepArgs args;
    uint32_t n = 0;
    bool stepped[PALSGD_MAX_K];
    palsgd_status rc =
        plan_slots(ctx, "palsgd_step_sync", t, alpha_t, eta_t, grad_scale, mask_override, true, true, args, n, stepped);
    if (rc != PALSGD_OK) return rc;
    const uint32_t K = ctx->cfg.K;  // both branches requested: n == K and slot s is replica s
    bool any_grad = false;
    for (uint32_t k = 0; k < K; ++k) any_grad = any_grad || stepped[k];
    hipStream_t st = (hipStream_t)stream;
    rc = begin_launches(ctx, "palsgd_step_sync");
    if (rc == PALSGD_OK) rc = refuse_captured_outer_adamw(ctx, "palsgd_step_sync", st);
    if (rc != PALSGD_OK) return rc;
    rc = end_warmup_sharing(ctx, "palsgd_step_sync", st);
    if (rc != PALSGD_OK) return rc;
    const float* clip = any_grad && ctx->clip_armed ? clip_scales(ctx) : nullptr;
    const OuterArgs a = outer_args_of(ctx);
    const bool adamw = ctx->cfg.inner == PALSGD_INNER_ADAMW, bf16 = ctx->cfg.grad_dtype == PALSGD_GRAD_BF16;
    if (adamw && bf16) launch_sync_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_BF16>(ctx, args, clip, a, st);
    else if (adamw) launch_sync_step<PALSGD_INNER_ADAMW, PALSGD_GRAD_F32>(ctx, args, clip, a, st);
    else if (bf16) launch_sync_step<PALSGD_INNER_SGDM, PALSGD_GRAD_BF16>(ctx, args, clip, a, st);
    else launch_sync_step<PALSGD_INNER_SGDM, PALSGD_GRAD_F32>(ctx, args, clip, a, st);
    rc = check_launch(ctx, "palsgd_step_sync");
    if (rc != PALSGD_OK) return rc;
    ctx->clip_armed = false;
    for (uint32_t k = 0; k < K; ++k)
        if (stepped[k]) ctx->tau[k] += 1;
    ctx->n_outer += 1;
    ctx->last_outer_t = t;
    return PALSGD_OK;
}

static palsgd_status outer_impl(palsgd_ctx* ctx, const char* who, uint64_t t, float* diag_out_dev, void* stream) {
    if (!ctx) {
        set_error(g_error, "%s: NULL context", who);
        return PALSGD_EINVAL;
    }
    const uint32_t K = ctx->cfg.K;
    const OuterArgs a = outer_args_of(ctx);
    const uint64_t n = ctx->P_padded;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t variant = ctx->outer_variant ? ctx->outer_variant : 1u;
    // One launch (rows go 8 at a time; 4 resident wavefronts per CU are best from K = 16 up), or, for many workers
    // and a global model that fits the memory-side cache (restart_apart; or variant 3), two: the reduction with
    // OuterOPT, 6 wavefronts per CU, then the restart of the rows.
    const bool split = restart_apart(ctx);
    const uint32_t waves = ctx->outer_waves ? ctx->outer_waves : (split ? 6u : auto_waves((8u * K + 16u) * kTile, 4));
    const palsgd_buffers& b = ctx->buf;
    const bool oadam = ctx->cfg.outer_opt == PALSGD_OUTER_ADAMW;
    {
        palsgd_status rc = begin_launches(ctx, who);
        if (rc == PALSGD_OK) rc = refuse_captured_outer_adamw(ctx, who, st);
        if (rc == PALSGD_OK) rc = end_warmup_sharing(ctx, who, st);  // the rows of X are read here
        if (rc != PALSGD_OK) return rc;
    }
    const uint32_t tiles = tile_count(ctx);
    const uint32_t lds = lds_cap(waves, 0);
    float* part = diag_out_dev ? scratch_partials(ctx) : nullptr;
    const uint32_t n_part = diag_out_dev ? tiles : 0u;
#define PALSGD_WALK(DIAG, OADAM)                                                                                      \
    if (split)                                                                                                        \
        outer_kernel_walk<DIAG, OADAM, false><<<tiles, kWave, lds, st>>>(b.X, b.XG, b.OM, b.OV, n, b.row_stride, K, a, part, n_part); \
    else                                                                                                              \
        outer_kernel_walk<DIAG, OADAM, true><<<tiles, kWave, lds, st>>>(b.X, b.XG, b.OM, b.OV, n, b.row_stride, K, a, part, n_part)
    if (diag_out_dev) {
        if (oadam) { PALSGD_WALK(true, true); }
        else { PALSGD_WALK(true, false); }
        fold_kernel<<<dim3(kFold, 2), kThreads, 0, st>>>(scratch_partials(ctx), tiles, scratch_fold(ctx));
        diag_finish_kernel<<<1, kThreads, 0, st>>>(scratch_fold(ctx), a.inv_k, diag_out_dev);
    } else if (variant == 2) {
        const uint64_t n4 = n / 4;
        uint32_t blocks = (uint32_t)((n4 + 255) / 256);
        uint32_t groups = waves / 4 ? waves / 4 : 1;  // a workgroup of this variant is four wavefronts
        if (oadam)
            outer_kernel_lds<true><<<blocks, kThreads, lds_cap(groups, 16384), st>>>(b.X, b.XG, b.OM, b.OV, n4, b.row_stride, K, a);
        else
            outer_kernel_lds<false><<<blocks, kThreads, lds_cap(groups, 16384), st>>>(b.X, b.XG, b.OM, b.OV, n4, b.row_stride, K, a);
    } else if (oadam) {
        PALSGD_WALK(false, true);
    } else {
        PALSGD_WALK(false, false);
    }
#undef PALSGD_WALK
    if (split) launch_restart_rows(ctx, st);
    palsgd_status rc = check_launch(ctx, who);
    if (rc != PALSGD_OK) return rc;
    ctx->n_outer += 1;
    ctx->last_outer_t = t;
    return PALSGD_OK;
}

palsgd_status palsgd_outer_step(palsgd_ctx* ctx, uint64_t t, void* stream) {
    return outer_impl(ctx, "palsgd_outer_step", t, nullptr, stream);
}

palsgd_status palsgd_outer_step_diag(palsgd_ctx* ctx, uint64_t t, float* diag_out_dev, void* stream) {
    if (ctx && !diag_out_dev) {
        set_error(ctx->error, "palsgd_outer_step_diag: NULL output");
        return PALSGD_EINVAL;
    }
    return outer_impl(ctx, "palsgd_outer_step_diag", t, diag_out_dev, stream);
}

static palsgd_status ddp_impl(palsgd_ctx* ctx, const char* who, float alpha_t, const float* grad_scale, bool share_model,
                              void* stream) {
    if (!ctx) {
        set_error(g_error, "%s: NULL context", who);
        return PALSGD_EINVAL;
    }
    if (!(alpha_t >= 0.0f) || !std::isfinite(alpha_t)) {
        set_error(ctx->error, "%s: alpha_t must be finite and >= 0", who);
        return PALSGD_EINVAL;
    }
    if (ctx->capturable) {
        set_error(ctx->error, "%s: not available while the schedule is device-resident", who);
        return PALSGD_ESTATE;
    }
    const uint32_t K = ctx->cfg.K;
    for (uint32_t k = 1; k < K; ++k)
        if (ctx->tau[k] != ctx->tau[0]) {
            set_error(ctx->error, "%s: workers have taken different numbers of gradient steps "
                                  "(%llu vs %llu): the DDP step needs identical workers",
                      who, (unsigned long long)ctx->tau[0], (unsigned long long)ctx->tau[k]);
            return PALSGD_ESTATE;
        }
    DdpArgs a;
    for (uint32_t k = 0; k < PALSGD_MAX_K; ++k) a.w[k] = 1.0f;
    if (grad_scale)
        for (uint32_t k = 0; k < K; ++k) {
            if (!std::isfinite(grad_scale[k])) {
                set_error(ctx->error, "%s: grad_scale[%u] is not finite", who, k);
                return PALSGD_EINVAL;
            }
            a.w[k] = grad_scale[k];
        }
    const double tau = (double)(ctx->tau[0] + 1);
    a.inv_k = (float)(1.0 / (double)K);
    a.lr = alpha_t;  // DDP has no mixing branch, so no 1/(1-p) rescale
    a.c1 = a.c2 = 0.0f;
    const bool adamw = ctx->cfg.inner == PALSGD_INNER_ADAMW, bf16 = ctx->cfg.grad_dtype == PALSGD_GRAD_BF16;
    if (adamw) {
        a.c1 = (float)((double)alpha_t / (1.0 - std::pow((double)ctx->cfg.beta1, tau)));
        a.c2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)ctx->cfg.beta2, tau)));
    }
    const uint64_t n = ctx->P_padded;
    const uint32_t tiles = (uint32_t)((n + kTile - 1) / kTile);
    // rows of X this launch stores: all K, or none when the model stays shared (it is then XG alone) and when
    // the rows are many enough for a restart launch of their own to be faster (as in the outer step)
    const bool rows_apart = !share_model && restart_apart(ctx);
    const uint32_t x_rows = share_model || rows_apart ? 0u : K;
    const uint32_t per_elem = (adamw ? 24u : 16u) + 4u * x_rows + K * (bf16 ? 2u : 4u);
    const uint32_t lds = lds_cap(ctx->outer_waves ? ctx->outer_waves : auto_waves(per_elem * kTile, 4), 0);
    Hyper h = hyper_of(ctx);
    hipStream_t st = (hipStream_t)stream;
    const palsgd_buffers& b = ctx->buf;
    const float* clip = ctx->clip_mean_armed ? mean_clip_scale(ctx) : nullptr;
    {
        palsgd_status rc = begin_launches(ctx, who);
        if (rc != PALSGD_OK) return rc;
    }
#define PALSGD_DDP(I, D)                                                                                           \
    if (ctx->wd_uniform)                                                                                           \
        ddp_kernel<I, D, false><<<tiles, kWave, lds, st>>>(a, nullptr, b.X, b.M, b.V, b.G, b.XG, clip, n, b.row_stride, K, x_rows, h); \
    else                                                                                                           \
        ddp_kernel<I, D, true><<<tiles, kWave, lds, st>>>(a, ctx->d_wd_tab, b.X, b.M, b.V, b.G, b.XG, clip, n, b.row_stride, K, x_rows, h);
    if (adamw && bf16) { PALSGD_DDP(PALSGD_INNER_ADAMW, PALSGD_GRAD_BF16) }
    else if (adamw) { PALSGD_DDP(PALSGD_INNER_ADAMW, PALSGD_GRAD_F32) }
    else if (bf16) { PALSGD_DDP(PALSGD_INNER_SGDM, PALSGD_GRAD_BF16) }
    else { PALSGD_DDP(PALSGD_INNER_SGDM, PALSGD_GRAD_F32) }
#undef PALSGD_DDP
    if (rows_apart) launch_restart_rows(ctx, st);
    palsgd_status rc = check_launch(ctx, who);
    if (rc != PALSGD_OK) return rc;
    for (uint32_t k = 0; k < K; ++k) ctx->tau[k] += 1;
    ctx->moments_shared = true;
    ctx->model_shared = share_model;  // a step that stores all K rows also ends an earlier sharing of the model
    ctx->clip_mean_armed = false;
    return PALSGD_OK;
}

palsgd_status palsgd_ddp_step(palsgd_ctx* ctx, uint64_t t, float alpha_t, const float* grad_scale, void* stream) {
    (void)t;
    return ddp_impl(ctx, "palsgd_ddp_step", alpha_t, grad_scale, false, stream);
}

palsgd_status palsgd_ddp_step_shared(palsgd_ctx* ctx, uint64_t t, float alpha_t, const float* grad_scale, void* stream) {
    (void)t;
    return ddp_impl(ctx, "palsgd_ddp_step_shared", alpha_t, grad_scale, true, stream);
}

palsgd_status palsgd_ddp_finish(palsgd_ctx* ctx, void* stream) {
    if (!ctx) {
        set_error(g_error, "palsgd_ddp_finish: NULL context");
        return PALSGD_EINVAL;
    }
    palsgd_status rc = begin_launches(ctx, "palsgd_ddp_finish");
    return rc != PALSGD_OK ? rc : end_warmup_sharing(ctx, "palsgd_ddp_finish", (hipStream_t)stream);
}

// Shared body of palsgd_clip_grad_norm and palsgd_clip_grad_norm_noalloc: `partial` holds K * norm_parts floats
// and `fold` K * kFold doubles; the scales go to the context's own memory in both cases.
static palsgd_status clip_norm_launches(palsgd_ctx* ctx, const char* who, float max_norm, float* norms_out_dev,
                                        float* partial, double* fold, hipStream_t st) {
    const uint32_t K = ctx->cfg.K, per_row = norm_parts(ctx);
    dim3 grid(per_row, K);
    if (ctx->cfg.grad_dtype == PALSGD_GRAD_BF16)
        sumsq_kernel<PALSGD_GRAD_BF16><<<grid, kWave, lds_cap(16, 0), st>>>(ctx->buf.G, partial, ctx->P_padded,
                                                                           ctx->buf.row_stride, per_row);
    else
        sumsq_kernel<PALSGD_GRAD_F32><<<grid, kWave, lds_cap(16, 0), st>>>(ctx->buf.G, partial, ctx->P_padded,
                                                                          ctx->buf.row_stride, per_row);
    fold_kernel<<<dim3(kFold, K), kThreads, 0, st>>>(partial, per_row, fold);
    clip_finish_kernel<<<K, kThreads, 0, st>>>(fold, max_norm, clip_scales(ctx), norms_out_dev);
    palsgd_status rc = check_launch(ctx, who);
    if (rc != PALSGD_OK) return rc;
    ctx->clip_armed = true;
    return PALSGD_OK;
}

static palsgd_status clip_norm_checks(palsgd_ctx* ctx, const char* who, float max_norm) {
    if (!ctx) {
        set_error(g_error, "%s: NULL context", who);
        return PALSGD_EINVAL;
    }
    if (!(max_norm > 0.0f) || !std::isfinite(max_norm)) {
        set_error(ctx->error, "%s: max_norm must be finite and > 0", who);
        return PALSGD_EINVAL;
    }
    return PALSGD_OK;
}

palsgd_status palsgd_clip_grad_norm(palsgd_ctx* ctx, float max_norm, float* norms_out_dev, void* stream) {
    palsgd_status rc = clip_norm_checks(ctx, "palsgd_clip_grad_norm", max_norm);
    if (rc == PALSGD_OK) rc = begin_launches(ctx, "palsgd_clip_grad_norm");
    if (rc != PALSGD_OK) return rc;
    return clip_norm_launches(ctx, "palsgd_clip_grad_norm", max_norm, norms_out_dev, scratch_partials(ctx),
                              scratch_fold(ctx), (hipStream_t)stream);
}

palsgd_status palsgd_clip_grad_norm_noalloc(palsgd_ctx* ctx, float max_norm, float* norms_out_dev, void* stream) {
    const char* who = "palsgd_clip_grad_norm_noalloc";
    palsgd_status rc = clip_norm_checks(ctx, who, max_norm);
    if (rc != PALSGD_OK) return rc;
    const uint64_t parts = (uint64_t)ctx->cfg.K * norm_parts(ctx);
    if (parts > kStaticMaxParts) {
        set_error(ctx->error, "%s: K * ceil(P_padded / %d) = %llu partial sums, the static scratch holds %u; use "
                              "palsgd_clip_grad_norm", who, kTile * kNormTiles, (unsigned long long)parts, kStaticMaxParts);
        return PALSGD_EINVAL;
    }
    rc = begin_launches(ctx, who);
    if (rc != PALSGD_OK) return rc;
    float* base = nullptr;  // the array's device address on the current device, never the array's name
    rc = static_scratch(ctx->error, &base);
    if (rc != PALSGD_OK) return rc;
    // nothing needs clearing: the launches overwrite every partial sum and every second-stage sum they read
    return clip_norm_launches(ctx, who, max_norm, norms_out_dev, base + kStaticFoldFloats, (double*)base,
                              (hipStream_t)stream);
}

palsgd_status palsgd_clip_mean_grad_norm(palsgd_ctx* ctx, float max_norm, const float* grad_scale,
                                         float* norm_out_dev, void* stream) {
    if (!ctx) {
        set_error(g_error, "palsgd_clip_mean_grad_norm: NULL context");
        return PALSGD_EINVAL;
    }
    if (!(max_norm > 0.0f) || !std::isfinite(max_norm)) {
        set_error(ctx->error, "palsgd_clip_mean_grad_norm: max_norm must be finite and > 0");
        return PALSGD_EINVAL;
    }
    const uint32_t K = ctx->cfg.K;
    DdpArgs a;
    for (uint32_t k = 0; k < PALSGD_MAX_K; ++k) a.w[k] = 1.0f;
    if (grad_scale)
        for (uint32_t k = 0; k < K; ++k) {
            if (!std::isfinite(grad_scale[k])) {
                set_error(ctx->error, "palsgd_clip_mean_grad_norm: grad_scale[%u] is not finite", k);
                return PALSGD_EINVAL;
            }
            a.w[k] = grad_scale[k];
        }
    a.inv_k = (float)(1.0 / (double)K);
    a.lr = a.c1 = a.c2 = 0.0f;
    palsgd_status rc;
    const uint64_t span = (uint64_t)kTile * kMeanTiles;
    const uint32_t parts = (uint32_t)((ctx->P_padded + span - 1) / span);
    const uint32_t gbytes = ctx->cfg.grad_dtype == PALSGD_GRAD_BF16 ? 2u : 4u;
    // a wavefront has at most eight row loads in flight at a time: size the cap on those
    const uint32_t lds = lds_cap(auto_waves(gbytes * (K < 8 ? K : 8u) * kTile, 4), 0);
    hipStream_t st = (hipStream_t)stream;
    rc = begin_launches(ctx, "palsgd_clip_mean_grad_norm");
    if (rc != PALSGD_OK) return rc;
    if (ctx->cfg.grad_dtype == PALSGD_GRAD_BF16)
        sumsq_mean_kernel<PALSGD_GRAD_BF16><<<parts, kWave, lds, st>>>(ctx->buf.G, a, scratch_partials(ctx),
                                                                      ctx->P_padded, ctx->buf.row_stride, K);
    else
        sumsq_mean_kernel<PALSGD_GRAD_F32><<<parts, kWave, lds, st>>>(ctx->buf.G, a, scratch_partials(ctx),
                                                                     ctx->P_padded, ctx->buf.row_stride, K);
    fold_kernel<<<dim3(kFold, 1), kThreads, 0, st>>>(scratch_partials(ctx), parts, scratch_fold(ctx));
    clip_finish_kernel<<<1, kThreads, 0, st>>>(scratch_fold(ctx), max_norm, mean_clip_scale(ctx), norm_out_dev);
    rc = check_launch(ctx, "palsgd_clip_mean_grad_norm");
    if (rc != PALSGD_OK) return rc;
    ctx->clip_mean_armed = true;
    return PALSGD_OK;
}

palsgd_status palsgd_diagnostics(palsgd_ctx* ctx, float* out_dev, void* stream) {
    if (!ctx || !out_dev) {
        set_error(ctx ? ctx->error : g_error, "palsgd_diagnostics: NULL argument");
        return PALSGD_EINVAL;
    }
    palsgd_status rc;
    const uint32_t K = ctx->cfg.K, n_part = diag_parts(ctx);
    const float inv_k = (float)(1.0 / (double)K);
    hipStream_t st = (hipStream_t)stream;
    rc = begin_launches(ctx, "palsgd_diagnostics");
    if (rc != PALSGD_OK) return rc;
    rc = end_warmup_sharing(ctx, "palsgd_diagnostics", st);  // the rows of X are read here
    if (rc != PALSGD_OK) return rc;
    diag_kernel<<<n_part, kWave, 0, st>>>(ctx->buf.X, ctx->buf.XG, scratch_partials(ctx), ctx->P_padded,
                                          ctx->buf.row_stride, K, inv_k, n_part);
    fold_kernel<<<dim3(kFold, 2), kThreads, 0, st>>>(scratch_partials(ctx), n_part, scratch_fold(ctx));
    diag_finish_kernel<<<1, kThreads, 0, st>>>(scratch_fold(ctx), inv_k, out_dev);
    return check_launch(ctx, "palsgd_diagnostics");
}

palsgd_status palsgd_capturable_begin(palsgd_ctx* ctx, uint64_t t0, void* stream) {
    if (!ctx) {
        set_error(g_error, "palsgd_capturable_begin: NULL context");
        return PALSGD_EINVAL;
    }
    if (ctx->capturable) {
        set_error(ctx->error, "palsgd_capturable_begin: the schedule is already device-resident; call "
                              "palsgd_capturable_end first");
        return PALSGD_ESTATE;
    }
    {
        palsgd_status rc = begin_launches(ctx, "palsgd_capturable_begin");
        if (rc == PALSGD_OK) rc = end_warmup_sharing(ctx, "palsgd_capturable_begin", (hipStream_t)stream);
        if (rc != PALSGD_OK) return rc;
    }
    TauArgs a;
    for (uint32_t k = 0; k < PALSGD_MAX_K; ++k) a.tau[k] = k < ctx->cfg.K ? ctx->tau[k] : 0;
    schedule_set_kernel<<<1, kWave, 0, (hipStream_t)stream>>>((DevSchedule*)ctx->d_schedule, t0, a);
    palsgd_status rc = check_launch(ctx, "palsgd_capturable_begin");
    if (rc != PALSGD_OK) return rc;
    ctx->capturable = true;
    return PALSGD_OK;
}

palsgd_status palsgd_step_capturable(palsgd_ctx* ctx, const float* alpha_eta_dev, void* stream) {
    if (!ctx || !alpha_eta_dev) {
        set_error(ctx ? ctx->error : g_error, "palsgd_step_capturable: NULL argument");
        return PALSGD_EINVAL;
    }
    if (!ctx->capturable) {
        set_error(ctx->error, "palsgd_step_capturable: call palsgd_capturable_begin first");
        return PALSGD_ESTATE;
    }
    hipStream_t st = (hipStream_t)stream;
    {
        palsgd_status rc = begin_launches(ctx, "palsgd_step_capturable");
        if (rc != PALSGD_OK) return rc;
    }
    DevSchedule* ds = (DevSchedule*)ctx->d_schedule;
    PlanArgs a{ctx->cfg.seed, ctx->cfg.p, (double)ctx->cfg.beta1, (double)ctx->cfg.beta2, ctx->cfg.K,
               ctx->draw_threshold, ctx->cfg.inner == PALSGD_INNER_ADAMW ? 1u : 0u};
    plan_kernel<<<1, kWave, 0, st>>>(ds, alpha_eta_dev, a);
    StepArgs none;
    memset(&none, 0, sizeof none);
    const float* clip = ctx->clip_armed ? clip_scales(ctx) : nullptr;
    dispatch_step(ctx, none, ds->slot, ctx->cfg.K, true, clip, st);
    palsgd_status rc = check_launch(ctx, "palsgd_step_capturable");
    if (rc != PALSGD_OK) return rc;
    ctx->clip_armed = false;
    return PALSGD_OK;
}

palsgd_status palsgd_capturable_end(palsgd_ctx* ctx, uint64_t* t_out, void* stream) {
    if (!ctx) {
        set_error(g_error, "palsgd_capturable_end: NULL context");
        return PALSGD_EINVAL;
    }
    if (!ctx->capturable) {
        set_error(ctx->error, "palsgd_capturable_end: not in capturable mode");
        return PALSGD_ESTATE;
    }
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    uint64_t host[1 + PALSGD_MAX_K];
    if (e == hipSuccess) e = hipMemcpy(host, ctx->d_schedule, sizeof host, hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        set_error(ctx->error, "palsgd_capturable_end: %s", hipGetErrorString(e));
        return PALSGD_EHIP;
    }
    for (uint32_t k = 0; k < ctx->cfg.K; ++k) ctx->tau[k] = host[1 + k];
    if (t_out) *t_out = host[0];
    ctx->capturable = false;
    return PALSGD_OK;
}

palsgd_status palsgd_get_state(const palsgd_ctx* ctx, uint64_t* tau, uint64_t* n_outer) {
    if (!ctx) {
        set_error(g_error, "palsgd_get_state: NULL context");
        return PALSGD_EINVAL;
    }
    if (ctx->capturable) {
        set_error(ctx->error, "palsgd_get_state: the step counts are on the device; call palsgd_capturable_end first");
        return PALSGD_ESTATE;
    }
    if (ctx->moments_shared || ctx->model_shared) {
        // what a checkpoint would save next to these counts is not there yet: rows 1..K-1 of M, V (and the rows of
        // X after palsgd_ddp_step_shared) are stale until the warm-up's broadcast has run
        set_error(ctx->error, "palsgd_get_state: DDP warm-up steps left the workers' rows shared; call "
                              "palsgd_ddp_finish before saving state");
        return PALSGD_ESTATE;
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
    if (ctx->capturable) {
        set_error(ctx->error, "palsgd_set_state: the step counts are on the device; call palsgd_capturable_end first");
        return PALSGD_ESTATE;
    }
    memcpy(ctx->tau, tau, ctx->cfg.K * sizeof(uint64_t));
    ctx->n_outer = n_outer;
    return PALSGD_OK;
}

const char* palsgd_last_error(const palsgd_ctx* ctx) { return ctx ? ctx->error : g_error; }

void palsgd_destroy(palsgd_ctx* ctx) {
    if (!ctx) return;
    if (ctx->d_wd_tab) (void)hipFree(ctx->d_wd_tab);
    if (ctx->d_scratch) (void)hipFree(ctx->d_scratch);
    if (ctx->d_schedule) (void)hipFree(ctx->d_schedule);
    delete ctx;
}

palsgd_status palsgd_set_outer_lr(palsgd_ctx* ctx, float outer_lr) {
    if (!ctx) {
        set_error(g_error, "palsgd_set_outer_lr: NULL context");
        return PALSGD_EINVAL;
    }
    if (!std::isfinite(outer_lr) || !(outer_lr >= 0.0f)) {
        set_error(ctx->error, "palsgd_set_outer_lr: outer_lr must be finite and >= 0");
        return PALSGD_EINVAL;
    }
    ctx->cfg.outer_lr = outer_lr;
    return PALSGD_OK;
}

palsgd_status palsgd_set_tuning(palsgd_ctx* ctx, uint32_t step_waves_per_cu, uint32_t outer_waves_per_cu,
                                uint32_t outer_variant) {
    if (!ctx) {
        set_error(g_error, "palsgd_set_tuning: NULL context");
        return PALSGD_EINVAL;
    }
    auto bad = [](uint32_t w) { return w != 0 && (w < 3 || w > 32); };
    if (bad(step_waves_per_cu) || bad(outer_waves_per_cu) || outer_variant > 3) {
        set_error(ctx->error, "palsgd_set_tuning: waves per CU must be 0 or 3..32, outer_variant 0..3");
        return PALSGD_EINVAL;
    }
    ctx->step_waves = step_waves_per_cu;
    ctx->outer_waves = outer_waves_per_cu;
    ctx->outer_variant = outer_variant;
    return PALSGD_OK;
}

}  // extern "C"
