// Host half of the PALSGD library (layout, argument checks, per-step planning, draws, scalar state) driven
// through the C ABI in a build whose host code carries AddressSanitizer and UndefinedBehaviorSanitizer.
// No device is needed: without one palsgd_init creates a context that answers the host-side calls and
// refuses every launch, which is also checked here.  Arrays handed to the library have exactly the size the
// header states, so a read past them is a sanitizer report.  Prints "host ok" at the end.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/palsgd.h"

#define REQUIRE(cond)                                                       \
    do {                                                                    \
        if (!(cond)) {                                                      \
            fprintf(stderr, "line %d: %s\n", __LINE__, #cond);              \
            return 1;                                                       \
        }                                                                   \
    } while (0)

static palsgd_config config(uint32_t K, const std::vector<uint64_t>& numel, const float* wdm, double p) {
    palsgd_config c;
    memset(&c, 0, sizeof c);
    c.K = K;
    c.n_tensors = (uint32_t)numel.size();
    c.tensor_numel = numel.data();
    c.tensor_wd_mult = wdm;
    c.inner = PALSGD_INNER_ADAMW;
    c.grad_dtype = PALSGD_GRAD_BF16;
    c.beta1 = 0.9f; c.beta2 = 0.999f; c.eps = 1e-8f; c.weight_decay = 0.01f; c.momentum = 0.9f;
    c.p = p; c.H = 4; c.outer_lr = 0.7f; c.outer_momentum = 0.9f; c.outer_nesterov = 1; c.seed = 42;
    return c;
}

int main() {
    float* fake = (float*)(uintptr_t)4096;  // aligned, never dereferenced: nothing is launched here
    // layouts: exact-size offset arrays, one tensor up to many
    for (uint32_t nt : {1u, 2u, 7u, 160u, 1000u}) {
        std::vector<uint64_t> numel(nt), offs(nt);
        for (uint32_t j = 0; j < nt; ++j) numel[j] = 1 + (j * 2654435761u) % 5000;
        palsgd_config c = config(4, numel, nullptr, 0.1);
        uint64_t P = 0;
        REQUIRE(palsgd_layout(&c, &P, offs.data()) == PALSGD_OK);
        REQUIRE(P % 256 == 0 && offs[0] == 0);
        for (uint32_t j = 1; j < nt; ++j) REQUIRE(offs[j] % 64 == 0 && offs[j] >= offs[j - 1] + numel[j - 1]);
        REQUIRE(palsgd_layout(&c, &P, nullptr) == PALSGD_OK);
        // context over that layout, with per-tensor multipliers of exactly nt entries
        std::vector<float> wdm(nt);
        for (uint32_t j = 0; j < nt; ++j) wdm[j] = (float)(j % 3) * 0.5f;
        c = config(4, numel, wdm.data(), 0.1);
        palsgd_buffers b;
        memset(&b, 0, sizeof b);
        b.X = b.M = b.V = b.XG = b.OM = fake; b.G = fake; b.row_stride = P;
        palsgd_ctx* ctx = nullptr;
        palsgd_status st = palsgd_init(&c, &b, nullptr, nullptr, &ctx);
        if (st != PALSGD_OK) { fprintf(stderr, "init: %s\n", palsgd_last_error(nullptr)); return 1; }
        palsgd_destroy(ctx);
    }
    // draws, state, argument errors of the step calls for every K
    for (uint32_t K : {1u, 2u, 3u, 8u, 33u, 64u}) {
        std::vector<uint64_t> numel = {100, 7};
        palsgd_config c = config(K, numel, nullptr, 0.25);
        palsgd_buffers b;
        memset(&b, 0, sizeof b);
        b.X = b.M = b.V = b.XG = b.OM = fake; b.G = fake; b.row_stride = 256;
        palsgd_ctx* ctx = nullptr;
        REQUIRE(palsgd_init(&c, &b, nullptr, nullptr, &ctx) == PALSGD_OK);
        std::vector<uint8_t> mask(K);
        unsigned mixed = 0;
        for (uint64_t t : {0ull, 1ull, 1000ull, 1ull << 40, ~0ull}) {
            REQUIRE(palsgd_draw(ctx, t, mask.data()) == PALSGD_OK);
            for (uint32_t k = 0; k < K; ++k) mixed += mask[k];
        }
        REQUIRE(mixed <= 5 * K);
        std::vector<uint64_t> tau(K), got(K);
        for (uint32_t k = 0; k < K; ++k) tau[k] = 5 + k;
        uint64_t n_outer = 0;
        REQUIRE(palsgd_set_state(ctx, tau.data(), 9) == PALSGD_OK);
        REQUIRE(palsgd_get_state(ctx, got.data(), &n_outer) == PALSGD_OK && n_outer == 9 && got == tau);
        std::vector<float> gs(K, 1.0f);
        std::vector<uint8_t> all_mix(K, 1), none_mix(K, 0);
        // argument errors come before any launch; a valid call is then refused because there is no device
        REQUIRE(palsgd_step(ctx, 0, -1.0f, 16.0f, gs.data(), nullptr, nullptr) == PALSGD_EINVAL);
        gs[K - 1] = 1.0f / 0.0f;
        REQUIRE(palsgd_inner_step(ctx, 0, 1e-3f, gs.data(), none_mix.data(), nullptr) == PALSGD_EINVAL);
        gs[K - 1] = 1.0f;
        REQUIRE(palsgd_inner_step(ctx, 0, 1e-3f, gs.data(), all_mix.data(), nullptr) == PALSGD_OK);  // nothing to do
        palsgd_status st = palsgd_step(ctx, 3, 1e-3f, 16.0f, gs.data(), none_mix.data(), nullptr);
        REQUIRE(st == PALSGD_EHIP || st == PALSGD_OK);       // EHIP without a device; with one, nothing is checked here
        if (st == PALSGD_EHIP) {
            REQUIRE(strstr(palsgd_last_error(ctx), "no GPU") != nullptr);
            REQUIRE(palsgd_step_sync(ctx, 3, 1e-3f, 16.0f, gs.data(), all_mix.data(), nullptr) == PALSGD_EHIP);
            // workers whose step counts differ cannot take a DDP step; a single worker can, but not without a device
            REQUIRE(palsgd_ddp_step(ctx, 0, 1e-3f, gs.data(), nullptr) == (K > 1 ? PALSGD_ESTATE : PALSGD_EHIP));
            REQUIRE(palsgd_clip_mean_grad_norm(ctx, 1.0f, gs.data(), nullptr, nullptr) == PALSGD_EHIP);
            REQUIRE(palsgd_get_state(ctx, got.data(), &n_outer) == PALSGD_OK && got == tau && n_outer == 9);
        }
        REQUIRE(palsgd_set_tuning(ctx, 2, 0, 0) == PALSGD_EINVAL && palsgd_set_tuning(ctx, 12, 4, 2) == PALSGD_OK);
        REQUIRE(palsgd_set_outer_lr(ctx, -1.0f) == PALSGD_EINVAL && palsgd_set_outer_lr(ctx, 0.5f) == PALSGD_OK);
        palsgd_destroy(ctx);
    }
    puts("host ok");
    return 0;
}
