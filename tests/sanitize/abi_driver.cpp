// Host sanitizer driver for the C ABI: links the library's API translation unit, compiled with
// -fsanitize=address,undefined on the host side, and walks the argument checks that return before any
// device work: bad dimensions, null pointers, sizes beyond the static buffer, messages.  Needs no GPU.
#include <cstdio>
#include <cstring>

#include "bagel.h"

static bagel_dims good()
{
    bagel_dims d;
    std::memset(&d, 0, sizeof(d));
    d.d_s = 2; d.d_a = 1; d.d_g = 1; d.N = 8; d.L = 8; d.S = 4; d.B = 16; d.H = 5;
    d.n_hidden = 1; d.hidden[0] = 8; d.q[0] = 1.0f; d.sigma_r = 1.0f;
    return d;
}

#define EXPECT(cond)                                                   \
    do {                                                               \
        if (!(cond)) {                                                 \
            std::printf("abi sanitizer driver: FAILED at %s\n", #cond); \
            return 1;                                                  \
        }                                                              \
    } while (0)

int main()
{
    bagel_dims d = good();
    EXPECT(bagel_num_params(&d) == 3 * 8 + 8 + 8 + 1);
    EXPECT(bagel_num_params(nullptr) == BAGEL_EINVAL);
    struct { int bagel_dims::*field; int value; } bad[] = {
        {&bagel_dims::d_s, 0}, {&bagel_dims::d_s, 9}, {&bagel_dims::d_a, 0}, {&bagel_dims::d_g, 3}, {&bagel_dims::N, 0},
        {&bagel_dims::L, -1}, {&bagel_dims::S, 3}, {&bagel_dims::S, 32}, {&bagel_dims::H, 0}, {&bagel_dims::n_hidden, 0},
        {&bagel_dims::n_hidden, 3}, {&bagel_dims::ckpt_interval, -1}, {&bagel_dims::cost_kind, 2},
    };
    for (auto &b : bad) {
        bagel_dims e = good();
        e.*(b.field) = b.value;
        bagel_ctx *ctx = reinterpret_cast<bagel_ctx *>(0x1);
        EXPECT(bagel_num_params(&e) == BAGEL_EINVAL);
        EXPECT(bagel_create(&ctx, &e, nullptr) == BAGEL_EINVAL);
        EXPECT(ctx == nullptr);
        EXPECT(std::strncmp(bagel_last_error(nullptr), "bagel_create:", 13) == 0);
    }
    bagel_dims e = good();
    e.hidden[0] = 257;
    EXPECT(bagel_num_params(&e) == BAGEL_EINVAL);
    e = good(); e.tracked[0] = 2;
    EXPECT(bagel_num_params(&e) == BAGEL_EINVAL);
    e = good(); e.cost_kind = 1; e.sigma_r = 0.0f;
    EXPECT(bagel_num_params(&e) == BAGEL_EINVAL);
    EXPECT(bagel_create(nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_destroy(nullptr) == BAGEL_OK);
    EXPECT(bagel_workspace_bytes(nullptr) == 0);
    EXPECT(bagel_rollout_loss(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_rollout_loss_grad(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_set_samples(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_prepare_samples(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_sample_eval(nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_adam_step(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1e-2f, 0.9f, 0.999f, 1e-8f) == BAGEL_EINVAL);
    EXPECT(bagel_optimize(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, 1, 1e-2f, 0.9f, 0.999f, 1e-8f, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_hyper_lml_grad(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_hyper_fit(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, 1e-2f, 0.9f, 0.999f, 1e-8f, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_prepare_posterior(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_posterior_rollout_loss(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == BAGEL_EINVAL);
    EXPECT(bagel_profile_enable(nullptr, 1) == BAGEL_EINVAL);
    // the allocation-free entry point: null dims, bad dims, null arrays, sizes beyond the static buffer
    float dummy = 0.0f;
    const float *p = &dummy;
    EXPECT(bagel_sample_eval_static(nullptr, nullptr, p, p, p, p, p, p, p, p, &dummy, nullptr) == BAGEL_EINVAL);
    e = good(); e.S = 3;
    EXPECT(bagel_sample_eval_static(&e, nullptr, p, p, p, p, p, p, p, p, &dummy, nullptr) == BAGEL_EINVAL);
    e = good();
    EXPECT(bagel_sample_eval_static(&e, nullptr, nullptr, p, p, p, p, p, p, p, &dummy, nullptr) == BAGEL_EINVAL);
    e.N = 4096; e.L = 4096; e.S = 4096; e.B = 4096;
    EXPECT(bagel_sample_eval_static(&e, nullptr, p, p, p, p, p, p, p, p, &dummy, nullptr) == BAGEL_EINVAL);
    EXPECT(std::strstr(bagel_last_error(nullptr), "static buffer") != nullptr);
    std::printf("abi sanitizer driver: ok\n");
    return 0;
}
