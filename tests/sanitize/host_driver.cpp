// Host-side robustness driver: random layer lists (valid and invalid) through
// bs_stack_create, host-only bs_stack_plan with random options, every query, the backward
// plan on top of it, the error paths of bs_stack_run / bs_stack_backward, and bs_stack_destroy.  Built with AddressSanitizer and
// UndefinedBehaviorSanitizer against a host-only build of the library (tests/test_host_sanitize.py);
// touches no device.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "brainslug.h"

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n)
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33) % n;
}

int main(int argc, char **argv)
{
    const int cases = argc > 1 ? std::atoi(argv[1]) : 2000;
    int created = 0, planned = 0, declined = 0, backward_plans = 0;
    for (int it = 0; it < cases; ++it) {
        const int64_t shape[4] = {1 + rnd(3), 1 + rnd(6), 1 + rnd(48), 1 + rnd(48)};
        const int64_t C = shape[1];
        std::vector<float> ones(C, 1.0f), zeros(C, 0.0f), var(C);
        for (int64_t c = 0; c < C; ++c) var[c] = 0.5f + 0.25f * rnd(5);
        std::vector<bs_layer_desc> layers(rnd(10) + (rnd(20) == 0 ? 0 : 1));
        for (bs_layer_desc &d : layers) {
            d = bs_layer_desc{};
            d.kind = 1 + rnd(rnd(30) == 0 ? 9 : 7);  // now and then an unknown kind
            if (d.kind == BS_BATCHNORM) {
                d.gamma = ones.data(); d.beta = zeros.data(); d.running_mean = zeros.data();
                d.running_var = rnd(40) == 0 ? nullptr : var.data();
                d.eps = rnd(40) == 0 ? -1.0 : 1e-5;
            } else if (d.kind == BS_MAXPOOL || d.kind == BS_AVGPOOL) {
                d.kh = rnd(25) == 0 ? 0 : 1 + rnd(6); d.kw = 1 + rnd(6);
                d.sh = 1 + rnd(3); d.sw = rnd(25) == 0 ? 0 : 1 + rnd(3);
                d.ph = rnd(d.kh / 2 + 1 + (rnd(25) == 0)); d.pw = rnd(d.kw / 2 + 1);
                d.count_include_pad = rnd(2); d.return_indices = rnd(2); d.ceil_mode = rnd(3) == 0;
                d.dilation_h = rnd(30) == 0 ? 2 : rnd(2);
            } else if (d.kind == BS_LEAKY_RELU) {
                d.negative_slope = 0.1f;
            } else if (d.kind == BS_CLAMP) {
                d.clamp_min = rnd(30) == 0 ? 2.0f : 0.0f; d.clamp_max = 1.0f;
            }
        }
        bs_stack *s = nullptr;
        const bs_status st = bs_stack_create(layers.empty() ? nullptr : layers.data(), (int32_t)layers.size(), shape,
                                             (int32_t)rnd(rnd(20) == 0 ? 3 : 2), &s);
        (void)bs_status_string(st);
        if (st != BS_OK) { ++declined; if (s) { std::puts("handle returned on failure"); return 1; } continue; }
        ++created;
        int64_t os[4];
        if (bs_stack_output_shape(s, os) != BS_OK || os[2] < 1 || os[3] < 1) { std::puts("bad output shape"); return 1; }
        for (int32_t i = -1; i <= bs_stack_num_residuals(s); ++i) (void)bs_stack_residual_shape(s, i, os);
        for (int32_t i = -1; i <= bs_stack_num_index_outputs(s); ++i) (void)bs_stack_index_shape(s, i, os);
        for (int32_t i = -1; i <= (int32_t)layers.size(); ++i) {
            std::vector<float> a(C), b(C);
            (void)bs_stack_folded_bn(s, i, a.data(), b.data());
        }
        for (int rep = 0; rep < 3; ++rep) {
            bs_plan_options o{};
            o.host_only = 1;
            o.num_cus = rnd(3) == 0 ? 0 : 1 + rnd(300);
            const uint64_t budgets[] = {0, 1024, 4096, 16384, 65536, 1u << 20};
            o.max_lds_bytes = budgets[rnd(6)];
            o.max_steps_per_sequence = rnd(4) == 0 ? (int32_t)rnd(7) - 1 : 0;
            const int32_t thr[] = {0, 64, 128, 256, 512, 100};
            o.threads_per_group = thr[rnd(6)];
            o.breadth_first = rnd(5) == 0;
            o.force_variant = rnd(3) == 0 ? (int32_t)rnd(7) : 0;
            o.tile_rows = rnd(4) == 0 ? (int32_t)rnd(40) : 0;
            o.tile_cols = rnd(4) == 0 ? (int32_t)rnd(40) : 0;
            o.planes_per_group = rnd(6) == 0 ? (int32_t)rnd(20) : 0;
            o.jit = (int32_t)rnd(4) - 1 - (rnd(40) == 0);
            const bs_status ps = bs_stack_plan(s, rnd(8) == 0 ? nullptr : &o);
            bs_plan_info pi{};
            if (ps != BS_OK) {
                if (bs_stack_plan_info(s, &pi) == BS_OK && pi.device_planned) { std::puts("device plan without a device?"); }
                continue;
            }
            ++planned;
            if (bs_stack_plan_info(s, &pi) != BS_OK || pi.n_sequences < 1 || pi.n_steps < pi.n_sequences) {
                std::puts("inconsistent plan info");
                return 1;
            }
            int32_t steps = 0;
            for (int32_t q = -1; q <= pi.n_sequences; ++q) {
                bs_sequence_info si{};
                if (bs_stack_sequence_info(s, q, &si) == BS_OK) steps += si.n_steps;
            }
            if (steps != pi.n_steps) { std::puts("sequences do not partition the steps"); return 1; }
            for (int32_t t = -1; t <= pi.n_steps; ++t) { bs_step_info ti{}; (void)bs_stack_step_info(s, t, &ti); }
            for (int32_t t = -1; t <= pi.n_operations; ++t) (void)bs_stack_operation_name(s, t);
            (void)bs_stack_workspace_bytes(s);
            // backward plan on the host-only plan: stages and their forward plans are built and freed
            if (rnd(2) == 0) {
                const bs_status bp = bs_stack_plan_backward(s);
                const int32_t stages = bs_stack_backward_num_stages(s);
                if ((bp == BS_OK) != (stages >= 1)) { std::puts("backward plan and stage count disagree"); return 1; }
                if (bp == BS_OK && stages > pi.n_operations + 1) { std::puts("more stages than operations"); return 1; }
                (void)bs_stack_backward_workspace_bytes(s);
                float dummy[4] = {0, 0, 0, 0};
                if (bs_stack_backward(s, dummy, nullptr, nullptr, dummy, dummy, nullptr, nullptr, 0, nullptr) == BS_OK) {
                    std::puts("backward succeeded on a host-only plan");
                    return 1;
                }
                ++backward_plans;
            }
            if (pi.device_planned == 0) {
                float dummy[4] = {0, 0, 0, 0};
                if (bs_stack_run(s, dummy, nullptr, dummy, nullptr, nullptr, 0, nullptr) == BS_OK) {
                    std::puts("run succeeded on a host-only plan");
                    return 1;
                }
            }
        }
        bs_stack_destroy(s);
    }
    bs_stack_destroy(nullptr);
    std::printf("ok: %d created, %d declined at create, %d plans, %d backward plans\n", created, declined, planned, backward_plans);
    return 0;
}
