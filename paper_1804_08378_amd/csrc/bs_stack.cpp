// Stack handle: validation of the layer list, host copies, BatchNorm folding and
// the shape queries of the scheduler (Section 4.2).
// Pure host code: nothing in this file touches a device.
#include <cmath>
#include <cstring>
#include <new>

#include "bs_internal.h"

namespace bs {

size_t dtype_size(int32_t dtype) { return dtype == BS_F32 ? 4 : 2; }

static thread_local int32_t g_last_hip_error = 0;
void set_hip_error(int32_t e) { g_last_hip_error = e; }

FastDiv make_fastdiv(uint32_t d)
{
    // For 0 <= n < 2^31 and d >= 2:  n / d == umulhi(n, m) >> (l - 1)
    // with l = ceil(log2 d) and m = floor(2^(31+l) / d) + 1  (m < 2^32).
    FastDiv f;
    f.d = d ? d : 1;
    if (f.d == 1) {
        f.mul = 0;
        f.shift = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < f.d) ++l;
    f.mul = (uint32_t)(((1ull << (31 + l)) / f.d) + 1);
    f.shift = l - 1;
    return f;
}

static bool finite_all(const float *p, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        if (!std::isfinite(p[i])) return false;
    return true;
}

}  // namespace bs

using namespace bs;

extern "C" {

bs_status bs_stack_create(const bs_layer_desc *layers, int32_t n_layers, const int64_t in_shape[4],
                          int32_t dtype, bs_stack **out)
{
    if (!layers || !in_shape || !out) return BS_ERR_NULL;
    if (n_layers < 1 || n_layers > BS_MAX_LAYERS) return BS_ERR_UNSUPPORTED;
    if (dtype != BS_F32 && dtype != BS_BF16 && dtype != BS_F16) return BS_ERR_UNSUPPORTED;
    for (int i = 0; i < 4; ++i)
        if (in_shape[i] < 1) return BS_ERR_SHAPE;
    const int64_t limit = (1ll << 31) - 1;
    // every tensor of the stack must be indexable with 31 bits
    if (in_shape[0] * in_shape[1] > limit || in_shape[2] * in_shape[3] > limit ||
        (double)in_shape[0] * (double)in_shape[1] * (double)in_shape[2] * (double)in_shape[3] >
            (double)limit)
        return BS_ERR_UNSUPPORTED;

    bs_stack *s = new (std::nothrow) bs_stack();
    if (!s) return BS_ERR_ALLOC;
    bs_status err = BS_OK;
    try {
        s->dtype = dtype;
        std::memcpy(s->in_shape, in_shape, sizeof(s->in_shape));
        int64_t cur[4] = {in_shape[0], in_shape[1], in_shape[2], in_shape[3]};
        const int64_t C = in_shape[1];
        s->layers.resize(n_layers);
        for (int32_t i = 0; i < n_layers && err == BS_OK; ++i) {
            const bs_layer_desc &d = layers[i];
            Layer &L = s->layers[i];
            L.desc = d;
            L.desc.gamma = L.desc.beta = L.desc.running_mean = L.desc.running_var = nullptr;
            std::memcpy(L.in_shape, cur, sizeof(cur));
            switch (d.kind) {
            case BS_BATCHNORM: {
                if (!d.gamma || !d.beta || !d.running_mean || !d.running_var) { err = BS_ERR_NULL; break; }
                if (!std::isfinite(d.eps) || d.eps < 0) { err = BS_ERR_PARAM; break; }
                if (!finite_all(d.gamma, C) || !finite_all(d.beta, C) || !finite_all(d.running_mean, C) ||
                    !finite_all(d.running_var, C)) { err = BS_ERR_PARAM; break; }
                L.gamma.assign(d.gamma, d.gamma + C);
                L.beta.assign(d.beta, d.beta + C);
                L.mean.assign(d.running_mean, d.running_mean + C);
                L.var.assign(d.running_var, d.running_var + C);
                L.scale.resize(C);
                L.shift.resize(C);
                for (int64_t c = 0; c < C; ++c) {
                    const double v = (double)L.var[c] + d.eps;
                    if (!(v > 0.0)) { err = BS_ERR_PARAM; break; }
                    // fold in float64, round each of scale and shift once
                    const double sc = (double)L.gamma[c] / std::sqrt(v);
                    L.scale[c] = (float)sc;
                    L.shift[c] = (float)((double)L.beta[c] - (double)L.mean[c] * sc);
                    if (!std::isfinite(L.scale[c]) || !std::isfinite(L.shift[c])) { err = BS_ERR_PARAM; break; }
                }
                break;
            }
            case BS_RELU:
                break;
            case BS_LEAKY_RELU:
                if (!std::isfinite(d.negative_slope)) { err = BS_ERR_PARAM; break; }
                break;
            case BS_CLAMP:
                if (!std::isfinite(d.clamp_min) || !std::isfinite(d.clamp_max) || d.clamp_min > d.clamp_max) {
                    err = BS_ERR_PARAM;
                    break;
                }
                break;
            case BS_ADD:
                if (s->n_res >= BS_MAX_RESIDUALS) { err = BS_ERR_UNSUPPORTED; break; }
                std::memcpy(s->res_shape[s->n_res++], cur, sizeof(cur));
                break;
            case BS_MAXPOOL:
            case BS_AVGPOOL: {
                if ((d.dilation_h != 0 && d.dilation_h != 1) || (d.dilation_w != 0 && d.dilation_w != 1)) {
                    err = BS_ERR_UNSUPPORTED;
                    break;
                }
                if (d.kh < 1 || d.kw < 1 || d.sh < 1 || d.sw < 1 || d.ph < 0 || d.pw < 0 ||
                    d.ph > d.kh / 2 || d.pw > d.kw / 2 || d.kh > 1024 || d.kw > 1024 || d.sh > 1024 ||
                    d.sw > 1024) { err = BS_ERR_PARAM; break; }
                const int64_t nh = cur[2] + 2 * d.ph - d.kh, nw = cur[3] + 2 * d.pw - d.kw;
                if (nh < 0 || nw < 0) { err = BS_ERR_SHAPE; break; }
                // floor mode: the windows that fit; ceil mode: one more window if cells are left
                // uncovered, unless it would start beyond the input and its leading padding
                auto out_size = [&](int64_t in, int64_t n, int64_t st, int64_t pad) {
                    int64_t o = n / st + 1;
                    if (d.ceil_mode != 0 && n % st != 0 && o * st < in + pad) ++o;
                    return o;
                };
                const int64_t oh = out_size(cur[2], nh, d.sh, d.ph), ow = out_size(cur[3], nw, d.sw, d.pw);
                // recorded only where it changes the result: an overhanging last window
                L.desc.ceil_mode = (oh != nh / d.sh + 1 || ow != nw / d.sw + 1) ? 1 : 0;
                cur[2] = oh;
                cur[3] = ow;
                s->has_pool = true;
                if (d.kind == BS_MAXPOOL && d.return_indices) {
                    if (s->n_idx >= BS_MAX_INDEX_OUTPUTS) { err = BS_ERR_UNSUPPORTED; break; }
                    std::memcpy(s->idx_shape[s->n_idx++], cur, sizeof(cur));
                }
                break;
            }
            default:
                err = BS_ERR_UNSUPPORTED;
            }
            std::memcpy(L.out_shape, cur, sizeof(cur));
        }
        std::memcpy(s->out_shape, cur, sizeof(cur));
    } catch (const std::bad_alloc &) {
        err = BS_ERR_ALLOC;
    }
    if (err != BS_OK) {
        delete s;
        return err;
    }
    *out = s;
    return BS_OK;
}

void bs_stack_destroy(bs_stack *stack)
{
    if (!stack) return;
    free_backward(stack);
    free_params(stack);
    delete stack;
}

bs_status bs_stack_output_shape(const bs_stack *stack, int64_t out_shape[4])
{
    if (!stack || !out_shape) return BS_ERR_NULL;
    std::memcpy(out_shape, stack->out_shape, sizeof(stack->out_shape));
    return BS_OK;
}

int32_t bs_stack_num_residuals(const bs_stack *stack) { return stack ? stack->n_res : -1; }

bs_status bs_stack_residual_shape(const bs_stack *stack, int32_t i, int64_t shape[4])
{
    if (!stack || !shape) return BS_ERR_NULL;
    if (i < 0 || i >= stack->n_res) return BS_ERR_RANGE;
    std::memcpy(shape, stack->res_shape[i], sizeof(stack->res_shape[i]));
    return BS_OK;
}

int32_t bs_stack_num_index_outputs(const bs_stack *stack) { return stack ? stack->n_idx : -1; }

bs_status bs_stack_index_shape(const bs_stack *stack, int32_t i, int64_t shape[4])
{
    if (!stack || !shape) return BS_ERR_NULL;
    if (i < 0 || i >= stack->n_idx) return BS_ERR_RANGE;
    std::memcpy(shape, stack->idx_shape[i], sizeof(stack->idx_shape[i]));
    return BS_OK;
}

bs_status bs_stack_folded_bn(const bs_stack *stack, int32_t layer, float *scale, float *shift)
{
    if (!stack) return BS_ERR_NULL;
    if (layer < 0 || layer >= (int32_t)stack->layers.size() ||
        stack->layers[layer].desc.kind != BS_BATCHNORM)
        return BS_ERR_RANGE;
    const Layer &L = stack->layers[layer];
    if (scale) std::memcpy(scale, L.scale.data(), L.scale.size() * sizeof(float));
    if (shift) std::memcpy(shift, L.shift.data(), L.shift.size() * sizeof(float));
    return BS_OK;
}

const char *bs_status_string(bs_status status)
{
    switch (status) {
    case BS_OK: return "ok";
    case BS_ERR_NULL: return "a required pointer is NULL";
    case BS_ERR_SHAPE: return "invalid shape (non-positive dimension or empty pooling output)";
    case BS_ERR_PARAM: return "invalid layer parameter or plan option";
    case BS_ERR_UNSUPPORTED: return "unsupported layer kind, mode, dtype or size";
    case BS_ERR_NOT_PLANNED: return "stack has no device plan";
    case BS_ERR_NO_FIT: return "a step does not fit the on-chip memory budget";
    case BS_ERR_ALIGN: return "device pointer is not 16-byte aligned";
    case BS_ERR_WORKSPACE: return "workspace missing or too small";
    case BS_ERR_HIP: return "HIP call failed";
    case BS_ERR_ALLOC: return "host allocation failed";
    case BS_ERR_RANGE: return "index out of range";
    case BS_ERR_ALIAS: return "output overlaps an input";
    case BS_ERR_JIT: return "run-time kernel build failed";
    case BS_ERR_DEVICE: return "current device is not the device the stack was planned on";
    }
    return "unknown status";
}

const char *bs_version(void) { return "brainslug-hip 0.1.0 (gfx950)"; }

int32_t bs_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
