// Backward kernel of one stage (element-wise operations, then at most one pooling operation)
// for dense NCHW tensors; see bs_backward.cpp for how a stack is cut into stages.
//
// A lane owns VEC consecutive cells of one row of the stage's INPUT (one 128-bit vector, or one
// cell when the row length is no multiple of that) and does, per cell:
//   1. the forward pass of the stage's element-wise operations on the stored input value, in
//      the forward kernels' arithmetic (float32, rounded to the storage type after every
//      layer), so that every ReLU / clamp sees exactly the value it saw going forward.  Each
//      operation is diagonal, so the derivative of the whole list is a product of per-operation
//      factors; the lane keeps that product (t) and, for every Add passed so far, the product of
//      the factors after it (r[n]): the gradient of that Add's residual operand.
//   2. the gradient with respect to the list's output: the upstream gradient itself for a stage
//      without pooling; otherwise a gather over the pooling windows that hold the cell, in
//      row-major window order -- max pooling: the gradients of the windows whose recorded pick
//      is this cell; average pooling: every window's gradient times the float32 reciprocal of
//      the divisor the forward pass used for it.  A gather needs no atomics and gives the same
//      sums on every run.
//   3. grad_in = that gradient * t, grad_residual[n] = that gradient * r[n], rounded once.
// Traffic: the stage input and the gradients in and out move once; the upstream gradient and
// the picks of overlapping windows are re-read from cache.
#include "bs_device.h"
#include "bs_internal.h"

namespace bs {

// float32 reciprocal of the divisor of the average pooling window (oh, ow): the forward
// kernels' rule (0: in-range cells, 1: kh * kw, 2: cells inside the padded plane).
BS_DEV float bwd_avg_inv(const PoolK &p, int32_t H, int32_t W, int32_t oh, int32_t ow)
{
    if (p.count_include_pad == 1) return p.inv_kk;
    const int32_t h0 = oh * p.sh - p.ph, w0 = ow * p.sw - p.pw;
    if (p.count_include_pad == 2) {
        const int32_t nr = min(h0 + p.kh, H + p.ph) - h0, nc = min(w0 + p.kw, W + p.pw) - w0;
        return 1.0f / (float)max(nr * nc, 1);
    }
    const int32_t nr = min(h0 + p.kh, H) - max(h0, 0), nc = min(w0 + p.kw, W) - max(w0, 0);
    return 1.0f / (float)max(nr * nc, 1);
}

template <int DT, int VEC>
__global__ __launch_bounds__(256) void bwd_stage_kernel(const BwdK k)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t rowi = fdiv(i, k.div_wv);         // plane * H + ih
    const uint32_t wv = i - rowi * k.div_wv.d;
    const uint32_t plane = fdiv(rowi, k.div_h);
    const int32_t ih = (int32_t)(rowi - plane * (uint32_t)k.H);
    const int32_t iw0 = (int32_t)(wv * VEC);
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c = (int32_t)(plane - img * (uint32_t)k.C);
    const uint32_t off = rowi * (uint32_t)k.W + (uint32_t)iw0;  // < N*C*H*W: i < total, or 0

    // ---- 1. forward through the element-wise list, collecting derivative products
    float x[VEC], t[VEC], r[K_MAX_RES][VEC];
    unpack<DT, VEC>(load_raw<DT, VEC, true>(k.a, off), x);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        t[e] = 1.0f;
#pragma unroll
        for (int n = 0; n < K_MAX_RES; ++n) r[n][e] = 0.0f;
    }
    int32_t adds = 0;
#pragma clang loop unroll(disable)
    for (int32_t j = 0; j < k.n_ew; ++j) {
        const int32_t kind = k.ew[j].kind, arg = k.ew[j].arg;
        if (kind == OP_ADD) {
            float v[VEC];
            unpack<DT, VEC>(load_raw<DT, VEC, true>(k.res[adds], off), v);
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(x[e] + v[e]);
            // from here on the residual's gradient collects the same factors as the input's
#pragma unroll
            for (int n = 0; n < K_MAX_RES; ++n)
                if (n == adds) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) r[n][e] = 1.0f;
                }
            ++adds;
            continue;
        }
        float f[VEC];  // d(output) / d(input) of this operation at x
        if (kind == OP_BN) {
            const float sc = k.params[arg + c], sh = k.params[arg + k.C + c];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                f[e] = sc;
                x[e] = round_store<DT>(__builtin_fmaf(x[e], sc, sh));
            }
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                f[e] = x[e] > 0.0f ? 1.0f : 0.0f;
                x[e] = __builtin_fmaxf(x[e], 0.0f);
            }
        } else if (kind == OP_LEAKY) {
            const float slope = k.params[arg];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                f[e] = x[e] > 0.0f ? 1.0f : slope;
                x[e] = round_store<DT>(x[e] > 0.0f ? x[e] : x[e] * slope);
            }
        } else {  // OP_CLAMP: the gradient passes where lo <= x <= hi
            const float lo = k.params[arg], hi = k.params[arg + 1];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                f[e] = (x[e] >= lo && x[e] <= hi) ? 1.0f : 0.0f;
                x[e] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[e], lo), hi));
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            t[e] *= f[e];
#pragma unroll
            for (int n = 0; n < K_MAX_RES; ++n) r[n][e] *= f[e];
        }
    }

    // ---- 2. gradient with respect to the list's output
    float s[VEC];
    const PoolK &p = k.pool;
    if (p.kind == 0) {
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.g_out, off), s);
    } else {
        const bool is_max = p.kind == OP_MAXPOOL;
        // windows (oh, ow) whose rows hold ih: oh * sh - ph <= ih < oh * sh - ph + kh
        const int32_t th = ih + p.ph - p.kh + 1;
        const int32_t oh_lo = th <= 0 ? 0 : (th + p.sh - 1) / p.sh;
        const int32_t oh_hi = min((ih + p.ph) / p.sh, k.Ho - 1);
        const uint32_t obase = plane * (uint32_t)(k.Ho * k.Wo);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int32_t iw = iw0 + e;
            const int32_t tw = iw + p.pw - p.kw + 1;
            const int32_t ow_lo = tw <= 0 ? 0 : (tw + p.sw - 1) / p.sw;
            const int32_t ow_hi = min((iw + p.pw) / p.sw, k.Wo - 1);
            const int32_t cell = ih * k.W + iw;
            float acc = 0.0f;
            for (int32_t oh = oh_lo; oh <= oh_hi; ++oh)
                for (int32_t ow = ow_lo; ow <= ow_hi; ++ow) {
                    const uint32_t o = obase + (uint32_t)(oh * k.Wo + ow);  // 0 <= oh < Ho, 0 <= ow < Wo
                    float g[1];
                    unpack<DT, 1>(load_raw<DT, 1>(k.g_out, o), g);
                    if (is_max) acc += k.idx[o] == cell ? g[0] : 0.0f;
                    else acc += g[0] * bwd_avg_inv(p, k.H, k.W, oh, ow);
                }
            s[e] = acc;
        }
    }

    // ---- 3. results
    if (!live) return;
    if (k.g_in) {
        float v[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = s[e] * t[e];
        store_elems<DT, VEC>(k.g_in, off, v);
    }
#pragma unroll
    for (int n = 0; n < K_MAX_RES; ++n)
        if (n < adds && k.g_res[n]) {
            float v[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = s[e] * r[n][e];
            store_elems<DT, VEC>(k.g_res[n], off, v);
        }
}

static void set_error(hipError_t e) { set_hip_error((int32_t)e); }

bs_status launch_backward_stage(const BwdK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t full = dtype == BS_F32 ? 4 : 8;
    // the launch must cover exactly the lanes the argument block describes
    if (grid < 1 || grid > 0x7fffffffll || threads != 256) return BS_ERR_UNSUPPORTED;
    if ((vec != 1 && vec != full) || k.W % vec != 0 || (int64_t)k.div_wv.d * vec != k.W || (int64_t)k.div_h.d != k.H ||
        (int64_t)k.div_c.d != k.C || (int64_t)grid * threads < (int64_t)k.total)
        return BS_ERR_UNSUPPORTED;
    if (k.n_ew < 0 || k.n_ew > K_BWD_EW) return BS_ERR_UNSUPPORTED;
    if (k.pool.kind == OP_MAXPOOL && !k.idx) return BS_ERR_NULL;
    const dim3 g((uint32_t)grid), b((uint32_t)threads);
    if (dtype == BS_F32) {
        if (vec == 4) bwd_stage_kernel<DT_F32, 4><<<g, b, 0, st>>>(k);
        else bwd_stage_kernel<DT_F32, 1><<<g, b, 0, st>>>(k);
    } else if (dtype == BS_BF16) {
        if (vec == 8) bwd_stage_kernel<DT_BF16, 8><<<g, b, 0, st>>>(k);
        else bwd_stage_kernel<DT_BF16, 1><<<g, b, 0, st>>>(k);
    } else if (dtype == BS_F16) {
        if (vec == 8) bwd_stage_kernel<DT_F16, 8><<<g, b, 0, st>>>(k);
        else bwd_stage_kernel<DT_F16, 1><<<g, b, 0, st>>>(k);
    } else {
        return BS_ERR_UNSUPPORTED;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(e);
        return BS_ERR_HIP;
    }
    return BS_OK;
}

}  // namespace bs
