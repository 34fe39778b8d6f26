// Channels-last (NHWC) kernels.  The tensor is N x H x W x C in memory: the channels of one
// pixel are contiguous, so a lane takes one 128-bit vector of VEC consecutive channels of one
// pixel and consecutive lanes take consecutive vectors: every access of a wave is one
// contiguous run, for element-wise layers and for pooling windows alike (a window cell is a
// pixel, i.e. the same channel vector W * C elements or C elements further on).  BatchNorm
// parameters are per-lane vectors here (one 128-bit load of scale and of shift per lane).
//
//   nhwc_stream_kernel  element-wise only sequence, U vectors per lane.
//   nhwc_pool_kernel    [element-wise]* pool [element-wise]*: a lane produces VEC channels of
//                       one output pixel.  Overlapping windows re-read their shared cells
//                       through the caches and recompute the element-wise operations on them.
//
// The arithmetic and its order are those of the NCHW kernels (float32, BatchNorm one fused
// multiply-add, window cells visited row-major, first maximum wins, the average's sum taken
// over the in-range cells from +0 and multiplied by a float32 reciprocal, every layer's
// output rounded to the storage type), so the results are the same numbers in another
// memory order.  Index outputs hold ih * W + iw like the NCHW ones and are laid out like
// the output tensor.
#include "bs_device.h"
#include "bs_internal.h"

namespace bs {

// VEC consecutive float32 parameters starting at element `off` (a multiple of VEC; BatchNorm
// tables start at multiples of 8 floats): 128-bit loads, served by the caches.
template <int VEC>
BS_DEV void load_params(const float *__restrict__ params, uint32_t off, float (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            const float4 t = *reinterpret_cast<const float4 *>(params + off + 4 * q);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = params[off + i];
    }
}

// Apply an element-wise list to U register vectors that all hold channels c0 .. c0 + VEC - 1.
//   off[u]  element offset of vector u in this level's tensors (residual loads)
template <int DT, int VEC, int U>
BS_DEV void apply_ew_nhwc(float (&x)[U][VEC], uint32_t c0, const uint32_t (&off)[U], const EwOp *ew,
                          int32_t n_ew, const float *__restrict__ params, int32_t C, const void *const *res)
{
#pragma clang loop unroll(disable)
    for (int32_t j = 0; j < n_ew; ++j) {
        const int32_t kind = ew[j].kind, arg = ew[j].arg;
        if (kind == OP_BN) {
            float sc[VEC], sh[VEC];
            load_params<VEC>(params, (uint32_t)arg + c0, sc);
            load_params<VEC>(params, (uint32_t)(arg + C) + c0, sh);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(__builtin_fmaf(x[u][i], sc[i], sh[i]));
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = __builtin_fmaxf(x[u][i], 0.0f);  // NaN, -0 -> +0
        } else if (kind == OP_LEAKY) {
            const float slope = params[arg];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(x[u][i] > 0.0f ? x[u][i] : x[u][i] * slope);
        } else if (kind == OP_CLAMP) {
            const float lo = params[arg], hi = params[arg + 1];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    x[u][i] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[u][i], lo), hi));
        } else {  // OP_ADD
            const void *rp = res[arg];
            Raw<DT, VEC> rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) rr[u] = load_raw<DT, VEC, true>(rp, off[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float r[VEC];
                unpack<DT, VEC>(rr[u], r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(x[u][i] + r[i]);
            }
        }
    }
}

// Element-wise only.  A work-group takes nthr * U consecutive vectors; lane t handles vectors
// t, t + nthr, ...
template <int DT, int VEC, int U>
__global__ __launch_bounds__(512) void nhwc_stream_kernel(const NhwcK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t cvn = k.div_cv.d;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        const bool valid = i < k.total;
        i = valid ? i : 0u;
        const uint32_t off1[1] = {i * VEC};
        const uint32_t c0 = (i - fdiv(i, k.div_cv) * cvn) * VEC;
        float x[1][VEC];
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.in, off1[0]), x[0]);
        apply_ew_nhwc<DT, VEC, 1>(x, c0, off1, k.pre, k.n_pre, k.params, k.C, k.res);
        if (valid) store_elems<DT, VEC>(k.out, off1[0], x[0]);
    }
}

// One pooling operation.  KH, KW > 0: the window is a compile-time constant, all its cells
// are requested at once and the element-wise operations run once over all of them; KH == 0:
// any window, one cell at a time.
template <int DT, int VEC, int KH, int KW>
__global__ __launch_bounds__(256) void nhwc_pool_kernel(const NhwcK k)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    // lane -> (image n, output row oh, output column ow, channel vector cv), cv fastest
    const uint32_t pix = fdiv(i, k.div_cv);
    const uint32_t c0 = (i - pix * k.div_cv.d) * VEC;
    const uint32_t t = fdiv(pix, k.div_wo);
    const int32_t ow = (int32_t)(pix - t * (uint32_t)k.Wo);
    const uint32_t n = fdiv(t, k.div_ho);
    const int32_t oh = (int32_t)(t - n * (uint32_t)k.Ho);
    const PoolK &p = k.pool;
    const int32_t kh = KH > 0 ? KH : p.kh, kw = KH > 0 ? KW : p.kw;
    const int32_t h0 = oh * p.sh - p.ph, w0 = ow * p.sw - p.pw;
    // in-range part of the window; never empty (the padding is at most half the window)
    const int32_t hlo = max(h0, 0), hhi = min(h0 + kh, k.H), wlo = max(w0, 0), whi = min(w0 + kw, k.W);
    const uint32_t img = n * (uint32_t)(k.H * k.W);  // first pixel of the image
    const bool is_max = p.kind == OP_MAXPOOL;

    float acc[VEC];
    int32_t bi[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        acc[e] = is_max ? -INFINITY : 0.0f;
        bi[e] = hlo * k.W + wlo;  // first in-range cell
    }
    auto take = [&](const float (&v)[VEC], int32_t ih, int32_t iw) {
        if (is_max) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const bool g = v[e] > acc[e];
                acc[e] = g ? v[e] : acc[e];
                bi[e] = g ? ih * k.W + iw : bi[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = acc[e] + v[e];
        }
    };

    if constexpr (KH > 0) {
        constexpr int NCELL = KH * KW;
        float x[NCELL][VEC];
        uint32_t off[NCELL];
        bool in[NCELL];
        Raw<DT, VEC> raw[NCELL];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh)
#pragma unroll
            for (int dw = 0; dw < KW; ++dw) {
                const int32_t ih = h0 + dh, iw = w0 + dw;
                const int cell = dh * KW + dw;
                in[cell] = ih >= hlo && ih < hhi && iw >= wlo && iw < whi;
                // a cell outside the plane is the pooling operation's padding: requested from a
                // safe address (the first in-range cell) and never used
                const int32_t ch = in[cell] ? ih : hlo, cw = in[cell] ? iw : wlo;
                off[cell] = (img + (uint32_t)(ch * k.W + cw)) * (uint32_t)k.C + c0;
                raw[cell] = load_raw<DT, VEC>(k.in, off[cell]);
            }
#pragma unroll
        for (int cell = 0; cell < NCELL; ++cell) unpack<DT, VEC>(raw[cell], x[cell]);
        apply_ew_nhwc<DT, VEC, NCELL>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
        for (int dh = 0; dh < KH; ++dh)
#pragma unroll
            for (int dw = 0; dw < KW; ++dw)
                if (in[dh * KW + dw]) take(x[dh * KW + dw], h0 + dh, w0 + dw);
    } else {
        for (int32_t ih = hlo; ih < hhi; ++ih)
            for (int32_t iw = wlo; iw < whi; ++iw) {
                const uint32_t off1[1] = {(img + (uint32_t)(ih * k.W + iw)) * (uint32_t)k.C + c0};
                float x[1][VEC];
                unpack<DT, VEC>(load_raw<DT, VEC>(k.in, off1[0]), x[0]);
                apply_ew_nhwc<DT, VEC, 1>(x, c0, off1, k.pre, k.n_pre, k.params, k.C, k.res);
                take(x[0], ih, iw);
            }
    }

    float y[1][VEC];
    if (is_max) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[0][e] = acc[e];
    } else {
        float inv = p.inv_kk;
        if (!p.count_include_pad) {
            inv = 1.0f / (float)((hhi - hlo) * (whi - wlo));
        } else if (p.count_include_pad == 2) {  // ceil mode: cells inside the padded plane
            const int32_t nr = min(h0 + kh, k.H + p.ph) - h0, nc = min(w0 + kw, k.W + p.pw) - w0;
            inv = 1.0f / (float)max(nr * nc, 1);
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[0][e] = round_store<DT>(acc[e] * inv);
    }
    const uint32_t ooff[1] = {pix * (uint32_t)k.C + c0};
    apply_ew_nhwc<DT, VEC, 1>(y, c0, ooff, k.post, k.n_post, k.params, k.C, k.res);
    if (live) {
        store_elems<DT, VEC>(k.out, ooff[0], y[0]);
        if (k.idx && is_max) store_indices<VEC>(k.idx + ooff[0], bi);
    }
}

template <int DT, int VEC>
static void launch_nhwc_t(const NhwcK &k, dim3 grid, dim3 block, hipStream_t st)
{
    if (k.pool.kind == 0) {
        nhwc_stream_kernel<DT, VEC, 4><<<grid, block, 0, st>>>(k);
    } else if (k.pool.kh == 2 && k.pool.kw == 2) {
        nhwc_pool_kernel<DT, VEC, 2, 2><<<grid, block, 0, st>>>(k);
    } else if (k.pool.kh == 3 && k.pool.kw == 3) {
        nhwc_pool_kernel<DT, VEC, 3, 3><<<grid, block, 0, st>>>(k);
    } else {
        nhwc_pool_kernel<DT, VEC, 0, 0><<<grid, block, 0, st>>>(k);
    }
}

bs_status launch_nhwc(const NhwcK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (grid < 1 || grid > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    const int32_t full = dtype == BS_F32 ? 4 : 8;
    // the vector width the plan was made for must be one the kernels exist for and must divide C
    if ((vec != 1 && vec != full) || k.C % vec != 0 || (int64_t)k.div_cv.d * vec != k.C) return BS_ERR_UNSUPPORTED;
    const dim3 g((uint32_t)grid), b((uint32_t)threads);
    if (dtype == BS_F32) {
        if (vec == 4) launch_nhwc_t<DT_F32, 4>(k, g, b, st);
        else launch_nhwc_t<DT_F32, 1>(k, g, b, st);
    } else if (dtype == BS_BF16) {
        if (vec == 8) launch_nhwc_t<DT_BF16, 8>(k, g, b, st);
        else launch_nhwc_t<DT_BF16, 1>(k, g, b, st);
    } else if (dtype == BS_F16) {
        if (vec == 8) launch_nhwc_t<DT_F16, 8>(k, g, b, st);
        else launch_nhwc_t<DT_F16, 1>(k, g, b, st);
    } else {
        return BS_ERR_UNSUPPORTED;
    }
    return BS_OK;
}

}  // namespace bs
