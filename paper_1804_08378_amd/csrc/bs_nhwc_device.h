// Device helpers shared by the channels-last kernels: per-lane parameter vectors, the
// element-wise list applied to channel vectors, the average's divisor.
#pragma once
#include "bs_device.h"

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
//   off[u]  element offset of vector u in this level's tensors (residual loads), counted from
//           element res_base (the same for all lanes)
//   CODE    >= 0: the list's kinds as a code of base-K_EW_BASE digits (n_ew is ignored): the list unrolls into
//           straight code and only the arguments come from `ew`; -1: kinds and length are read at run time
template <int DT, int VEC, int U, int CODE = -1>
BS_DEV void apply_ew_nhwc(float (&x)[U][VEC], uint32_t c0, const uint32_t (&off)[U], const EwOp *ew,
                          int32_t n_ew, const float *__restrict__ params, int32_t C, const void *const *res,
                          uint32_t res_base = 0)
{
    auto one = [&](const int32_t kind, const int32_t arg) {
        if (kind == OP_BN) {
            float sc[VEC], sh[VEC];
            load_params<VEC>(params, (uint32_t)arg + c0, sc);
            load_params<VEC>(params, (uint32_t)(arg + C) + c0, sh);
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = __builtin_fmaf(x[u][i], sc[i], sh[i]);
                round_store_all<DT, VEC>(x[u]);
            }
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
            for (int u = 0; u < U; ++u) rr[u] = load_raw<DT, VEC, true>(rp, off[u] + res_base);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float r[VEC];
                unpack<DT, VEC>(rr[u], r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(x[u][i] + r[i]);
            }
        }
    };
    if constexpr (CODE >= 0) {
#pragma unroll
        for (int j = 0; j < ew_code_len(CODE); ++j) one(ew_code_kind(CODE, j), ew[j].arg);
    } else {
#pragma clang loop unroll(disable)
        for (int32_t j = 0; j < n_ew; ++j) one(ew[j].kind, ew[j].arg);
    }
}

// float32 reciprocal of the average's divisor for the window at (h0, w0), in-range part
// [hlo, hhi) x [wlo, whi)
BS_DEV float avg_inv(const PoolK &p, int32_t kh, int32_t kw, int32_t H, int32_t W, int32_t h0, int32_t w0,
                     int32_t hlo, int32_t hhi, int32_t wlo, int32_t whi)
{
    if (!p.count_include_pad) return 1.0f / (float)max((hhi - hlo) * (whi - wlo), 1);
    if (p.count_include_pad == 2) {  // ceil mode: cells inside the padded plane
        const int32_t nr = min(h0 + kh, H + p.ph) - h0, nc = min(w0 + kw, W + p.pw) - w0;
        return 1.0f / (float)max(nr * nc, 1);
    }
    return p.inv_kk;
}

}  // namespace bs
