// Shared pieces of the register sliding-window pooling kernels (bs_rows.hip, bs_rows2.hip):
// compile-time pooling shapes, compile-time BatchNorm / ReLU lists and their parameters.
#pragma once
#include <type_traits>

#include "bs_device.h"

namespace bs {

template <int KIND, int KH, int KW, int SH, int SW, int PH, int PW>
struct RowsSpec {
    static constexpr int kind = KIND, kh = KH, kw = KW, sh = SH, sw = SW, ph = PH, pw = PW;
};

// element-wise list codes (base 4 digits, first operation lowest): see rows_ew_code()
constexpr int K_ROWS_OR = 2;  // output rows per lane per iteration (all their input rows are requested at once)
constexpr int RW_NONE = 0;
constexpr int RW_RELU = OP_RELU;
constexpr int RW_BN_RELU = OP_BN + 4 * OP_RELU;

template <int CODE>
struct RowsEw {
    static constexpr int count()
    {
        int n = 0, c = CODE;
        while (c) { ++n; c /= 4; }
        return n;
    }
    static constexpr int n = count();
    __host__ __device__ static constexpr int kind(int j)
    {
        int c = CODE;
        for (int i = 0; i < j; ++i) c /= 4;
        return c % 4;
    }
};

template <class EW>
struct RowsParams {
    float sc[EW::n > 0 ? EW::n : 1], sh[EW::n > 0 ? EW::n : 1];
};

template <class EW>
BS_DEV void rows_load_params(const EwOp *ew, const float *__restrict__ params, int32_t C, int32_t c,
                             RowsParams<EW> &p)
{
#pragma unroll
    for (int j = 0; j < EW::n; ++j) {
        p.sc[j] = 1.0f;
        p.sh[j] = 0.0f;
        if (EW::kind(j) == OP_BN) {
            p.sc[j] = params[ew[j].arg + c];
            p.sh[j] = params[ew[j].arg + C + c];
        }
    }
}

// BatchNorm / ReLU lists only (a residual Add would need its own halo loads; such stacks
// take the LDS path).
template <bool BF16, class EW, int N>
BS_DEV void rows_apply(float (&x)[N], const RowsParams<EW> &p)
{
#pragma unroll
    for (int j = 0; j < EW::n; ++j) {
        if (EW::kind(j) == OP_BN) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<BF16>(__builtin_fmaf(x[i], p.sc[j], p.sh[j]));
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = __builtin_fmaxf(x[i], 0.0f);  // NaN, -0 -> +0
        }
    }
}

using RMax3s2p1 = RowsSpec<OP_MAXPOOL, 3, 3, 2, 2, 1, 1>;
using RMax3s2p0 = RowsSpec<OP_MAXPOOL, 3, 3, 2, 2, 0, 0>;
using RMax3s1p1 = RowsSpec<OP_MAXPOOL, 3, 3, 1, 1, 1, 1>;
using RAvg3s1p1 = RowsSpec<OP_AVGSUM, 3, 3, 1, 1, 1, 1>;

// base-4 code of a BatchNorm / ReLU list (first operation lowest digit), -1 for other lists
inline int rows_ew_code(const EwOp *ew, int n)
{
    int code = 0, mul = 1;
    for (int j = 0; j < n; ++j) {
        if (ew[j].kind != OP_BN && ew[j].kind != OP_RELU) return -1;
        code += ew[j].kind * mul;
        mul *= 4;
    }
    return code;
}

template <class P>
inline bool rows_pool_is(const PoolK &q)
{
    return q.kind == P::kind && q.kh == P::kh && q.kw == P::kw && q.sh == P::sh && q.sw == P::sw &&
           q.ph == P::ph && q.pw == P::pw;
}

}  // namespace bs
