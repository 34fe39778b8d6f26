// Device code of the register sliding-window pooling kernels: compile-time pooling shapes,
// compile-time BatchNorm / ReLU lists and their parameters, and the two kernels.
#pragma once
#include "bs_device.h"

namespace bs {

template <int KIND, int KH, int KW, int SH, int SW, int PH, int PW>
struct RowsSpec {
    static constexpr int kind = KIND, kh = KH, kw = KW, sh = SH, sw = SW, ph = PH, pw = PW;
};

// element-wise list codes (base K_EW_BASE digits, first operation lowest): see rows_ew_code()
constexpr int RW_NONE = 0;
constexpr int RW_RELU = OP_RELU;
constexpr int RW_BN_RELU = OP_BN + K_EW_BASE * OP_RELU;

template <int CODE>
struct RowsEw {
    static constexpr int n = ew_code_len(CODE);
    __host__ __device__ static constexpr int kind(int j) { return ew_code_kind(CODE, j); }
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
        } else if (EW::kind(j) == OP_LEAKY || EW::kind(j) == OP_CLAMP) {  // [slope, -] / [lo, hi]
            p.sc[j] = params[ew[j].arg];
            p.sh[j] = params[ew[j].arg + 1];
        }
    }
}

// Lists without a residual Add (it would need its own halo loads; such stacks take the LDS path).
template <int DT, class EW, int N>
BS_DEV void rows_apply(float (&x)[N], const RowsParams<EW> &p)
{
#pragma unroll
    for (int j = 0; j < EW::n; ++j) {
        if (EW::kind(j) == OP_BN) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = __builtin_fmaf(x[i], p.sc[j], p.sh[j]);
            round_store_all<DT, N>(x);
        } else if (EW::kind(j) == OP_LEAKY) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(x[i] > 0.0f ? x[i] : x[i] * p.sc[j]);
        } else if (EW::kind(j) == OP_CLAMP) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[i], p.sc[j]), p.sh[j]));
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

// code of an element-wise list without residual Add (first operation lowest digit), -1 otherwise
inline int rows_ew_code(const EwOp *ew, int n)
{
    int code = 0, mul = 1;
    for (int j = 0; j < n; ++j) {
        if (ew[j].kind == OP_ADD) return -1;
        code += ew[j].kind * mul;
        mul *= K_EW_BASE;
    }
    return code;
}

template <class P>
inline bool rows_pool_is(const PoolK &q)
{
    return q.kind == P::kind && q.kh == P::kh && q.kw == P::kw && q.sh == P::sh && q.sw == P::sw &&
           q.ph == P::ph && q.pw == P::pw;
}

// =============================================================================
// pool_rows_kernel: one pooling operation with overlapping or padded windows (plus the
// element-wise operations before and after it) without LDS: the "non-stacked" pooling
// building block of Section 4.4, where values pass from operation to operation directly
// (Section 4.1, single-step sequence).
//
// A lane owns one 128-bit column block of the input plane (VEC columns -> VO = VEC / sw
// outputs per output row) and walks down a chunk of rc output rows.  It keeps the kh input
// rows of the current windows in registers (after the leading element-wise operations), so
// every input row is loaded once per lane: per output row it loads only the sh new rows --
// one 128-bit vector each, plus the pw columns to the left and kw - sw - pw columns to the
// right of its block as scalar loads that hit the lines its neighbours fetch.  Cells outside
// the plane are the pooling operation's padding (-inf / +0) and are never computed from
// earlier layers.  A lane handles OR output rows per iteration and issues the loads for the
// next iteration before it reduces the current one.  Only the rows shared by two vertically
// adjacent chunks are read twice.
//
// The pooling shape and the element-wise lists are template arguments; the planner uses this
// kernel only for the signatures instantiated in the table at the end (rows_supported()).
template <int DT, int VEC, class P, int EWPRE, int EWPOST, bool WANT_IDX, int OR>
__global__ __launch_bounds__(256) void pool_rows_kernel(const PoolRowsK k)
{
    constexpr int KH = P::kh, KW = P::kw, SH = P::sh, SW = P::sw, PH = P::ph, PW = P::pw;
    constexpr int VO = VEC / SW;           // outputs per lane per output row
    constexpr int NL = PW;                 // columns left of the block
    constexpr int NX = KW - SW - PW;       // columns right of the block
    constexpr int NC = NL + VEC + NX;      // columns the VO windows span
    constexpr int WR = KH + (OR - 1) * SH;  // input rows of OR consecutive output rows
    constexpr int ST = OR * SH;             // rows the window slides per iteration
    constexpr int NS = ST < WR ? ST : WR;   // new input rows per iteration
    constexpr int ES = DT != DT_F32 ? 2 : 4;
    constexpr bool IS_MAX = P::kind == OP_MAXPOOL;
    static_assert(VEC % SW == 0 && NX >= 0 && NL >= 0, "unsupported pooling shape");
    using EWP = RowsEw<EWPRE>;
    using EWQ = RowsEw<EWPOST>;
    const float padv = IS_MAX ? -INFINITY : 0.0f;

    // lane -> (plane, chunk, column block j), column block fastest
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t t = fdiv(i, k.div_cbs);
    const int32_t j = (int32_t)(i - t * (uint32_t)k.cbs);
    const uint32_t plane = fdiv(t, k.div_chunks);
    const int32_t chunk = (int32_t)(t - plane * (uint32_t)k.chunks);
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c = (int32_t)(plane - img * (uint32_t)k.C);

    RowsParams<EWP> pp;
    RowsParams<EWQ> qp;
    rows_load_params<EWP>(k.pre, k.params, k.C, c, pp);
    rows_load_params<EWQ>(k.post, k.params, k.C, c, qp);

    const char *inp = static_cast<const char *>(image_base<DT>(k.in, img, k.in_extra)) +
                      (size_t)plane * (size_t)(k.H * k.W) * ES;
    void *outp = image_base<DT>(k.out, img, k.out_extra);
    const int32_t col0 = j * VEC;  // first column of the lane's block
    bool lin[NL > 0 ? NL : 1], xin[NX > 0 ? NX : 1];
#pragma unroll
    for (int n = 0; n < NL; ++n) lin[n] = col0 - NL + n >= 0;
#pragma unroll
    for (int n = 0; n < NX; ++n) xin[n] = col0 + VEC + n < k.W;

    struct RowRaw {
        Raw<DT, VEC> v;
        Raw<DT, 1> l[NL > 0 ? NL : 1], x[NX > 0 ? NX : 1];
        bool ok;
    };
    // issue the loads of input row ih (clamped to a safe address when the row is padding)
    auto fetch = [&](int32_t ih, RowRaw &r) {
        r.ok = ih >= 0 && ih < k.H;
        const uint32_t rowoff = r.ok ? (uint32_t)(ih * k.W) : 0u;
        r.v = load_raw<DT, VEC>(inp, rowoff + (uint32_t)col0);
#pragma unroll
        for (int n = 0; n < NL; ++n) r.l[n] = load_raw<DT, 1>(inp, lin[n] ? rowoff + (uint32_t)(col0 - NL + n) : 0u);
#pragma unroll
        for (int n = 0; n < NX; ++n) r.x[n] = load_raw<DT, 1>(inp, xin[n] ? rowoff + (uint32_t)(col0 + VEC + n) : 0u);
    };
    // registers -> window row: leading element-wise operations, then padding
    auto settle = [&](const RowRaw &r, float (&w)[NC]) {
        float xv[VEC];
        unpack<DT, VEC>(r.v, xv);
#pragma unroll
        for (int n = 0; n < VEC; ++n) w[NL + n] = xv[n];
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            float one[1];
            unpack<DT, 1>(r.l[n], one);
            w[n] = one[0];
        }
#pragma unroll
        for (int n = 0; n < NX; ++n) {
            float one[1];
            unpack<DT, 1>(r.x[n], one);
            w[NL + VEC + n] = one[0];
        }
        rows_apply<DT, EWP, NC>(w, pp);
#pragma unroll
        for (int n = 0; n < NL; ++n) w[n] = (r.ok && lin[n]) ? w[n] : padv;
#pragma unroll
        for (int n = 0; n < VEC; ++n) w[NL + n] = r.ok ? w[NL + n] : padv;
#pragma unroll
        for (int n = 0; n < NX; ++n) w[NL + VEC + n] = (r.ok && xin[n]) ? w[NL + VEC + n] : padv;
    };

    const int32_t oh0 = chunk * k.rc;
    const int32_t oh1 = live ? min(k.Ho, oh0 + k.rc) : oh0;
    const int32_t ow0 = j * VO;
    const bool vec_store = (k.Wo % VO) == 0 && ow0 + VO <= k.Wo;
    const uint32_t oplane = plane * (uint32_t)(k.Ho * k.Wo);

    // the window holds the input rows of OR consecutive output rows
    float win[WR][NC];
    {
        RowRaw r[WR];
#pragma unroll
        for (int w = 0; w < WR; ++w) fetch(oh0 * SH - PH + w, r[w]);
#pragma unroll
        for (int w = 0; w < WR; ++w) settle(r[w], win[w]);
    }
    for (int32_t oh = oh0; oh < oh1; oh += OR) {
        const int32_t h0 = oh * SH - PH;
        // loads for the next OR output rows first
        RowRaw nr[NS];
        const bool more = oh + OR < oh1;
        if (more) {
#pragma unroll
            for (int n = 0; n < NS; ++n) fetch(h0 + ST + (WR - NS) + n, nr[n]);
        }

#pragma unroll
        for (int o = 0; o < OR; ++o) {
            float y[VO];
            int32_t yi[VO];
            const int32_t hw = h0 + o * SH;  // first input row of this output row's windows
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                const int32_t w0 = col0 - PW + e * SW;
                if (IS_MAX) {
                    float best = -INFINITY;
                    int32_t bi = max(hw, 0) * k.W + max(w0, 0);  // first in-range cell
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            const float v = win[o * SH + dh][e * SW + dw];
                            if constexpr (WANT_IDX) {
                                const bool g = v > best;
                                best = g ? v : best;
                                bi = g ? (hw + dh) * k.W + w0 + dw : bi;
                            } else {
                                best = __builtin_fmaxf(best, v);
                            }
                        }
                    y[e] = best;
                    yi[e] = bi;
                } else {
                    float sum = 0.0f;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) sum = sum + win[o * SH + dh][e * SW + dw];
                    float inv = k.pool.inv_kk;
                    if (!k.pool.count_include_pad) {
                        const int32_t nr_ = min(hw + KH, k.H) - max(hw, 0);
                        const int32_t nc_ = min(w0 + KW, k.W) - max(w0, 0);
                        inv = 1.0f / (float)max(nr_ * nc_, 1);
                    } else if (k.pool.count_include_pad == 2) {  // ceil mode: cells inside the padded plane
                        const int32_t nr_ = min(hw + KH, k.H + PH) - hw;
                        const int32_t nc_ = min(w0 + KW, k.W + PW) - w0;
                        inv = 1.0f / (float)max(nr_ * nc_, 1);
                    }
                    y[e] = round_store<DT>(sum * inv);
                    yi[e] = 0;
                }
            }
            rows_apply<DT, EWQ, VO>(y, qp);
            if (oh + o < oh1) {
                const uint32_t ooff = oplane + (uint32_t)((oh + o) * k.Wo + ow0);
                if (vec_store) {
                    store_elems<DT, VO>(outp, ooff, y);
                    if constexpr (WANT_IDX) {
                        if (k.idx) store_indices<VO>(k.idx + ooff, yi);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < VO; ++e)
                        if (ow0 + e < k.Wo) {
                            const float one[1] = {y[e]};
                            store_elems<DT, 1>(outp, ooff + e, one);
                            if constexpr (WANT_IDX) {
                                if (k.idx) k.idx[ooff + e] = yi[e];
                            }
                        }
                }
            }
        }
        // slide the window down by OR * sh rows
#pragma unroll
        for (int w = 0; w + ST < WR; ++w)
#pragma unroll
            for (int n = 0; n < NC; ++n) win[w][n] = win[w + ST][n];
        if (more) {
#pragma unroll
            for (int n = 0; n < NS; ++n) settle(nr[n], win[WR - NS + n]);
        }
    }
}

// =============================================================================
// pool_rows2_kernel: two pooling operations in a row (each with element-wise operations
// around it) without LDS -- a two-step sequence of Section 4.1 whose intermediate values
// pass from step to step in registers instead of through the on-chip buffers of Section 4.4.
//
// A lane owns one 128-bit column block of the input plane (VEC columns -> VEC / (sw1 * sw2)
// final outputs per output row) and walks down a chunk of rc output rows.  It keeps two
// register windows: the kh1 level-0 rows (input after the leading element-wise operations)
// under the level-1 row being produced, and the kh2 level-1 rows (first pool's output after
// the middle element-wise operations) under the current output row.  Per output row it loads
// sh1 * sh2 new input rows, produces sh2 new level-1 rows and one output row.  Horizontally a
// lane recomputes the few level-1 columns its windows share with its neighbours, and reads
// the level-0 columns those need left and right of its block with scalar loads that hit the
// lines the neighbouring lanes fetch: lanes never exchange data, so there is no barrier.
//
// Cells outside a pooling operation's own input plane are that operation's padding
// (-inf for max, +0 for average) and are never computed from earlier layers.
template <int DT, int VEC, class P1, class P2, int EW0, int EW1, int EW2, bool WANT_IDX>
__global__ __launch_bounds__(256) void pool_rows2_kernel(const PoolRows2K k)
{
    constexpr int KH1 = P1::kh, KW1 = P1::kw, SH1 = P1::sh, SW1 = P1::sw, PH1 = P1::ph, PW1 = P1::pw;
    constexpr int KH2 = P2::kh, KW2 = P2::kw, SH2 = P2::sh, SW2 = P2::sw, PH2 = P2::ph, PW2 = P2::pw;
    constexpr int VB = VEC / SW1;                 // level-1 columns under the lane's block
    constexpr int VO = VB / SW2;                  // outputs per lane per output row
    constexpr int NC1 = (VO - 1) * SW2 + KW2;     // level-1 columns the VO windows span
    constexpr int NL = PW2 * SW1 + PW1;           // level-0 columns left of the block
    constexpr int NC0 = (NC1 - 1) * SW1 + KW1;    // level-0 columns the NC1 windows span
    constexpr int NX = NC0 - NL - VEC;            // level-0 columns right of the block
    constexpr int KEEP0 = KH1 - SH1;              // level-0 rows two consecutive level-1 rows share
    constexpr int KEEP1 = KH2 - SH2;              // level-1 rows two consecutive output rows share
    constexpr int R0 = (KH2 - 1) * SH1 + KH1;     // level-0 rows under one output row
    constexpr int NS0 = SH1 * SH2;                // new level-0 rows per output row
    constexpr int ES = DT != DT_F32 ? 2 : 4;
    constexpr int VPC = 16 / ES;                  // elements per 128-bit load
    constexpr int NV = VEC / VPC;                 // 128-bit loads per lane and row
    static_assert(VEC % VPC == 0, "a column block is a whole number of 128-bit vectors");
    constexpr bool MAX1 = P1::kind == OP_MAXPOOL, MAX2 = P2::kind == OP_MAXPOOL;
    static_assert(VEC % (SW1 * SW2) == 0 && NX >= 0 && KEEP0 >= 0 && KEEP1 >= 0, "unsupported pooling shapes");
    using E0 = RowsEw<EW0>;
    using E1 = RowsEw<EW1>;
    using E2 = RowsEw<EW2>;
    const float pad0 = MAX1 ? -INFINITY : 0.0f;  // value of a cell outside the level-0 plane
    const float pad1 = MAX2 ? -INFINITY : 0.0f;  // value of a cell outside the level-1 plane

    // lane -> (plane, chunk, column block j), column block fastest
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t t = fdiv(i, k.div_cbs);
    const int32_t j = (int32_t)(i - t * (uint32_t)k.cbs);
    const uint32_t plane = fdiv(t, k.div_chunks);
    const int32_t chunk = (int32_t)(t - plane * (uint32_t)k.chunks);
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c = (int32_t)(plane - img * (uint32_t)k.C);

    RowsParams<E0> p0;
    RowsParams<E1> p1;
    RowsParams<E2> p2;
    rows_load_params<E0>(k.pre, k.params, k.C, c, p0);
    rows_load_params<E1>(k.mid, k.params, k.C, c, p1);
    rows_load_params<E2>(k.post, k.params, k.C, c, p2);

    const char *inp = static_cast<const char *>(image_base<DT>(k.in, img, k.in_extra)) +
                      (size_t)plane * (size_t)(k.H * k.W) * ES;
    void *outp = image_base<DT>(k.out, img, k.out_extra);
    const int32_t col0 = j * VEC;            // first level-0 column of the lane's block
    const int32_t c1s = j * VB - PW2;        // first level-1 column the lane computes
    bool lin[NL > 0 ? NL : 1], xin[NX > 0 ? NX : 1], c1in[NC1];
#pragma unroll
    for (int n = 0; n < NL; ++n) lin[n] = col0 - NL + n >= 0;
#pragma unroll
    for (int n = 0; n < NX; ++n) xin[n] = col0 + VEC + n < k.W;
#pragma unroll
    for (int n = 0; n < NC1; ++n) c1in[n] = c1s + n >= 0 && c1s + n < k.W1;

    struct RowRaw {
        Raw<DT, VPC> v[NV];
        Raw<DT, 1> l[NL > 0 ? NL : 1], x[NX > 0 ? NX : 1];
        bool ok;
    };
    // issue the loads of input row ih (clamped to a safe address when the row is padding)
    auto fetch = [&](int32_t ih, RowRaw &r) {
        r.ok = ih >= 0 && ih < k.H;
        const uint32_t rowoff = r.ok ? (uint32_t)(ih * k.W) : 0u;
#pragma unroll
        for (int p = 0; p < NV; ++p) r.v[p] = load_raw<DT, VPC>(inp, rowoff + (uint32_t)(col0 + p * VPC));
#pragma unroll
        for (int n = 0; n < NL; ++n) r.l[n] = load_raw<DT, 1>(inp, lin[n] ? rowoff + (uint32_t)(col0 - NL + n) : 0u);
#pragma unroll
        for (int n = 0; n < NX; ++n) r.x[n] = load_raw<DT, 1>(inp, xin[n] ? rowoff + (uint32_t)(col0 + VEC + n) : 0u);
    };
    // registers -> level-0 row: leading element-wise operations, then the first pool's padding
    auto settle = [&](const RowRaw &r, float (&w)[NC0]) {
#pragma unroll
        for (int p = 0; p < NV; ++p) {
            float xv[VPC];
            unpack<DT, VPC>(r.v[p], xv);
#pragma unroll
            for (int n = 0; n < VPC; ++n) w[NL + p * VPC + n] = xv[n];
        }
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            float one[1];
            unpack<DT, 1>(r.l[n], one);
            w[n] = one[0];
        }
#pragma unroll
        for (int n = 0; n < NX; ++n) {
            float one[1];
            unpack<DT, 1>(r.x[n], one);
            w[NL + VEC + n] = one[0];
        }
        rows_apply<DT, E0, NC0>(w, p0);
#pragma unroll
        for (int n = 0; n < NL; ++n) w[n] = (r.ok && lin[n]) ? w[n] : pad0;
#pragma unroll
        for (int n = 0; n < VEC; ++n) w[NL + n] = r.ok ? w[NL + n] : pad0;
#pragma unroll
        for (int n = 0; n < NX; ++n) w[NL + VEC + n] = (r.ok && xin[n]) ? w[NL + VEC + n] : pad0;
    };
    // level-1 row r1 from the kh1 level-0 rows w0[0..KH1): first pool, middle element-wise
    // operations, then the second pool's padding
    auto level1 = [&](int32_t r1, const float (*w0)[NC0], float (&y)[NC1]) {
        const int32_t hw = r1 * SH1 - PH1;
#pragma unroll
        for (int n = 0; n < NC1; ++n) {
            if (MAX1) {
                float best = -INFINITY;
#pragma unroll
                for (int dh = 0; dh < KH1; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW1; ++dw) best = __builtin_fmaxf(best, w0[dh][n * SW1 + dw]);
                y[n] = best;
            } else {
                float sum = 0.0f;
#pragma unroll
                for (int dh = 0; dh < KH1; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW1; ++dw) sum = sum + w0[dh][n * SW1 + dw];
                float inv = k.pool1.inv_kk;
                if (k.pool1.count_include_pad != 1) {
                    const int32_t w0c = (c1s + n) * SW1 - PW1;
                    const bool padded = k.pool1.count_include_pad == 2;  // ceil mode: cells inside the padded plane
                    const int32_t nr_ = padded ? min(hw + KH1, k.H + PH1) - hw : min(hw + KH1, k.H) - max(hw, 0);
                    const int32_t nc_ = padded ? min(w0c + KW1, k.W + PW1) - w0c : min(w0c + KW1, k.W) - max(w0c, 0);
                    inv = 1.0f / (float)max(nr_ * nc_, 1);
                }
                y[n] = round_store<DT>(sum * inv);
            }
        }
        rows_apply<DT, E1, NC1>(y, p1);
        const bool rok = r1 >= 0 && r1 < k.H1;
#pragma unroll
        for (int n = 0; n < NC1; ++n) y[n] = (rok && c1in[n]) ? y[n] : pad1;
    };

    const int32_t oh0 = chunk * k.rc;
    const int32_t oh1 = live ? min(k.Ho, oh0 + k.rc) : oh0;
    const int32_t ow0 = j * VO;
    const bool vec_store = (k.Wo % VO) == 0 && ow0 + VO <= k.Wo;
    const uint32_t oplane = plane * (uint32_t)(k.Ho * k.Wo);

    float keep0[KEEP0 > 0 ? KEEP0 : 1][NC0];  // newest level-0 rows, shared with the next level-1 row
    float win1[KH2][NC1];                     // level-1 rows under the current output row
    {
        const int32_t r1f = oh0 * SH2 - PH2;   // first level-1 row of the first output row
        const int32_t h0f = r1f * SH1 - PH1;   // first level-0 row under it
        RowRaw r[R0];
#pragma unroll
        for (int w = 0; w < R0; ++w) fetch(h0f + w, r[w]);
        float l0[R0][NC0];
#pragma unroll
        for (int w = 0; w < R0; ++w) settle(r[w], l0[w]);
#pragma unroll
        for (int a = 0; a < KH2; ++a) level1(r1f + a, &l0[a * SH1], win1[a]);
#pragma unroll
        for (int w = 0; w < KEEP0; ++w)
#pragma unroll
            for (int n = 0; n < NC0; ++n) keep0[w][n] = l0[R0 - KEEP0 + w][n];
    }
    for (int32_t oh = oh0; oh < oh1; ++oh) {
        const int32_t r1w = oh * SH2 - PH2;              // first level-1 row of this output row's windows
        const int32_t r1n = r1w + KH2;                   // first new level-1 row of the next output row
        const int32_t h0n = (r1n - 1) * SH1 - PH1 + KH1;  // first new level-0 row of the next output row
        RowRaw nr[NS0];
        const bool more = oh + 1 < oh1;
        if (more) {
#pragma unroll
            for (int n = 0; n < NS0; ++n) fetch(h0n + n, nr[n]);
        }

        float y[VO];
        int32_t yi[VO];
#pragma unroll
        for (int e = 0; e < VO; ++e) {
            const int32_t w0 = c1s + e * SW2;  // first level-1 column of this output's window
            if (MAX2) {
                float best = -INFINITY;
                int32_t bi = max(r1w, 0) * k.W1 + max(w0, 0);  // first in-range cell
#pragma unroll
                for (int dh = 0; dh < KH2; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW2; ++dw) {
                        const float v = win1[dh][e * SW2 + dw];
                        if constexpr (WANT_IDX) {
                            const bool g = v > best;
                            best = g ? v : best;
                            bi = g ? (r1w + dh) * k.W1 + w0 + dw : bi;
                        } else {
                            best = __builtin_fmaxf(best, v);
                        }
                    }
                y[e] = best;
                yi[e] = bi;
            } else {
                float sum = 0.0f;
#pragma unroll
                for (int dh = 0; dh < KH2; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW2; ++dw) sum = sum + win1[dh][e * SW2 + dw];
                float inv = k.pool2.inv_kk;
                if (k.pool2.count_include_pad != 1) {
                    const bool padded = k.pool2.count_include_pad == 2;  // ceil mode: cells inside the padded plane
                    const int32_t nr_ = padded ? min(r1w + KH2, k.H1 + PH2) - r1w : min(r1w + KH2, k.H1) - max(r1w, 0);
                    const int32_t nc_ = padded ? min(w0 + KW2, k.W1 + PW2) - w0 : min(w0 + KW2, k.W1) - max(w0, 0);
                    inv = 1.0f / (float)max(nr_ * nc_, 1);
                }
                y[e] = round_store<DT>(sum * inv);
                yi[e] = 0;
            }
        }
        rows_apply<DT, E2, VO>(y, p2);
        {
            const uint32_t ooff = oplane + (uint32_t)(oh * k.Wo + ow0);
            if (vec_store) {
                store_elems<DT, VO, false>(outp, ooff, y);
                if constexpr (WANT_IDX) {
                    if (k.idx) store_indices<VO>(k.idx + ooff, yi);
                }
            } else {
#pragma unroll
                for (int e = 0; e < VO; ++e)
                    if (ow0 + e < k.Wo) {
                        const float one[1] = {y[e]};
                        store_elems<DT, 1, false>(outp, ooff + e, one);
                        if constexpr (WANT_IDX) {
                            if (k.idx) k.idx[ooff + e] = yi[e];
                        }
                    }
            }
        }
        // slide both windows down to the next output row
#pragma unroll
        for (int w = 0; w < KEEP1; ++w)
#pragma unroll
            for (int n = 0; n < NC1; ++n) win1[w][n] = win1[w + SH2][n];
        if (more) {
            float l0[KEEP0 + NS0][NC0];
#pragma unroll
            for (int w = 0; w < KEEP0; ++w)
#pragma unroll
                for (int n = 0; n < NC0; ++n) l0[w][n] = keep0[w][n];
#pragma unroll
            for (int n = 0; n < NS0; ++n) settle(nr[n], l0[KEEP0 + n]);
#pragma unroll
            for (int a = 0; a < SH2; ++a) level1(r1n + a, &l0[a * SH1], win1[KEEP1 + a]);
#pragma unroll
            for (int w = 0; w < KEEP0; ++w)
#pragma unroll
                for (int n = 0; n < NC0; ++n) keep0[w][n] = l0[NS0 + w][n];
        }
    }
}

}  // namespace bs
