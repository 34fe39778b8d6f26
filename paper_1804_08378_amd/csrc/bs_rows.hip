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
#include "bs_rows.h"

namespace bs {

template <bool BF16, int VEC, class P, int EWPRE, int EWPOST, bool WANT_IDX, int OR>
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
    constexpr int ES = BF16 ? 2 : 4;
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
    const int32_t c = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);

    RowsParams<EWP> pp;
    RowsParams<EWQ> qp;
    rows_load_params<EWP>(k.pre, k.params, k.C, c, pp);
    rows_load_params<EWQ>(k.post, k.params, k.C, c, qp);

    const char *inp = static_cast<const char *>(k.in) + (size_t)plane * (size_t)(k.H * k.W) * ES;
    const int32_t col0 = j * VEC;  // first column of the lane's block
    bool lin[NL > 0 ? NL : 1], xin[NX > 0 ? NX : 1];
#pragma unroll
    for (int n = 0; n < NL; ++n) lin[n] = col0 - NL + n >= 0;
#pragma unroll
    for (int n = 0; n < NX; ++n) xin[n] = col0 + VEC + n < k.W;

    struct RowRaw {
        Raw<BF16, VEC> v;
        Raw<BF16, 1> l[NL > 0 ? NL : 1], x[NX > 0 ? NX : 1];
        bool ok;
    };
    // issue the loads of input row ih (clamped to a safe address when the row is padding)
    auto fetch = [&](int32_t ih, RowRaw &r) {
        r.ok = ih >= 0 && ih < k.H;
        const uint32_t rowoff = r.ok ? (uint32_t)(ih * k.W) : 0u;
        r.v = load_raw<BF16, VEC>(inp, rowoff + (uint32_t)col0);
#pragma unroll
        for (int n = 0; n < NL; ++n) r.l[n] = load_raw<BF16, 1>(inp, lin[n] ? rowoff + (uint32_t)(col0 - NL + n) : 0u);
#pragma unroll
        for (int n = 0; n < NX; ++n) r.x[n] = load_raw<BF16, 1>(inp, xin[n] ? rowoff + (uint32_t)(col0 + VEC + n) : 0u);
    };
    // registers -> window row: leading element-wise operations, then padding
    auto settle = [&](const RowRaw &r, float (&w)[NC]) {
        float xv[VEC];
        unpack<BF16, VEC>(r.v, xv);
#pragma unroll
        for (int n = 0; n < VEC; ++n) w[NL + n] = xv[n];
#pragma unroll
        for (int n = 0; n < NL; ++n) {
            float one[1];
            unpack<BF16, 1>(r.l[n], one);
            w[n] = one[0];
        }
#pragma unroll
        for (int n = 0; n < NX; ++n) {
            float one[1];
            unpack<BF16, 1>(r.x[n], one);
            w[NL + VEC + n] = one[0];
        }
        rows_apply<BF16, EWP, NC>(w, pp);
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
                    }
                    y[e] = round_store<BF16>(sum * inv);
                    yi[e] = 0;
                }
            }
            rows_apply<BF16, EWQ, VO>(y, qp);
            if (oh + o < oh1) {
                const uint32_t ooff = oplane + (uint32_t)((oh + o) * k.Wo + ow0);
                if (vec_store) {
                    store_elems<BF16, VO>(k.out, ooff, y);
                    if constexpr (WANT_IDX) {
                        if (k.idx) {
#pragma unroll
                            for (int e = 0; e < VO; ++e) k.idx[ooff + e] = yi[e];
                        }
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < VO; ++e)
                        if (ow0 + e < k.Wo) {
                            const float one[1] = {y[e]};
                            store_elems<BF16, 1>(k.out, ooff + e, one);
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
// Signature table, applicability test and launcher.
// =============================================================================
// visit every instantiated signature; F(spec tag, pre code, post code) returns true to stop
template <class F>
static bool rows_for_each_signature(F &&f)
{
    return f(RMax3s2p1{}, std::integral_constant<int, RW_BN_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s2p1{}, std::integral_constant<int, RW_NONE>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s2p0{}, std::integral_constant<int, RW_BN_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s2p0{}, std::integral_constant<int, RW_NONE>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s2p0{}, std::integral_constant<int, RW_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s2p1{}, std::integral_constant<int, RW_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s1p1{}, std::integral_constant<int, RW_NONE>{}, std::integral_constant<int, RW_BN_RELU>{}) ||
           f(RMax3s1p1{}, std::integral_constant<int, RW_BN_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RMax3s1p1{}, std::integral_constant<int, RW_NONE>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RAvg3s1p1{}, std::integral_constant<int, RW_BN_RELU>{}, std::integral_constant<int, RW_NONE>{}) ||
           f(RAvg3s1p1{}, std::integral_constant<int, RW_NONE>{}, std::integral_constant<int, RW_NONE>{});
}

bool rows_supported(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post)
{
    const int cp = rows_ew_code(pre, n_pre), cq = rows_ew_code(post, n_post);
    if (cp < 0 || cq < 0) return false;
    return rows_for_each_signature([&](auto spec, auto pc, auto qc) {
        using P = decltype(spec);
        return rows_pool_is<P>(pool) && cp == decltype(pc)::value && cq == decltype(qc)::value;
    });
}

template <bool BF16, int VEC>
static bool rows_launch_t(const PoolRowsK &k, bool want_idx, dim3 grid, dim3 block, hipStream_t st)
{
    const int cp = rows_ew_code(k.pre, k.n_pre), cq = rows_ew_code(k.post, k.n_post);
    return rows_for_each_signature([&](auto spec, auto pc, auto qc) {
        using P = decltype(spec);
        constexpr int PC = decltype(pc)::value, QC = decltype(qc)::value;
        if (!rows_pool_is<P>(k.pool) || cp != PC || cq != QC) return false;
        if (want_idx) pool_rows_kernel<BF16, VEC, P, PC, QC, true, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        else pool_rows_kernel<BF16, VEC, P, PC, QC, false, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        return true;
    });
}

bs_status launch_rows(const PoolRowsK &k, bool bf16, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const bool want_idx = k.idx != nullptr && k.pool.kind == OP_MAXPOOL;
    const bool ok = bf16 ? rows_launch_t<true, 8>(k, want_idx, grid, block, st)
                         : rows_launch_t<false, 4>(k, want_idx, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
