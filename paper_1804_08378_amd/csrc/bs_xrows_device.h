// Device code of the sliding-window pooling kernels whose lanes exchange their edge columns
// inside the wave: the one-level kernel (one pooling operation with overlapping or padded
// windows) and the two-level kernel (two pooling operations in a row), for planes whose rows
// fit into one wave (at most 64 column blocks).
//
// Both are register-only versions of Section 4.4's pooling building blocks (values pass from
// operation to operation without the on-chip buffers; Section 4.1, single- and two-step
// sequences).  A lane owns one column block of the input plane (VEC columns, whole 128-bit
// vectors) and walks down a chunk of output rows with the rows of the current windows in
// registers, so every input element is loaded by exactly one lane.  The columns a window needs
// left and right of the block are the neighbouring lanes' edge columns *after* their
// element-wise operations (and, in the two-level kernel, after their first pooling operation):
// they arrive by one data-parallel-primitive move each (wave_shr / wave_shl by one lane)
// instead of being loaded and recomputed.  For that, all column blocks of a row sit in
// consecutive lanes of one wave: a wave holds spw = 64 / cbs (plane, chunk) segments of cbs
// lanes each, the remaining lanes idle, and every lane of a wave runs the same number of
// iterations whether or not its rows exist, so a neighbour's value is always the one of the
// same row.  Cells outside a pooling operation's own input plane are that operation's padding
// (-inf for max, +0 for average) and are never computed from earlier layers.
//
// A max pooling without index output takes the maximum down the window's rows first, on the
// lane's own columns, and exchanges that one row of column maxima; the order of a maximum
// does not change its value (v_max_f32 orders -0 below +0 whichever operand comes first).
// Sums and index-producing scans keep the row-major order of the layer definition and
// exchange the edge columns of every row.
//
// With 16-bit storage a layer's float32 result is rounded to the storage type.  Rounding to
// nearest is monotone and keeps zero and the sign, so it commutes with ReLU and with a
// maximum: where a max pooling without index output follows, the last rounding before it
// (of the element-wise list, or of an average in front of it) is left out and the maximum is
// rounded instead -- the same bits from a quarter of the conversions.
//
// Measured on MI355X: a wave issues at most one vector instruction per eight cycles, a SIMD
// one per 3.5 .. 5 cycles, scalar and branch instructions take comparable issue time, and
// these kernels are bound by that issue rate, not by memory latency: requesting rows several
// iterations ahead, a separate interior version of the loop body without padding tests,
// wider column blocks and non-temporal loads were all measured and gained nothing.
#pragma once
#include "bs_rows_device.h"

namespace bs {

// value of the same register in lane - 1 / lane + 1 of the wave (lane 0 / lane 63: zero bits)
BS_DEV float from_left_lane(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_mov_dpp((int)__float_as_uint(v), 0x138, 0xf, 0xf, true));  // wave_shr:1
}
BS_DEV float from_right_lane(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_mov_dpp((int)__float_as_uint(v), 0x130, 0xf, 0xf, true));  // wave_shl:1
}

// own[V] -> full[NL + V + NX]: the lane's columns with the NL columns before them (the left
// neighbour's last ones) and the NX after them (the right neighbour's first ones); beyond the
// ends of the row: pad.  Must be reached by all lanes of the wave.
template <int V, int NL, int NX>
BS_DEV void with_neighbours(const float (&own)[V], float (&full)[NL + V + NX], bool has_left, bool has_right, float pad)
{
    static_assert(NL <= V && NX <= V, "edge columns come from the adjacent lane only");
#pragma unroll
    for (int n = 0; n < NL; ++n) {
        const float t = from_left_lane(own[V - NL + n]);
        full[n] = has_left ? t : pad;
    }
#pragma unroll
    for (int n = 0; n < V; ++n) full[NL + n] = own[n];
#pragma unroll
    for (int n = 0; n < NX; ++n) {
        const float t = from_right_lane(own[n]);
        full[NL + V + n] = has_right ? t : pad;
    }
}

// lane -> (segment of the wave, column block); segment -> (plane, chunk).  Lanes without
// work of their own shadow the wave's first segment.
struct XLane {
    uint32_t plane, img;
    int32_t chunk, j, c;
    bool live;
};
template <class K>
BS_DEV XLane xrows_lane(const K &k)
{
    XLane x;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const uint32_t seg = fdiv(lane, k.div_cbs);
    x.j = (int32_t)(lane - seg * (uint32_t)k.cbs);
    uint32_t u = wave * (uint32_t)k.spw + seg;
    x.live = seg < (uint32_t)k.spw && u < k.units;
    if (!x.live) u = wave * (uint32_t)k.spw < k.units ? wave * (uint32_t)k.spw : 0u;
    x.plane = fdiv(u, k.div_chunks);
    x.chunk = (int32_t)(u - x.plane * (uint32_t)k.chunks);
    x.img = fdiv(x.plane, k.div_c);
    x.c = (int32_t)(x.plane - x.img * (uint32_t)k.C);
    return x;
}

template <int DT, int VEC>
struct XRowRaw {
    static constexpr int VPC = 16 / (DT != DT_F32 ? 2 : 4);  // elements per 128-bit load
    static constexpr int NV = VEC / VPC;
    Raw<DT, VPC> v[NV];
};

// issue the loads of the lane's block of input row ih, clamped into the plane (a row outside
// the plane is padding: its values are replaced when the row is settled)
template <int DT, int VEC>
BS_DEV void xrows_fetch(const char *inp, int32_t ih, int32_t H, int32_t W, int32_t col0, XRowRaw<DT, VEC> &r)
{
    using R = XRowRaw<DT, VEC>;
    const int32_t row = min(max(ih, 0), H - 1);
    const uint32_t off = (uint32_t)(row * W + col0);
#pragma unroll
    for (int p = 0; p < R::NV; ++p) r.v[p] = load_raw<DT, R::VPC>(inp, off + (uint32_t)(p * R::VPC));
}

template <int DT, int VEC>
BS_DEV void xrows_unpack(const XRowRaw<DT, VEC> &r, float (&x)[VEC])
{
    using R = XRowRaw<DT, VEC>;
#pragma unroll
    for (int p = 0; p < R::NV; ++p) {
        float xv[R::VPC];
        unpack<DT, R::VPC>(r.v[p], xv);
#pragma unroll
        for (int n = 0; n < R::VPC; ++n) x[p * R::VPC + n] = xv[n];
    }
}

// bfloat16 storage, index-producing scans: the rounded values of a settled row are used by every window that holds
// them.  Left to itself the compiler repeats the conversions at the uses; a value the optimiser cannot look into is
// converted once (measured on the ResNet stem with indices: 51 -> 42 us; binary16 gains nothing from it).
template <int DT, bool WANT_IDX, int N>
BS_DEV void xrows_pin(float (&x)[N])
{
    if constexpr (WANT_IDX && DT == DT_BF16) {
#pragma unroll
        for (int n = 0; n < N; ++n) asm("" : "+v"(x[n]));
    }
}

// Does this element-wise list end in a ReLU?  Its results are then never -0, and a sum over
// them may start from its first term instead of +0 with the same bits.
template <class EW>
constexpr bool ends_in_relu()
{
    return EW::n > 0 && EW::kind(EW::n > 0 ? EW::n - 1 : 0) == OP_RELU;
}

// row-major sum of a KH x KW window whose first column is w[.][c0]; from +0 unless the terms are never -0
template <int KH, int KW, bool NONNEG, int NC>
BS_DEV float xrows_window_sum(const float (*w)[NC], int c0)
{
    float sum = NONNEG ? w[0][c0] : 0.0f + w[0][c0];
#pragma unroll
    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
        for (int dw = 0; dw < KW; ++dw)
            if (dh + dw > 0) sum = sum + w[dh][c0 + dw];
    return sum;
}

// sums of N adjacent windows (first row h0, first columns w0, w0 + SW, ...) of an H x W plane
// -> averages: times the reciprocal of the divisor, rounded to the storage type (unless the
// caller rounds later)
template <int DT, int N, int KH, int KW, int SW, int PH, int PW, bool ROUND = true>
BS_DEV void xrows_normalise(float (&v)[N], const PoolK &p, int32_t h0, int32_t w0, int32_t H, int32_t W)
{
    if (p.count_include_pad == 1) {  // the same for every lane
#pragma unroll
        for (int n = 0; n < N; ++n) v[n] = ROUND ? round_store<DT>(v[n] * p.inv_kk) : v[n] * p.inv_kk;
    } else {
        const bool padded = p.count_include_pad == 2;  // ceil mode: cells inside the padded plane
        const int32_t nr_ = padded ? min(h0 + KH, H + PH) - h0 : min(h0 + KH, H) - max(h0, 0);
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int32_t c = w0 + n * SW;
            const int32_t nc_ = padded ? min(c + KW, W + PW) - c : min(c + KW, W) - max(c, 0);
            const float t = v[n] * (1.0f / (float)max(nr_ * nc_, 1));
            v[n] = ROUND ? round_store<DT>(t) : t;
        }
    }
}

// store the lane's VO outputs of one output row (and their indices) where pred holds
// NT: non-temporal stores.  Measured: 3 % faster in the one-level kernel (float32), 4 % slower in the
// two-level kernel, whose output rows of 28 elements leave partial cache lines that plain stores let
// the L2 cache complete before they go to memory (HBM write counter: 1.42 x the output with
// non-temporal stores).
template <int DT, int VO, bool WANT_IDX, bool NT>
BS_DEV void xrows_store(void *outp, int32_t *idx, uint32_t ooff, const float (&y)[VO], const int32_t (&yi)[VO], bool all_vec,
                        int32_t ow0, int32_t Wo, bool pred)
{
    if (all_vec) {  // the same for every lane: every lane's outputs are one aligned vector inside the row
        if (pred) {
            store_elems<DT, VO, NT>(outp, ooff, y);
            if constexpr (WANT_IDX) {
                if (idx) store_indices<VO>(idx + ooff, yi);
            }
        }
    } else if (pred) {
#pragma unroll
        for (int e = 0; e < VO; ++e)
            if (ow0 + e < Wo) {
                const float one[1] = {y[e]};
                store_elems<DT, 1, NT>(outp, ooff + e, one);
                if constexpr (WANT_IDX) {
                    if (idx) idx[ooff + e] = yi[e];
                }
            }
    }
}

// Element-wise list with the rounding of its last rounding operation left out (the caller rounds
// later, after operations that commute with rounding): everything after that operation is ReLU.
template <int DT, class EW, int N, bool DEFER>
BS_DEV void xrows_apply(float (&x)[N], const RowsParams<EW> &p)
{
    if constexpr (!DEFER || DT == DT_F32) {
        rows_apply<DT, EW, N>(x, p);
    } else {
        constexpr int last = [] {
            int l = -1;
            for (int j = 0; j < EW::n; ++j)
                if (EW::kind(j) != OP_RELU) l = j;
            return l;
        }();
#pragma unroll
        for (int j = 0; j < EW::n; ++j) {
            if (EW::kind(j) == OP_BN) {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    const float t = __builtin_fmaf(x[i], p.sc[j], p.sh[j]);
                    x[i] = j == last ? t : round_store<DT>(t);
                }
            } else if (EW::kind(j) == OP_LEAKY) {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    const float t = x[i] > 0.0f ? x[i] : x[i] * p.sc[j];
                    x[i] = j == last ? t : round_store<DT>(t);
                }
            } else if (EW::kind(j) == OP_CLAMP) {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    const float t = __builtin_fminf(__builtin_fmaxf(x[i], p.sc[j]), p.sh[j]);
                    x[i] = j == last ? t : round_store<DT>(t);
                }
            } else {
#pragma unroll
                for (int i = 0; i < N; ++i) x[i] = __builtin_fmaxf(x[i], 0.0f);  // NaN, -0 -> +0
            }
        }
    }
}

// does the list hold an operation whose result is rounded to the storage type?
template <class EW>
constexpr bool has_rounding()
{
    for (int j = 0; j < EW::n; ++j)
        if (EW::kind(j) != OP_RELU) return true;
    return false;
}

// =============================================================================
// pool_xrows_kernel: one pooling operation, the element-wise lists before and after it.
// OR output rows per iteration; a chunk is k.rc output rows (a multiple of OR).
// =============================================================================
template <int DT, int VEC, class P, int EWPRE, int EWPOST, bool WANT_IDX, int OR>
__global__ __launch_bounds__(256) void pool_xrows_kernel(const PoolRowsK k)
{
    constexpr int KH = P::kh, KW = P::kw, SH = P::sh, SW = P::sw, PH = P::ph, PW = P::pw;
    constexpr int VO = VEC / SW;            // outputs per lane per output row
    constexpr int NL = PW;                  // columns left of the block
    constexpr int NX = KW - SW - PW;        // columns right of the block
    constexpr int WR = KH + (OR - 1) * SH;  // input rows of OR consecutive output rows
    constexpr int ST = OR * SH;             // rows the window slides per iteration
    constexpr int NS = ST < WR ? ST : WR;   // new input rows per iteration
    constexpr int ES = DT != DT_F32 ? 2 : 4;
    constexpr bool IS_MAX = P::kind == OP_MAXPOOL;
    constexpr bool VF = IS_MAX && !WANT_IDX;        // maximum down the rows first, then one exchange
    constexpr int CW = VF ? VEC : NL + VEC + NX;    // columns kept per window row
    static_assert(VEC % SW == 0 && NX >= 0 && NL >= 0 && NL <= VEC && NX <= VEC, "unsupported pooling shape");
    using EWP = RowsEw<EWPRE>;
    using EWQ = RowsEw<EWPOST>;
    using Row = XRowRaw<DT, VEC>;
    constexpr bool NONNEG = ends_in_relu<EWP>();
    constexpr bool DEFER = VF && DT != DT_F32 && has_rounding<EWP>();  // round the maximum instead of the list's last result
    const float padv = IS_MAX ? -INFINITY : 0.0f;

    const XLane L = xrows_lane(k);
    RowsParams<EWP> pp;
    RowsParams<EWQ> qp;
    rows_load_params<EWP>(k.pre, k.params, k.C, L.c, pp);
    rows_load_params<EWQ>(k.post, k.params, k.C, L.c, qp);

    const char *inp = static_cast<const char *>(image_base<DT>(k.in, L.img, k.in_extra)) +
                      (size_t)L.plane * (size_t)(k.H * k.W) * ES;
    void *outp = image_base<DT>(k.out, L.img, k.out_extra);
    const int32_t col0 = L.j * VEC;
    const bool has_left = L.j > 0, has_right = L.j + 1 < k.cbs;

    // registers -> window row: leading element-wise operations, padding rows, edge columns
    auto settle = [&](const Row &r, int32_t ih, float (&w)[CW]) {
        float x[VEC];
        xrows_unpack<DT, VEC>(r, x);
        xrows_apply<DT, EWP, VEC, DEFER>(x, pp);
        xrows_pin<DT, WANT_IDX>(x);
        const bool ok = ih >= 0 && ih < k.H;
#pragma unroll
        for (int n = 0; n < VEC; ++n) x[n] = ok ? x[n] : padv;
        if constexpr (VF) {
#pragma unroll
            for (int n = 0; n < VEC; ++n) w[n] = x[n];
        } else {
            with_neighbours<VEC, NL, NX>(x, w, has_left, has_right, padv);
        }
    };

    const int32_t oh0 = L.chunk * k.rc;
    const int32_t ow0 = L.j * VO;
    const bool all_vec = (k.Wo % VO) == 0 && k.cbs * VO <= k.Wo;
    const uint32_t oplane = L.plane * (uint32_t)(k.Ho * k.Wo);

    // The rows of the next iteration that this one does not have are requested before this
    // iteration's windows are reduced, and settled after.
    const int32_t iters = k.rc / OR;  // the same for every lane
    auto new_row = [&](int32_t j, int n) { return (oh0 + j * OR) * SH - PH + (WR - NS) + n; };  // n-th new row of iteration j
    float win[WR][CW];
    {
        Row r[WR];
        const int32_t hf = oh0 * SH - PH;
#pragma unroll
        for (int w = 0; w < WR; ++w) xrows_fetch<DT, VEC>(inp, hf + w, k.H, k.W, col0, r[w]);
#pragma unroll
        for (int w = 0; w < WR; ++w) settle(r[w], hf + w, win[w]);
    }
    for (int32_t it = 0; it < iters; ++it) {
        const int32_t oh = oh0 + it * OR;
        const int32_t h0 = oh * SH - PH;
        const bool more = it + 1 < iters;  // the same for every lane
        Row nr[NS];
        if (more) {
#pragma unroll
            for (int n = 0; n < NS; ++n) xrows_fetch<DT, VEC>(inp, new_row(it + 1, n), k.H, k.W, col0, nr[n]);
        }

#pragma unroll
        for (int o = 0; o < OR; ++o) {
            float y[VO];
            int32_t yi[VO];
            const int32_t hw = h0 + o * SH;  // first input row of this output row's windows
            if constexpr (VF) {
                float m[VEC], full[NL + VEC + NX];
#pragma unroll
                for (int n = 0; n < VEC; ++n) {
                    m[n] = win[o * SH][n];
#pragma unroll
                    for (int dh = 1; dh < KH; ++dh) m[n] = __builtin_fmaxf(m[n], win[o * SH + dh][n]);
                }
                with_neighbours<VEC, NL, NX>(m, full, has_left, has_right, padv);
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    float best = full[e * SW];
#pragma unroll
                    for (int dw = 1; dw < KW; ++dw) best = __builtin_fmaxf(best, full[e * SW + dw]);
                    y[e] = DEFER ? round_store<DT>(best) : best;
                    yi[e] = 0;
                }
            } else if constexpr (IS_MAX) {
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    const int32_t w0 = col0 - PW + e * SW;
                    float best = -INFINITY;
                    int32_t bi = max(hw, 0) * k.W + max(w0, 0);  // first in-range cell
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            const float v = win[o * SH + dh][e * SW + dw];
                            const bool g = v > best;
                            best = g ? v : best;
                            bi = g ? (hw + dh) * k.W + w0 + dw : bi;
                        }
                    y[e] = best;
                    yi[e] = bi;
                }
            } else {
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    y[e] = xrows_window_sum<KH, KW, NONNEG, CW>(&win[o * SH], e * SW);
                    yi[e] = 0;
                }
                xrows_normalise<DT, VO, KH, KW, SW, PH, PW>(y, k.pool, hw, col0 - PW, k.H, k.W);
            }
            rows_apply<DT, EWQ, VO>(y, qp);
            const uint32_t ooff = oplane + (uint32_t)((oh + o) * k.Wo + ow0);
            xrows_store<DT, VO, WANT_IDX, true>(outp, k.idx, ooff, y, yi, all_vec, ow0, k.Wo, L.live && oh + o < k.Ho);
        }
        // slide the window down by OR * sh rows
#pragma unroll
        for (int w = 0; w + ST < WR; ++w)
#pragma unroll
            for (int n = 0; n < CW; ++n) win[w][n] = win[w + ST][n];
        if (more) {
#pragma unroll
            for (int n = 0; n < NS; ++n) settle(nr[n], new_row(it + 1, n), win[WR - NS + n]);
        }
    }
}

// =============================================================================
// pool_xrows2_kernel: pre, pool 1, mid, pool 2, post.  The lane keeps the kh1 - sh1 newest
// level-0 rows (input after the leading element-wise operations) and the kh2 level-1 rows
// (first pool's output after the middle operations) under the current output row; per output
// row it loads sh1 * sh2 new input rows and produces sh2 level-1 rows and one output row.
// PLAIN: the launcher has checked that every average divides by kh * kw, that no lane's level-1 columns reach
// past the plane and that every lane's outputs of a row are one aligned vector (xrows2_is_plain): the tests of
// these conditions, the same for all lanes and rows, are then not in the loop.
// =============================================================================
template <int DT, int VEC, class P1, class P2, int EW0, int EW1, int EW2, bool WANT_IDX, bool PLAIN = false>
__global__ __launch_bounds__(256) void pool_xrows2_kernel(const PoolRows2K k)
{
    constexpr int KH1 = P1::kh, KW1 = P1::kw, SH1 = P1::sh, SW1 = P1::sw, PH1 = P1::ph, PW1 = P1::pw;
    constexpr int KH2 = P2::kh, KW2 = P2::kw, SH2 = P2::sh, SW2 = P2::sw, PH2 = P2::ph, PW2 = P2::pw;
    constexpr int VB = VEC / SW1;                 // level-1 columns of the lane
    constexpr int VO = VB / SW2;                  // outputs per lane per output row
    constexpr int NL0 = PW1, NX0 = KW1 - SW1 - PW1;  // level-0 columns of the neighbours the lane's level-1 columns need
    constexpr int NL1 = PW2, NX1 = KW2 - SW2 - PW2;  // level-1 columns of the neighbours the lane's outputs need
    constexpr int KEEP0 = KH1 - SH1;              // level-0 rows two consecutive level-1 rows share
    constexpr int KEEP1 = KH2 - SH2;              // level-1 rows two consecutive output rows share
    constexpr int R0 = (KH2 - 1) * SH1 + KH1;     // level-0 rows under one output row
    constexpr int NS0 = SH1 * SH2;                // new level-0 rows per output row
    constexpr int ES = DT != DT_F32 ? 2 : 4;
    constexpr bool MAX1 = P1::kind == OP_MAXPOOL, MAX2 = P2::kind == OP_MAXPOOL;
    constexpr bool VF1 = MAX1, VF2 = MAX2 && !WANT_IDX;  // maximum down the rows first, then one exchange
    constexpr int C0 = VF1 ? VEC : NL0 + VEC + NX0;      // columns kept per level-0 row
    constexpr int C1 = VF2 ? VB : NL1 + VB + NX1;        // columns kept per level-1 row
    static_assert(VEC % (SW1 * SW2) == 0 && NX0 >= 0 && NX1 >= 0 && KEEP0 >= 0 && KEEP1 >= 0 && NL0 <= VEC &&
                      NX0 <= VEC && NL1 <= VB && NX1 <= VB,
                  "unsupported pooling shapes");
    using E0 = RowsEw<EW0>;
    using E1 = RowsEw<EW1>;
    using E2 = RowsEw<EW2>;
    using Row = XRowRaw<DT, VEC>;
    constexpr bool NONNEG0 = ends_in_relu<E0>(), NONNEG1 = ends_in_relu<E1>();
    // 16-bit storage, a maximum without indices last: the last rounding in front of it -- of the
    // middle list, else of an average as first pool -- moves behind it
    constexpr bool DEFER_E1 = VF2 && DT != DT_F32 && has_rounding<E1>();
    constexpr bool DEFER_AVG = VF2 && DT != DT_F32 && !has_rounding<E1>() && !MAX1;
    const float pad0 = MAX1 ? -INFINITY : 0.0f;  // value of a cell outside the level-0 plane
    const float pad1 = MAX2 ? -INFINITY : 0.0f;  // value of a cell outside the level-1 plane

    const XLane L = xrows_lane(k);
    RowsParams<E0> p0;
    RowsParams<E1> p1;
    RowsParams<E2> p2;
    rows_load_params<E0>(k.pre, k.params, k.C, L.c, p0);
    rows_load_params<E1>(k.mid, k.params, k.C, L.c, p1);
    rows_load_params<E2>(k.post, k.params, k.C, L.c, p2);

    const char *inp = static_cast<const char *>(image_base<DT>(k.in, L.img, k.in_extra)) +
                      (size_t)L.plane * (size_t)(k.H * k.W) * ES;
    void *outp = image_base<DT>(k.out, L.img, k.out_extra);
    const int32_t col0 = L.j * VEC;  // first level-0 column of the lane
    const int32_t c10 = L.j * VB;    // first level-1 column of the lane
    const bool has_left = L.j > 0, has_right = L.j + 1 < k.cbs;
    const bool ragged1 = !PLAIN && k.W1 < k.cbs * VB;  // the last lane's level-1 columns reach past the plane

    // registers -> level-0 row: leading element-wise operations, the first pool's padding
    auto settle = [&](const Row &r, int32_t ih, float (&w)[C0]) {
        float x[VEC];
        xrows_unpack<DT, VEC>(r, x);
        rows_apply<DT, E0, VEC>(x, p0);
        xrows_pin<DT, WANT_IDX>(x);
        const bool ok = ih >= 0 && ih < k.H;
#pragma unroll
        for (int n = 0; n < VEC; ++n) x[n] = ok ? x[n] : pad0;
        if constexpr (VF1) {
#pragma unroll
            for (int n = 0; n < VEC; ++n) w[n] = x[n];
        } else {
            with_neighbours<VEC, NL0, NX0>(x, w, has_left, has_right, pad0);
        }
    };
    // level-1 row r1 from the kh1 level-0 rows w0[0..KH1): first pool, middle element-wise
    // operations, the second pool's padding
    auto level1 = [&](int32_t r1, const float (*w0)[C0], float (&y)[C1]) {
        float v[VB];
        if constexpr (VF1) {
            float m[VEC], full[NL0 + VEC + NX0];
#pragma unroll
            for (int n = 0; n < VEC; ++n) {
                m[n] = w0[0][n];
#pragma unroll
                for (int dh = 1; dh < KH1; ++dh) m[n] = __builtin_fmaxf(m[n], w0[dh][n]);
            }
            with_neighbours<VEC, NL0, NX0>(m, full, has_left, has_right, pad0);
#pragma unroll
            for (int n = 0; n < VB; ++n) {
                float best = full[n * SW1];
#pragma unroll
                for (int dw = 1; dw < KW1; ++dw) best = __builtin_fmaxf(best, full[n * SW1 + dw]);
                v[n] = best;
            }
        } else {
#pragma unroll
            for (int n = 0; n < VB; ++n) v[n] = xrows_window_sum<KH1, KW1, NONNEG0, C0>(w0, n * SW1);
            if constexpr (PLAIN) {
#pragma unroll
                for (int n = 0; n < VB; ++n) v[n] = DEFER_AVG ? v[n] * k.pool1.inv_kk : round_store<DT>(v[n] * k.pool1.inv_kk);
            } else {
                xrows_normalise<DT, VB, KH1, KW1, SW1, PH1, PW1, !DEFER_AVG>(v, k.pool1, r1 * SH1 - PH1, col0 - PW1, k.H, k.W);
            }
        }
        xrows_apply<DT, E1, VB, DEFER_E1>(v, p1);
        const bool rok = r1 >= 0 && r1 < k.H1;
#pragma unroll
        for (int n = 0; n < VB; ++n) v[n] = rok ? v[n] : pad1;
        if (ragged1) {  // the same for every lane
#pragma unroll
            for (int n = 0; n < VB; ++n) v[n] = c10 + n < k.W1 ? v[n] : pad1;
        }
        if constexpr (VF2) {
#pragma unroll
            for (int n = 0; n < VB; ++n) y[n] = v[n];
        } else {
            with_neighbours<VB, NL1, NX1>(v, y, has_left, has_right, pad1);
        }
    };

    const int32_t oh0 = L.chunk * k.rc;
    const int32_t ow0 = L.j * VO;
    const bool all_vec = PLAIN || ((k.Wo % VO) == 0 && k.cbs * VO <= k.Wo);
    const uint32_t oplane = L.plane * (uint32_t)(k.Ho * k.Wo);

    auto new_l1 = [&](int32_t t) { return (oh0 + t - 1) * SH2 - PH2 + KH2; };    // first level-1 row output row t adds
    auto new_l0 = [&](int32_t t) { return (new_l1(t) - 1) * SH1 - PH1 + KH1; };  // first level-0 row it adds
    float keep0[KEEP0 > 0 ? KEEP0 : 1][C0];  // newest level-0 rows, shared with the next level-1 row
    float win1[KH2][C1];                     // level-1 rows under the current output row
    {
        const int32_t r1f = oh0 * SH2 - PH2;   // first level-1 row of the first output row
        const int32_t h0f = r1f * SH1 - PH1;   // first level-0 row under it
        Row r[R0];
#pragma unroll
        for (int w = 0; w < R0; ++w) xrows_fetch<DT, VEC>(inp, h0f + w, k.H, k.W, col0, r[w]);
        float l0[R0][C0];
#pragma unroll
        for (int w = 0; w < R0; ++w) settle(r[w], h0f + w, l0[w]);
#pragma unroll
        for (int a = 0; a < KH2; ++a) level1(r1f + a, &l0[a * SH1], win1[a]);
#pragma unroll
        for (int w = 0; w < KEEP0; ++w)
#pragma unroll
            for (int n = 0; n < C0; ++n) keep0[w][n] = l0[R0 - KEEP0 + w][n];
    }
    // output row t of the chunk from the level-1 rows under it
    auto reduce = [&](int32_t t, float (&y)[VO], int32_t (&yi)[VO]) {
        const int32_t r1w = (oh0 + t) * SH2 - PH2;  // first level-1 row of this output row's windows
        if constexpr (VF2) {
            float m[VB], full[NL1 + VB + NX1];
#pragma unroll
            for (int n = 0; n < VB; ++n) {
                m[n] = win1[0][n];
#pragma unroll
                for (int dh = 1; dh < KH2; ++dh) m[n] = __builtin_fmaxf(m[n], win1[dh][n]);
            }
            with_neighbours<VB, NL1, NX1>(m, full, has_left, has_right, pad1);
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                float best = full[e * SW2];
#pragma unroll
                for (int dw = 1; dw < KW2; ++dw) best = __builtin_fmaxf(best, full[e * SW2 + dw]);
                y[e] = (DEFER_E1 || DEFER_AVG) ? round_store<DT>(best) : best;
                yi[e] = 0;
            }
        } else if constexpr (MAX2) {
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                const int32_t w0 = c10 - PW2 + e * SW2;  // first level-1 column of this output's window
                float best = -INFINITY;
                int32_t bi = max(r1w, 0) * k.W1 + max(w0, 0);  // first in-range cell
#pragma unroll
                for (int dh = 0; dh < KH2; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW2; ++dw) {
                        const float v = win1[dh][e * SW2 + dw];
                        const bool g = v > best;
                        best = g ? v : best;
                        bi = g ? (r1w + dh) * k.W1 + w0 + dw : bi;
                    }
                y[e] = best;
                yi[e] = bi;
            }
        } else {
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                y[e] = xrows_window_sum<KH2, KW2, NONNEG1, C1>(win1, e * SW2);
                yi[e] = 0;
            }
            if constexpr (PLAIN) {
#pragma unroll
                for (int e = 0; e < VO; ++e) y[e] = round_store<DT>(y[e] * k.pool2.inv_kk);
            } else {
                xrows_normalise<DT, VO, KH2, KW2, SW2, PH2, PW2>(y, k.pool2, r1w, c10 - PW2, k.H1, k.W1);
            }
        }
        rows_apply<DT, E2, VO>(y, p2);
    };
    auto put = [&](int32_t t, const float (&y)[VO], const int32_t (&yi)[VO]) {
        const int32_t oh = oh0 + t;
        xrows_store<DT, VO, WANT_IDX, false>(outp, k.idx, oplane + (uint32_t)(oh * k.Wo + ow0), y, yi, all_vec, ow0, k.Wo,
                                             L.live && oh < k.Ho);
    };
    // One output row, and both windows slid down to the next: the NS0 input rows the next row adds are requested
    // before this row is reduced and settled after; the row's store comes last, so that the wait for the requested
    // rows has only a store issued a whole row earlier in front of them.
    auto step = [&](int32_t t) {
        Row nr[NS0];
        const int32_t r1n = new_l1(t + 1), h0n = new_l0(t + 1);
#pragma unroll
        for (int n = 0; n < NS0; ++n) xrows_fetch<DT, VEC>(inp, h0n + n, k.H, k.W, col0, nr[n]);
        float y[VO];
        int32_t yi[VO];
        reduce(t, y, yi);
#pragma unroll
        for (int w = 0; w < KEEP1; ++w)
#pragma unroll
            for (int n = 0; n < C1; ++n) win1[w][n] = win1[w + SH2][n];
        float l0[KEEP0 + NS0][C0];
#pragma unroll
        for (int w = 0; w < KEEP0; ++w)
#pragma unroll
            for (int n = 0; n < C0; ++n) l0[w][n] = keep0[w][n];
#pragma unroll
        for (int n = 0; n < NS0; ++n) settle(nr[n], h0n + n, l0[KEEP0 + n]);
#pragma unroll
        for (int a = 0; a < SH2; ++a) level1(r1n + a, &l0[a * SH1], win1[KEEP1 + a]);
#pragma unroll
        for (int w = 0; w < KEEP0; ++w)
#pragma unroll
            for (int n = 0; n < C0; ++n) keep0[w][n] = l0[NS0 + w][n];
        put(t, y, yi);
    };
    auto last = [&](int32_t t) {
        float y[VO];
        int32_t yi[VO];
        reduce(t, y, yi);
        put(t, y, yi);
    };
    // The compiler places the waits for loads by what may be in flight on *any* path to a use, so the loop leaves
    // it no doubt.  Nothing is in flight when the loop starts: a load whose first use lies inside the loop (the
    // trailing list's parameters) would make it wait for all loads at that use, in every iteration -- the rows just
    // requested included.  Every pass through the loop body requests rows and uses them, with no condition on
    // either (the chunk's last row, which requests nothing, stands behind the loop): a request skipped on one path
    // and a use skipped on another would look like a request that may still be open where the next ones are issued.
    // Two rows per pass: after two rows the sliding windows are back in the registers they started in.
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    int32_t t = 0;
    for (; t + 2 < k.rc; t += 2) {  // the same for every lane
        step(t);
        step(t + 1);
    }
    if (t + 2 == k.rc) {
        step(t);
        last(t + 1);
    } else {
        last(t);
    }
}

// a compile-time integer as a function argument (no standard-library headers here: run-time builds)
template <int V>
struct IntTag {
    static constexpr int value = V;
};

// =============================================================================
// pool_xrows_chain_kernel: L identical max-pooling steps that keep the plane's size, each followed by
// the element-wise list EW (the blocks of Section 5.1's stacked-pooling experiment), in registers.
// One new input row per step ripples through all L levels: level l's row h - l * PH needs level
// l - 1's rows up to h - (l - 1) * PH, the one the same step has just produced.  Per level the lane
// keeps the KH newest rows of the level below (own columns only: the maximum goes down the window's
// rows first, then one row of column maxima is exchanged with the neighbouring lanes); the loop
// body is unrolled KH times, so a row's place in its ring is known at compile time and nothing is
// moved.  A chunk of rc output rows starts L * PH rows above its first row; the rows computed
// before a level has seen KH real rows are never used by a row the chunk stores.
// =============================================================================
template <int DT, int VEC, class P, int EW, int L>
__global__ __launch_bounds__(256) void pool_xrows_chain_kernel(const RowsChainK k)
{
    constexpr int KH = P::kh, KW = P::kw, PH = P::ph, PW = P::pw;
    static_assert(P::kind == OP_MAXPOOL && P::sh == 1 && P::sw == 1 && KH == 2 * PH + 1 && KW == 2 * PW + 1 && PW <= VEC && L >= 1,
                  "max pooling that keeps the plane's size");
    using E = RowsEw<EW>;
    using Row = XRowRaw<DT, VEC>;
    constexpr int ES = DT != DT_F32 ? 2 : 4;
    const float pad = -INFINITY;

    const XLane lane = xrows_lane(k);
    RowsParams<E> par[L];
#pragma unroll
    for (int l = 0; l < L; ++l) rows_load_params<E>(k.ew[l], k.params, k.C, lane.c, par[l]);
    const char *inp = static_cast<const char *>(image_base<DT>(k.in, lane.img, k.in_extra)) + (size_t)lane.plane * (size_t)(k.H * k.W) * ES;
    void *outp = image_base<DT>(k.out, lane.img, k.out_extra);
    const int32_t col0 = lane.j * VEC;
    const bool has_left = lane.j > 0, has_right = lane.j + 1 < k.cbs;
    const uint32_t plane_off = lane.plane * (uint32_t)(k.H * k.W);
    const int32_t o0 = lane.chunk * k.rc, o1 = min(o0 + k.rc, k.H);  // output rows of the chunk
    const int32_t h_first = o0 - L * PH;                              // first input row the chunk needs
    const int32_t passes = (k.rc + 2 * L * PH + KH - 1) / KH;         // the same for every lane

    float ring[L][KH][VEC];  // ring[l]: the KH newest rows of level l (level 0: the input)
#pragma unroll
    for (int l = 0; l < L; ++l)
#pragma unroll
        for (int j = 0; j < KH; ++j)
#pragma unroll
            for (int n = 0; n < VEC; ++n) ring[l][j][n] = pad;

    // The KH input rows of a pass are requested two passes ahead (never under a branch: a row outside the plane is
    // requested from the nearest row inside and replaced by padding; the compiler then knows how many requests are in
    // flight and waits for the oldest only).  One pass ahead, a pass waited for the stores of the pass before it as well:
    // 26 us for one to four levels on 64 x 64 x 56 x 56 whatever the arithmetic.
    Row ahead[2][KH];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int j = 0; j < KH; ++j) xrows_fetch<DT, VEC>(inp, h_first + a * KH + j, k.H, k.W, col0, ahead[a][j]);
    auto one_pass = [&](auto slot_tag, int32_t pass) {
        constexpr int SLOT = decltype(slot_tag)::value;
        Row now[KH];
#pragma unroll
        for (int j = 0; j < KH; ++j) now[j] = ahead[SLOT][j];
#pragma unroll
        for (int j = 0; j < KH; ++j) xrows_fetch<DT, VEC>(inp, h_first + (pass + 2) * KH + j, k.H, k.W, col0, ahead[SLOT][j]);
#pragma unroll
        for (int j = 0; j < KH; ++j) {
            const int32_t h = h_first + pass * KH + j;
            {
                float x[VEC];
                xrows_unpack<DT, VEC>(now[j], x);
                const bool ok = h >= 0 && h < k.H;
#pragma unroll
                for (int n = 0; n < VEC; ++n) ring[0][j][n] = ok ? x[n] : pad;
            }
#pragma unroll
            for (int l = 1; l <= L; ++l) {
                const int32_t r = h - l * PH;  // the row of level l this step completes
                float m[VEC], full[PW + VEC + PW], v[VEC];
#pragma unroll
                for (int n = 0; n < VEC; ++n) {
                    m[n] = ring[l - 1][0][n];
#pragma unroll
                    for (int d = 1; d < KH; ++d) m[n] = __builtin_fmaxf(m[n], ring[l - 1][d][n]);
                }
                with_neighbours<VEC, PW, PW>(m, full, has_left, has_right, pad);
#pragma unroll
                for (int n = 0; n < VEC; ++n) {
                    v[n] = full[n];
#pragma unroll
                    for (int d = 1; d < KW; ++d) v[n] = __builtin_fmaxf(v[n], full[n + d]);
                }
                rows_apply<DT, E, VEC>(v, par[l - 1]);
                const bool rok = r >= 0 && r < k.H;
                if (l < L) {
#pragma unroll
                    for (int n = 0; n < VEC; ++n) ring[l < L ? l : 0][j][n] = rok ? v[n] : pad;
                } else if (lane.live && r >= o0 && r < o1) {
                    store_elems<DT, VEC>(outp, plane_off + (uint32_t)(r * k.W + col0), v);
                }
            }
        }
    };
    for (int32_t pass = 0; pass < passes; pass += 2) {  // an odd count runs one pass more: its rows lie behind the chunk
        one_pass(IntTag<0>{}, pass);
        one_pass(IntTag<1>{}, pass + 1);
    }
}

}  // namespace bs
