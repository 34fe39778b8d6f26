// Device code of the lds_tile kernels: depth-first execution of a multi-step (or overlapping-window)
// sequence, one tile per work-group (Section 4.4 "stacked" pooling: patches, two on-chip
// buffers, a barrier and a buffer swap after every step).
//
// Levels: level 0 is the sequence input, pooling operation l (1..L) turns level l-1
// into level l.  A work-group owns PPG planes x the TH x TW tile of level L whose
// top-left output is (ti*TH, tj*TW).  For every level it keeps a fixed-size rectangle
// (rows_l x cols_l) whose origin follows from the tile by origin[l-1] = origin[l] * s - p,
// so the rectangle of level l-1 holds exactly the windows of the rectangle of level l.
// Cells of a rectangle that fall outside the plane are the padding of the pooling
// operation that will read them: they hold -inf for a max (never selected) and +0 for an
// average (adding +0 to the running sum leaves it bit-identical, because a sum started at
// +0 is never -0).  They are never computed from earlier layers.  Level l (l < L) lives in
// LDS buffer l & 1.
//
// Lane grid.  In every phase the work-group's lanes form a ct x rt grid (one division per
// lane per phase): ct lanes along a row, rt rows in flight; a lane keeps its column and
// walks down the rows, so column arithmetic and predicates are loop-invariant and the plane
// (hence the BatchNorm channel) is uniform per iteration: folded parameters come from
// scalar loads.
//
// Phase 0 loads 128-bit global vectors and stores each with one 128-bit LDS write after the
// level-0 element-wise operations: the level-0 LDS row starts at the global vector that
// contains the rectangle's first column (delta0 columns earlier).  Phase l gives each lane a
// strip of four horizontally adjacent outputs: it reads the kh rows x (D + 3*sw + kw) columns
// it needs with aligned 128/64/32-bit LDS reads and keeps the windows in registers.
//
// Two builds of the same phase code (the paper generates code per stack, Section 4.1; here
// the planner picks among pre-compiled instances):
//   lds_sig_kernel<...>   every pooling shape and element-wise list is a template argument:
//                         instantiated for the stack signatures in the table at the end
//   lds_tile_kernel       shapes and lists are read from the argument block at run time
#pragma once
#include "bs_device.h"

namespace bs {

// --------------------------------------------------------------- shape policies
template <int KIND, int KH, int KW, int SH, int SW, int PH, int PW, int CIP>
struct PoolSpec {
    static constexpr bool is_static = true;
    BS_DEV explicit PoolSpec(const PoolK &) {}
    __host__ __device__ static constexpr int kind() { return KIND; }
    __host__ __device__ static constexpr int kh() { return KH; }
    __host__ __device__ static constexpr int kw() { return KW; }
    __host__ __device__ static constexpr int sh() { return SH; }
    __host__ __device__ static constexpr int sw() { return SW; }
    __host__ __device__ static constexpr int ph() { return PH; }
    __host__ __device__ static constexpr int pw() { return PW; }
    __host__ __device__ static constexpr int cip() { return CIP; }
    __host__ __device__ static constexpr float inv_kk() { return 1.0f / (float)(KH * KW); }
};

struct PoolDyn {
    static constexpr bool is_static = false;
    const PoolK &p;
    BS_DEV explicit PoolDyn(const PoolK &q) : p(q) {}
    BS_DEV int kind() const { return p.kind; }
    BS_DEV int kh() const { return p.kh; }
    BS_DEV int kw() const { return p.kw; }
    BS_DEV int sh() const { return p.sh; }
    BS_DEV int sw() const { return p.sw; }
    BS_DEV int ph() const { return p.ph; }
    BS_DEV int pw() const { return p.pw; }
    BS_DEV int cip() const { return p.count_include_pad; }
    BS_DEV float inv_kk() const { return p.inv_kk; }
};

// Element-wise list of a level: CODE packs up to K_MAX_EW operation kinds, base K_EW_BASE, first
// operation in the lowest digit (the OpKind value; 0 = end); CODE < 0: run time.
template <int CODE>
struct EwList {
    static constexpr bool is_static = CODE >= 0;
    static constexpr int code = CODE;
    __host__ __device__ static constexpr int count_static() { return ew_code_len(CODE); }
    static constexpr int slots = CODE >= 0 ? count_static() : K_MAX_EW;
    BS_DEV static int count(const LevelK &lv) { return CODE >= 0 ? count_static() : lv.n_ew; }
    BS_DEV static int kind(const LevelK &lv, int j)
    {
        if (CODE >= 0) return ew_code_kind(CODE, j);  // digits are the operation kinds
        return lv.ew[j].kind;
    }
};
static_assert(OP_CLAMP < K_EW_BASE, "EwList digits are the operation kinds");

template <class P>
BS_DEV float pad_value(const P &p) { return p.kind() == OP_MAXPOOL ? -INFINITY : 0.0f; }

typedef const __attribute__((address_space(4))) float *const_f32_ptr;

// Folded BatchNorm parameters of one level for one (uniform) channel, fetched with scalar loads.
template <class EW>
struct EwRegs {
    float sc[EW::slots > 0 ? EW::slots : 1], sh[EW::slots > 0 ? EW::slots : 1];
};

template <class EW>
BS_DEV void load_ew_regs(const LevelK &lv, const float *params, int32_t C, int32_t c, EwRegs<EW> &e)
{
    const_f32_ptr cp = (const_f32_ptr)params;
#pragma unroll
    for (int j = 0; j < EW::slots; ++j) {
        e.sc[j] = 1.0f;
        e.sh[j] = 0.0f;
        if (j < EW::count(lv)) {
            const int32_t kind = EW::kind(lv, j);
            if (kind == OP_BN) {
                e.sc[j] = cp[lv.ew[j].arg + c];
                e.sh[j] = cp[lv.ew[j].arg + C + c];
            } else if (kind == OP_LEAKY || kind == OP_CLAMP) {  // [slope, -] / [lo, hi]
                e.sc[j] = cp[lv.ew[j].arg];
                e.sh[j] = cp[lv.ew[j].arg + 1];
            }
        }
    }
}

// Element-wise operations of a level on N values of one plane.  CONTIG: the N values are
// consecutive elements starting at off[0] (one vector residual load); else off[i] each.
template <int DT, int N, bool CONTIG, class EW>
BS_DEV void apply_level_ew(float (&x)[N], const LevelK &lv, const EwRegs<EW> &er, const void *const *res,
                           const uint32_t (&off)[CONTIG ? 1 : N])
{
#pragma unroll
    for (int j = 0; j < EW::slots; ++j) {
        if (j >= EW::count(lv)) break;
        const int32_t kind = EW::kind(lv, j);
        if (kind == OP_BN) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(__builtin_fmaf(x[i], er.sc[j], er.sh[j]));
        } else if (kind == OP_RELU) {
            // v_max_f32: NaN -> 0, and max(-0, +0) = +0 in either operand order
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = __builtin_fmaxf(x[i], 0.0f);
        } else if (kind == OP_LEAKY) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(x[i] > 0.0f ? x[i] : x[i] * er.sc[j]);
        } else if (kind == OP_CLAMP) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[i], er.sc[j]), er.sh[j]));
        } else {
            const void *rp = res[lv.ew[j].arg];
            float r[N];
            if constexpr (CONTIG) {
                const Raw<DT, N> rr = load_raw<DT, N>(rp, off[0]);
                unpack<DT, N>(rr, r);
            } else {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    const Raw<DT, 1> rr = load_raw<DT, 1>(rp, off[i]);
                    float one[1];
                    unpack<DT, 1>(rr, one);
                    r[i] = one[0];
                }
            }
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<DT>(x[i] + r[i]);
        }
    }
}

// Read N consecutive floats starting at a 16-byte aligned LDS address.
template <int N>
BS_DEV void lds_read_row(const float *p, float (&r)[N])
{
    constexpr int Q = N / 4, R = N % 4;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const float4 t = *reinterpret_cast<const float4 *>(p + 4 * q);
        r[4 * q] = t.x; r[4 * q + 1] = t.y; r[4 * q + 2] = t.z; r[4 * q + 3] = t.w;
    }
    if constexpr (R >= 2) {
        const float2 t = *reinterpret_cast<const float2 *>(p + 4 * Q);
        r[4 * Q] = t.x; r[4 * Q + 1] = t.y;
    }
    if constexpr (R == 1) r[4 * Q] = p[4 * Q];
    if constexpr (R == 3) r[4 * Q + 2] = p[4 * Q + 2];
}

template <class P>
struct StripVO {
    static constexpr int value = 4;  // run-time shapes: register room for the widest strip
};
template <int KIND, int KH, int KW, int SH, int SW, int PH, int PW, int CIP>
struct StripVO<PoolSpec<KIND, KH, KW, SH, SW, PH, PW, CIP>> {
    static constexpr int value = strip_outputs(SW);
};

// One strip of VO outputs of pooling operation P from the cached level below.
//   src      16-byte aligned LDS address; the strip's first window starts D (static shapes)
//            or d_rt (run-time shapes) floats after it
//   h0, w0   global row / column of the first window's first cell in the input plane (may be
//            negative: padding)
//   vo       outputs actually wanted (run-time shapes; static shapes produce all VO)
template <class P, int VO, int D, bool WANT_IDX>
BS_DEV void pool_strip(const P &p, const float *src, int32_t d_rt, int32_t vo, int32_t pitch, int32_t h0,
                       int32_t w0, int32_t Hp, int32_t Wp, float (&val)[VO], int32_t (&bidx)[VO])
{
    const bool is_max = p.kind() == OP_MAXPOOL;
    float acc[VO];
#pragma unroll
    for (int e = 0; e < VO; ++e) {
        acc[e] = is_max ? -INFINITY : 0.0f;
        if constexpr (WANT_IDX) bidx[e] = max(h0, 0) * Wp + max(w0 + e * p.sw(), 0);  // first in-range cell
    }
    if constexpr (P::is_static) {
        constexpr int KH = P::kh(), KW = P::kw(), SW = P::sw();
        constexpr int NC = (VO - 1) * SW + KW;                    // columns the windows span
        constexpr int NR = D == 0 ? NC : (D + NC + 3) / 4 * 4;    // floats read per row
        float r[KH][NR];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) lds_read_row<NR>(src + dh * pitch, r[dh]);
        if (is_max) {
#pragma unroll
            for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                for (int e = 0; e < VO; ++e)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) {
                        const float v = r[dh][D + e * SW + dw];
                        if constexpr (WANT_IDX) {
                            const bool g = v > acc[e];
                            acc[e] = g ? v : acc[e];
                            bidx[e] = g ? (h0 + dh) * Wp + w0 + e * SW + dw : bidx[e];
                        } else {
                            acc[e] = __builtin_fmaxf(acc[e], v);
                        }
                    }
        } else {
#pragma unroll
            for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                for (int e = 0; e < VO; ++e)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) acc[e] = acc[e] + r[dh][D + e * SW + dw];
        }
    } else {
        const int32_t kh = p.kh(), kw = p.kw(), sw = p.sw();
        for (int32_t dh = 0; dh < kh; ++dh) {
            const float *rowp = src + dh * pitch + d_rt;
            const int32_t rbase = (h0 + dh) * Wp + w0;
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                if (e >= vo) break;
                for (int32_t dw = 0; dw < kw; ++dw) {
                    const float v = rowp[e * sw + dw];
                    if (is_max) {
                        const bool g = v > acc[e];
                        acc[e] = g ? v : acc[e];
                        if constexpr (WANT_IDX) bidx[e] = g ? rbase + e * sw + dw : bidx[e];
                    } else {
                        acc[e] = acc[e] + v;
                    }
                }
            }
        }
    }
    if (is_max) {
#pragma unroll
        for (int e = 0; e < VO; ++e) val[e] = acc[e];
    } else if (p.cip() == 1) {
#pragma unroll
        for (int e = 0; e < VO; ++e) val[e] = acc[e] * p.inv_kk();
    } else {
        // 0: in-range cells; 2 (ceil mode with count_include_pad): cells inside the padded plane
        const bool padded = p.cip() == 2;
        const int32_t nr = padded ? min(h0 + p.kh(), Hp + p.ph()) - h0 : min(h0 + p.kh(), Hp) - max(h0, 0);
#pragma unroll
        for (int e = 0; e < VO; ++e) {
            const int32_t we = w0 + e * p.sw();
            const int32_t nc = padded ? min(we + p.kw(), Wp + p.pw()) - we : min(we + p.kw(), Wp) - max(we, 0);
            // windows wholly outside the plane can make nr * nc <= 0; such outputs are never stored
            val[e] = acc[e] * (1.0f / (float)max(nr * nc, 1));
        }
    }
}

// RB consecutive output rows of one strip (static shapes): the kh input rows of the current
// windows stay in registers and slide down by sh rows per output row, so an input row is read
// from LDS once per block instead of once per output row it contributes to.  Without index
// outputs a max is taken column-wise first and then across each window (same value: max is
// exact and order-free for the finite inputs the library accepts).
//   src      16-byte aligned LDS address of the first window row of the block
//   nrows    output rows wanted (1..RB); rows beyond are neither read nor emitted
//   h0, w0   global row / column of the first window's first cell in the input plane
//   emit(i, val, bidx)  receives output row i of the block
template <class P, int VO, int D, bool WANT_IDX, int RB, class F>
BS_DEV void pool_block(const P &p, const float *src, int32_t pitch, int32_t nrows, int32_t h0, int32_t w0,
                       int32_t Hp, int32_t Wp, F &&emit)
{
    constexpr int KH = P::kh(), KW = P::kw(), SH = P::sh(), SW = P::sw();
    constexpr int NC = (VO - 1) * SW + KW;                    // columns the windows span
    constexpr int NR = D == 0 ? NC : (D + NC + 3) / 4 * 4;    // floats read per row
    constexpr int KEEP = KH > SH ? KH - SH : 0;               // rows two consecutive windows share
    constexpr bool IS_MAX = P::kind() == OP_MAXPOOL;
    float w[KH][NR];
#pragma unroll
    for (int dh = 0; dh < KH; ++dh) lds_read_row<NR>(src + dh * pitch, w[dh]);
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        if (i < nrows) {
            const int32_t hi = h0 + i * SH;
            float val[VO];
            int32_t bidx[VO];
            if constexpr (IS_MAX && !WANT_IDX) {
                float cm[NC];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    cm[c] = w[0][D + c];
#pragma unroll
                    for (int dh = 1; dh < KH; ++dh) cm[c] = __builtin_fmaxf(cm[c], w[dh][D + c]);
                }
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    val[e] = cm[e * SW];
#pragma unroll
                    for (int dw = 1; dw < KW; ++dw) val[e] = __builtin_fmaxf(val[e], cm[e * SW + dw]);
                    bidx[e] = 0;
                }
            } else if constexpr (IS_MAX) {
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    float best = -INFINITY;
                    int32_t bi = max(hi, 0) * Wp + max(w0 + e * SW, 0);  // first in-range cell
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            const float v = w[dh][D + e * SW + dw];
                            const bool g = v > best;
                            best = g ? v : best;
                            bi = g ? (hi + dh) * Wp + w0 + e * SW + dw : bi;
                        }
                    val[e] = best;
                    bidx[e] = bi;
                }
            } else {
#pragma unroll
                for (int e = 0; e < VO; ++e) {
                    float sum = 0.0f;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) sum = sum + w[dh][D + e * SW + dw];
                    if (p.cip() == 1) {
                        val[e] = sum * p.inv_kk();
                    } else {
                        // 0: in-range cells; 2 (ceil mode with count_include_pad): cells inside the padded plane
                        const bool padded = p.cip() == 2;
                        const int32_t we = w0 + e * SW;
                        const int32_t nr = padded ? min(hi + KH, Hp + P::ph()) - hi : min(hi + KH, Hp) - max(hi, 0);
                        const int32_t nc = padded ? min(we + KW, Wp + P::pw()) - we : min(we + KW, Wp) - max(we, 0);
                        // windows wholly outside the plane can make nr * nc <= 0; such outputs are never stored
                        val[e] = sum * (1.0f / (float)max(nr * nc, 1));
                    }
                    bidx[e] = 0;
                }
            }
            emit(i, val, bidx);
        }
        if (i + 1 < RB) {
#pragma unroll
            for (int dh = 0; dh < KEEP; ++dh)
#pragma unroll
                for (int n = 0; n < NR; ++n) w[dh][n] = w[dh + SH][n];
            if (i + 1 < nrows) {
#pragma unroll
                for (int dh = KEEP; dh < KH; ++dh) lds_read_row<NR>(src + ((i + 1) * SH + dh) * pitch, w[dh]);
            }
        }
    }
}

// What a work-group knows about its tile.
struct TileCtx {
    int32_t ti, tj, plane0, nplanes;
};

BS_DEV TileCtx tile_ctx(const LdsSeqK &k)
{
    TileCtx t;
    const uint32_t pg = fdiv(blockIdx.x, k.div_tiles_hw);
    const uint32_t trem = blockIdx.x - pg * (uint32_t)(k.tiles_h * k.tiles_w);
    t.ti = (int32_t)fdiv(trem, k.div_tiles_w);
    t.tj = (int32_t)(trem - (uint32_t)t.ti * (uint32_t)k.tiles_w);
    t.plane0 = (int32_t)pg * k.PPG;
    t.nplanes = min(k.PPG, k.NC - t.plane0);
    return t;
}

// ---------------- phase 0: load the level-0 rectangle, apply its element-wise ops ----
// (r0, c0): global row / column of the rectangle's origin; padv: padding of pooling op 1.
template <int DT, int VEC, class EW>
BS_DEV void phase0(const LdsSeqK &k, const TileCtx &t, float *lds, int32_t r0, int32_t c0, float padv)
{
    const LevelK &lv = k.level[0];
    const uint32_t tid = threadIdx.x;
    const int32_t g0 = c0 - k.delta0;  // global column of LDS column 0: a multiple of VEC
    const uint32_t ty = fdiv(tid, lv.div_ct), tx = tid - ty * (uint32_t)lv.ct;
    if ((int32_t)ty >= lv.rt) return;
    constexpr int U = (VEC == 8) ? 2 : 4;
    float *dst = lds + lv.buf_off;
    for (int32_t pl = 0; pl < t.nplanes; ++pl) {
        const uint32_t plane = (uint32_t)(t.plane0 + pl);
        const uint32_t img = fdiv(plane, k.div_c);
        const int32_t ch = (int32_t)(plane - img * (uint32_t)k.C);
        const void *inp = image_base<DT>(k.in, img, k.in_extra);
        EwRegs<EW> er;
        load_ew_regs<EW>(lv, k.params, k.C, ch, er);
        const uint32_t gplane = plane * (uint32_t)(lv.H * lv.W);
        float *dplane = dst + pl * lv.plane_stride;
        for (int32_t v = (int32_t)tx; v < lv.items_per_row; v += lv.ct) {
            const int32_t gc = g0 + v * VEC;
            const bool col_in = gc >= 0 && gc < lv.W;  // W % VEC == 0: a vector is all in or all out
            for (int32_t rb = (int32_t)ty; rb < lv.rows; rb += lv.rt * U) {
                Raw<DT, VEC> raw[U];
                bool inimg[U];
                uint32_t off[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int32_t r = rb + u * lv.rt;
                    const int32_t gr = r0 + r;
                    inimg[u] = col_in && r < lv.rows && gr >= 0 && gr < lv.H;
                    off[u] = inimg[u] ? gplane + (uint32_t)gr * (uint32_t)lv.W + (uint32_t)gc : 0u;
                    raw[u] = load_raw<DT, VEC, true>(inp, off[u]);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int32_t r = rb + u * lv.rt;
                    float x[VEC];
                    unpack<DT, VEC>(raw[u], x);
                    const uint32_t o1[1] = {off[u]};
                    apply_level_ew<DT, VEC, true, EW>(x, lv, er, k.res, o1);
                    if (r < lv.rows) {
                        float *d = dplane + r * lv.pitch + v * VEC;
                        if constexpr (VEC >= 4) {
#pragma unroll
                            for (int h = 0; h < VEC / 4; ++h) {
                                float4 w;
                                w.x = inimg[u] ? x[4 * h] : padv;
                                w.y = inimg[u] ? x[4 * h + 1] : padv;
                                w.z = inimg[u] ? x[4 * h + 2] : padv;
                                w.w = inimg[u] ? x[4 * h + 3] : padv;
                                *reinterpret_cast<float4 *>(d + 4 * h) = w;
                            }
                        } else {
                            d[0] = inimg[u] ? x[0] : padv;
                        }
                    }
                }
            }
        }
    }
}

// Everything a pooling phase needs that does not depend on the lane.
struct PhaseCtx {
    const float *src;
    float *dst;
    int32_t r0, c0;        // global row / column of this level's rectangle origin
    int32_t end_r, end_c;  // rows / columns below which this tile writes memory at this level
    int32_t d_lo;          // LDS column of the rectangle's first column in the level below
    bool last, vec_store_ok;
    float padv;            // padding of the next pooling operation (unused at the last level)
    int32_t *idxp;
};

// ---------------- phase l: pooling operation l on the cached level l-1 --------------
template <int DT, class P, class EW, int D, bool WANT_IDX, bool LAST>
BS_DEV void pool_phase(const LdsSeqK &k, const TileCtx &t, const LevelK &lv, const LevelK &pv, const P &p,
                       const PhaseCtx &cx)
{
    constexpr int VO = StripVO<P>::value;
    const int32_t vo = P::is_static ? VO : lv.vo;
    const uint32_t tid = threadIdx.x;
    const uint32_t ty = fdiv(tid, lv.div_ct), tx = tid - ty * (uint32_t)lv.ct;
    if ((int32_t)ty >= lv.rt) return;
    const int32_t spr = lv.items_per_row;
    for (int32_t pl = 0; pl < t.nplanes; ++pl) {
        const uint32_t plane = (uint32_t)(t.plane0 + pl);
        const uint32_t img = fdiv(plane, k.div_c);
        const int32_t ch = (int32_t)(plane - img * (uint32_t)k.C);
        void *outp = LAST ? image_base<DT>(k.out, img, k.out_extra) : nullptr;
        EwRegs<EW> er;
        load_ew_regs<EW>(lv, k.params, k.C, ch, er);
        const float *splane = cx.src + pl * pv.plane_stride;
        float *dplane = cx.dst + pl * lv.plane_stride;
        const uint32_t gplane = plane * (uint32_t)(lv.H * lv.W);
        for (int32_t j = (int32_t)tx; j < spr; j += lv.ct) {
            const int32_t gc = cx.c0 + vo * j;
            const int32_t w0 = gc * p.sw() - p.pw();
            // aligned LDS column where this strip's reads start; its first window starts D (or,
            // for run-time shapes, d_rt) floats later
            const int32_t scol = vo * j * p.sw() + (P::is_static ? (cx.d_lo - D) : 0);
            const int32_t d_rt = P::is_static ? 0 : cx.d_lo;
            bool cin[VO];
#pragma unroll
            for (int e = 0; e < VO; ++e) cin[e] = e < vo && gc + e >= 0 && gc + e < lv.W;
            const bool strip_vec = P::is_static && cx.vec_store_ok && gc >= 0 && gc + VO - 1 < cx.end_c;
            // what happens to the VO outputs of rectangle row r once they are pooled
            auto finish = [&](int32_t r, float (&val)[VO], int32_t (&bi)[VO]) {
                const int32_t gr = cx.r0 + r;
                if (p.kind() != OP_MAXPOOL) {
#pragma unroll
                    for (int e = 0; e < VO; ++e) val[e] = round_store<DT>(val[e]);
                }
                const bool row_in = gr >= 0 && gr < lv.H;
                const uint32_t goff = gplane + (uint32_t)(row_in ? gr : 0) * (uint32_t)lv.W;
                if constexpr (WANT_IDX) {
                    if (cx.idxp && row_in && gr < cx.end_r) {
#pragma unroll
                        for (int e = 0; e < VO; ++e)
                            if (cin[e] && gc + e < cx.end_c) cx.idxp[goff + (uint32_t)(gc + e)] = bi[e];
                    }
                }
                if (EW::count(lv) > 0) {
                    uint32_t o4[VO];
#pragma unroll
                    for (int e = 0; e < VO; ++e) o4[e] = (row_in && cin[e]) ? goff + (uint32_t)(gc + e) : 0u;
                    apply_level_ew<DT, VO, false, EW>(val, lv, er, k.res, o4);
                }
                if (LAST) {
                    if (row_in && gr < cx.end_r) {
                        if (strip_vec) {
                            store_elems<DT, VO>(outp, goff + (uint32_t)gc, val);
                        } else {
#pragma unroll
                            for (int e = 0; e < VO; ++e)
                                if (cin[e] && gc + e < cx.end_c) {
                                    const float one[1] = {val[e]};
                                    store_elems<DT, 1>(outp, goff + (uint32_t)(gc + e), one);
                                }
                        }
                    }
                } else {
                    float w[VO];
#pragma unroll
                    for (int e = 0; e < VO; ++e) w[e] = (row_in && cin[e]) ? val[e] : cx.padv;
                    float *d = dplane + r * lv.pitch + vo * j;
                    if constexpr (P::is_static && VO == 4) {
                        *reinterpret_cast<float4 *>(d) = make_float4(w[0], w[1], w[2], w[3]);
                    } else if constexpr (P::is_static && VO == 2) {
                        *reinterpret_cast<float2 *>(d) = make_float2(w[0], w[1]);
                    } else {
#pragma unroll
                        for (int e = 0; e < VO; ++e)
                            if (e < vo) d[e] = w[e];
                    }
                }
            };
            if constexpr (P::is_static) {
                // lanes of the ct x rt grid take blocks of K_LDS_RB consecutive rows
                constexpr int RB = K_LDS_RB;
                const int32_t nblk = (lv.rows + RB - 1) / RB;
                for (int32_t b = (int32_t)ty; b < nblk; b += lv.rt) {
                    const int32_t rb0 = b * RB;
                    pool_block<P, VO, D, WANT_IDX, RB>(
                        p, splane + (rb0 * P::sh()) * pv.pitch + scol, pv.pitch, min(RB, lv.rows - rb0),
                        (cx.r0 + rb0) * P::sh() - P::ph(), w0, pv.H, pv.W,
                        [&](int i, float (&val)[VO], int32_t (&bi)[VO]) { finish(rb0 + i, val, bi); });
                }
            } else {
                for (int32_t r = (int32_t)ty; r < lv.rows; r += lv.rt) {
                    const int32_t h0 = (cx.r0 + r) * p.sh() - p.ph();
                    float val[VO];
                    int32_t bi[VO];
#pragma unroll
                    for (int e = 0; e < VO; ++e) bi[e] = 0;
                    pool_strip<P, VO, D, WANT_IDX>(p, splane + (r * p.sh()) * pv.pitch + scol, d_rt, vo, pv.pitch, h0,
                                                   w0, pv.H, pv.W, val, bi);
                    finish(r, val, bi);
                }
            }
        }
    }
}

// Lane-independent context of phase l for tile t.
BS_DEV PhaseCtx phase_ctx(const LdsSeqK &k, const TileCtx &t, float *lds, int32_t l)
{
    const int32_t L = k.n_levels;
    const LevelK &lv = k.level[l];
    PhaseCtx cx;
    cx.r0 = t.ti * k.TH;
    cx.c0 = t.tj * k.TW;
    int32_t step_r = k.TH, step_c = k.TW;  // distance between neighbouring tiles' origins
    for (int32_t m = L; m > l; --m) {
        origin_step(k.pool[m], cx.r0, cx.c0);
        step_r *= k.pool[m].sh;
        step_c *= k.pool[m].sw;
    }
    cx.src = lds + k.level[l - 1].buf_off;
    cx.dst = lds + lv.buf_off;
    cx.last = (l == L);
    cx.padv = cx.last ? 0.0f : (k.pool[l + 1].kind == OP_MAXPOOL ? -INFINITY : 0.0f);
    cx.idxp = k.pool[l].idx_slot >= 0 ? k.idx[k.pool[l].idx_slot] : nullptr;
    // rows / columns of this level the tile may write to memory: its own tile at the last
    // level; elsewhere (index output in the middle of a sequence) up to where the next
    // tile's rectangle starts, so every cell is written exactly once
    const int32_t own_r = (t.ti + 1 < k.tiles_h) ? cx.r0 + step_r : lv.H;
    const int32_t own_c = (t.tj + 1 < k.tiles_w) ? cx.c0 + step_c : lv.W;
    cx.end_r = min(own_r, lv.H);
    cx.end_c = min(own_c, lv.W);
    cx.d_lo = (l == 1) ? k.delta0 : 0;
    cx.vec_store_ok = cx.last && (lv.W % lv.vo) == 0 && ((k.TW % lv.vo) == 0 || k.tiles_w == 1);
    return cx;
}

// =============================================================================
// Run-time build: any sequence.
// =============================================================================
template <int DT, int VEC>
__global__ __launch_bounds__(512) void lds_tile_kernel(const LdsSeqK k)
{
    extern __shared__ __align__(16) float lds[];
    const int32_t L = k.n_levels;
    const TileCtx t = tile_ctx(k);
    {
        int32_t r0 = t.ti * k.TH, c0 = t.tj * k.TW;
        for (int32_t l = L; l >= 1; --l) origin_step(k.pool[l], r0, c0);
        phase0<DT, VEC, EwList<-1>>(k, t, lds, r0, c0, pad_value(PoolDyn(k.pool[1])));
    }
    __syncthreads();
    for (int32_t l = 1; l <= L; ++l) {
        const PhaseCtx cx = phase_ctx(k, t, lds, l);
        const PoolDyn p(k.pool[l]);
        if (cx.last) {
            if (cx.idxp) pool_phase<DT, PoolDyn, EwList<-1>, 0, true, true>(k, t, k.level[l], k.level[l - 1], p, cx);
            else pool_phase<DT, PoolDyn, EwList<-1>, 0, false, true>(k, t, k.level[l], k.level[l - 1], p, cx);
        } else {
            if (cx.idxp) pool_phase<DT, PoolDyn, EwList<-1>, 0, true, false>(k, t, k.level[l], k.level[l - 1], p, cx);
            else pool_phase<DT, PoolDyn, EwList<-1>, 0, false, false>(k, t, k.level[l], k.level[l - 1], p, cx);
            __syncthreads();
        }
    }
}

// =============================================================================
// Signature build: the whole sequence shape is a template argument.
//   Lvl<P, EWCODE>...: pooling shape and element-wise list of levels 1..L.
// =============================================================================
template <class P_, int EWCODE>
struct Lvl {
    using P = P_;
    using EW = EwList<EWCODE>;
};

// delta0 of a signature: the rectangle's first column of tile 0 modulo the vector width
template <int VEC, class... Ls>
constexpr int sig_delta0()
{
    constexpr int n = (int)sizeof...(Ls);
    const int sw[n] = {Ls::P::sw()...}, pw[n] = {Ls::P::pw()...};
    int c = 0;
    for (int l = n - 1; l >= 0; --l) c = c * sw[l] - pw[l];
    return ((c % VEC) + VEC) % VEC;
}

// phases L, L + 1, ... of a signature, a barrier between them
template <int DT, bool WANT_IDX, int L, int D0, class... Ls>
struct SigPhases {
    BS_DEV static void run(const LdsSeqK &, const TileCtx &, float *) {}
};
template <int DT, bool WANT_IDX, int L, int D0, class L1, class... Rest>
struct SigPhases<DT, WANT_IDX, L, D0, L1, Rest...> {
    BS_DEV static void run(const LdsSeqK &k, const TileCtx &t, float *lds)
    {
        constexpr bool LAST = sizeof...(Rest) == 0;
        PhaseCtx cx = phase_ctx(k, t, lds, L);
        if (L == 1) cx.d_lo = D0;  // compile-time; the planner's argument block carries the same value
        const typename L1::P p(k.pool[L]);
        pool_phase<DT, typename L1::P, typename L1::EW, (L == 1 ? (D0 & 3) : 0), WANT_IDX, LAST>(
            k, t, k.level[L], k.level[L - 1], p, cx);
        if constexpr (!LAST) {
            __syncthreads();
            SigPhases<DT, WANT_IDX, L + 1, D0, Rest...>::run(k, t, lds);
        }
    }
};

template <class L1, class...>
struct FirstLvl {
    using type = L1;
};

template <int DT, int VEC, bool WANT_IDX, int EW0, class... Ls>
__global__ __launch_bounds__(512) void lds_sig_kernel(const LdsSeqK k)
{
    extern __shared__ __align__(16) float lds[];
    constexpr int NL = (int)sizeof...(Ls);
    constexpr int D0 = sig_delta0<VEC, Ls...>();
    const TileCtx t = tile_ctx(k);
    {
        int32_t r0 = t.ti * k.TH, c0 = t.tj * k.TW;
#pragma unroll
        for (int l = NL; l >= 1; --l) origin_step(k.pool[l], r0, c0);
        phase0<DT, VEC, EwList<EW0>>(k, t, lds, r0, c0, pad_value(typename FirstLvl<Ls...>::type::P(k.pool[1])));
    }
    __syncthreads();
    SigPhases<DT, WANT_IDX, 1, D0, Ls...>::run(k, t, lds);
}

// =============================================================================
// Repeated build: every level has the same pooling shape and element-wise list (the
// blocks of Section 5.1 stacked L deep); L is read at run time, the phase code is the
// signature build's.  The first phase reads the level-0 rows, whose rectangle starts
// delta0 & 3 floats into an aligned vector: one instance per value.
// =============================================================================
template <int DT, int VEC, bool WANT_IDX, int EW0, class LV>
__global__ __launch_bounds__(512) void lds_rep_kernel(const LdsSeqK k)
{
    extern __shared__ __align__(16) float lds[];
    using P = typename LV::P;
    using EW = typename LV::EW;
    const int32_t L = k.n_levels;
    const TileCtx t = tile_ctx(k);
    {
        int32_t r0 = t.ti * k.TH, c0 = t.tj * k.TW;
        for (int32_t l = L; l >= 1; --l) origin_step(k.pool[l], r0, c0);
        phase0<DT, VEC, EwList<EW0>>(k, t, lds, r0, c0, pad_value(P(k.pool[1])));
    }
    __syncthreads();
    for (int32_t l = 1; l <= L; ++l) {
        const PhaseCtx cx = phase_ctx(k, t, lds, l);
        const P p(k.pool[l]);
        const LevelK &lv = k.level[l], &pv = k.level[l - 1];
        const int32_t d = cx.d_lo & 3;
        if (cx.last) {
            if (d == 0) pool_phase<DT, P, EW, 0, WANT_IDX, true>(k, t, lv, pv, p, cx);
            else if (d == 1) pool_phase<DT, P, EW, 1, WANT_IDX, true>(k, t, lv, pv, p, cx);
            else if (d == 2) pool_phase<DT, P, EW, 2, WANT_IDX, true>(k, t, lv, pv, p, cx);
            else pool_phase<DT, P, EW, 3, WANT_IDX, true>(k, t, lv, pv, p, cx);
        } else {
            if (d == 0) pool_phase<DT, P, EW, 0, WANT_IDX, false>(k, t, lv, pv, p, cx);
            else if (d == 1) pool_phase<DT, P, EW, 1, WANT_IDX, false>(k, t, lv, pv, p, cx);
            else if (d == 2) pool_phase<DT, P, EW, 2, WANT_IDX, false>(k, t, lv, pv, p, cx);
            else pool_phase<DT, P, EW, 3, WANT_IDX, false>(k, t, lv, pv, p, cx);
            __syncthreads();
        }
    }
}

}  // namespace bs
