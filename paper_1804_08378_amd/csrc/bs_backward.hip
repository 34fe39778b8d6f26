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
#include "bs_xrows_device.h"
#include "bs_internal.h"

namespace bs {


// Build with -DBS_BWD_AUDIT to check every element offset into the stage input, the upstream gradient and the
// input gradient against the extents the host passes (k.audit_lim[0..2], in elements) before it is used: an
// offset outside is counted in k.audit[site] and replaced by 0, so such a build cannot read or write outside
// those tensors.  Without the macro the checks compile to nothing.
#if defined(BS_BWD_AUDIT)
BS_DEV uint32_t audited(const BwdK &k, int which, int site, uint32_t off, uint32_t n)
{
    if (k.audit && (uint64_t)off + n > k.audit_lim[which]) {
        atomicAdd(&k.audit[site], 1u);
        return 0u;
    }
    return off;
}
#else
BS_DEV uint32_t audited(const BwdK &, int, int, uint32_t off, uint32_t) { return off; }
#endif

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

// Forward pass of the stage's element-wise list on R register rows of VEC cells each (row j
// starts at element offset off[j] and lies in channel c[j]), collecting for every cell the
// product t of the operations' derivatives and, for the n-th Add, the product r[n] of the
// derivatives of the operations after it (0 for Adds the list does not have).
// CL: channels-last -- the VEC cells of a row are consecutive channels c[j] .. c[j] + VEC - 1 of one
// pixel (all rows hold the same channels), so BatchNorm parameters are per-cell vectors.
// NR: residual gradients kept (K_MAX_RES, or 0 for a stage without Add: no registers for them).
// FLAT (row-major only): nfirst[j] cells of row j lie in channel c[j], the rest in the next channel
// (a vector that straddles two planes).  Otherwise every cell of row j lies in channel c[j].
// The list is k.ew[first .. first + count).
// CODE >= 0: the kinds of the list's operations are known at compile time (a code of base-K_EW_BASE digits; `count` is
// ignored) and the loop over the list unrolls into straight code; their arguments still come from k.ew.
// cache (CODE >= 0, row-major, not FLAT, all rows in one channel): scale and shift of the list's q-th operation at
// cache[2 * q], cache[2 * q + 1], read once by ew_load_cache.  A kernel that calls this in a loop and stores between the
// calls would otherwise read the parameters again in every iteration (the compiler cannot know that the stores leave
// them alone) and wait for them, with everything else it has in flight.
template <int CODE>
BS_DEV void ew_load_cache(const BwdK &k, int32_t c, int32_t first, float (&cache)[2 * (ew_code_len(CODE) > 0 ? ew_code_len(CODE) : 1)])
{
#pragma unroll
    for (int q = 0; q < ew_code_len(CODE); ++q)
        if (ew_code_kind(CODE, q) == OP_BN) {
            const int32_t arg = k.ew[first + q].arg;
            cache[2 * q] = k.params[arg + c];
            cache[2 * q + 1] = k.params[arg + k.C + c];
        }
}

template <int DT, int VEC, int R, bool CL, int NR, bool FLAT, int CODE = -1>
BS_DEV int32_t ew_sweep_impl(const BwdK &k, const int32_t (&c)[R], const uint32_t (&off)[R], float (&x)[R][VEC],
                             float (&t)[R][VEC], float (&r)[NR ? NR : 1][R][VEC], const uint32_t (&nfirst)[R], int32_t first,
                             int32_t count, const float *cache = nullptr)
{
#pragma unroll
    for (int j = 0; j < R; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            t[j][e] = 1.0f;
#pragma unroll
            for (int n = 0; n < NR; ++n) r[n][j][e] = 0.0f;
        }
    int32_t adds = 0;
    auto one = [&](const int32_t kind, const int32_t arg, const int q) {
        if (kind == OP_ADD) {
            if constexpr (NR == 0) return;  // instances for stages without Add (chosen at launch): nothing to read
            Raw<DT, VEC> raw[R];
#pragma unroll
            for (int j = 0; j < R; ++j) raw[j] = load_raw<DT, VEC, true>(k.res[adds], off[j]);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                float v[VEC];
                unpack<DT, VEC>(raw[j], v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[j][e] = round_store<DT>(x[j][e] + v[e]);
            }
            // from here on the residual's gradient collects the same factors as the input's
#pragma unroll
            for (int n = 0; n < NR; ++n)
                if (n == adds) {
#pragma unroll
                    for (int j = 0; j < R; ++j)
#pragma unroll
                        for (int e = 0; e < VEC; ++e) r[n][j][e] = 1.0f;
                }
            ++adds;
            return;
        }
        float f[R][VEC];  // d(output) / d(input) of this operation at x
        if (kind == OP_BN) {
            if constexpr (CL) {
                // tables start at multiples of 8 floats and c[0], C are multiples of VEC: 128-bit loads
                float sc[VEC], sh[VEC];
                if constexpr (VEC % 4 == 0) {
#pragma unroll
                    for (int q = 0; q < VEC / 4; ++q) {
                        const float4 a = *reinterpret_cast<const float4 *>(k.params + arg + c[0] + 4 * q);
                        const float4 b = *reinterpret_cast<const float4 *>(k.params + arg + k.C + c[0] + 4 * q);
                        sc[4 * q] = a.x; sc[4 * q + 1] = a.y; sc[4 * q + 2] = a.z; sc[4 * q + 3] = a.w;
                        sh[4 * q] = b.x; sh[4 * q + 1] = b.y; sh[4 * q + 2] = b.z; sh[4 * q + 3] = b.w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        sc[e] = k.params[arg + c[0] + e];
                        sh[e] = k.params[arg + k.C + c[0] + e];
                    }
                }
#pragma unroll
                for (int j = 0; j < R; ++j)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        f[j][e] = sc[e];
                        x[j][e] = round_store<DT>(__builtin_fmaf(x[j][e], sc[e], sh[e]));
                    }
            } else {
                float sc[R], sh[R], sc1[R], sh1[R];
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    if (CODE >= 0 && !FLAT && cache) {
                        sc[j] = cache[2 * q];
                        sh[j] = cache[2 * q + 1];
                    } else {
                        sc[j] = k.params[arg + c[j]];
                        sh[j] = k.params[arg + k.C + c[j]];
                    }
                    if constexpr (FLAT) {
                        const int32_t cn = c[j] + 1 == k.C ? 0 : c[j] + 1;
                        sc1[j] = k.params[arg + cn];
                        sh1[j] = k.params[arg + k.C + cn];
                    } else {
                        sc1[j] = sc[j];
                        sh1[j] = sh[j];
                    }
                }
#pragma unroll
                for (int j = 0; j < R; ++j)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const bool first = !FLAT || (uint32_t)e < nfirst[j];
                        f[j][e] = first ? sc[j] : sc1[j];
                        x[j][e] = round_store<DT>(__builtin_fmaf(x[j][e], f[j][e], first ? sh[j] : sh1[j]));
                    }
            }
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    f[j][e] = x[j][e] > 0.0f ? 1.0f : 0.0f;
                    x[j][e] = __builtin_fmaxf(x[j][e], 0.0f);
                }
        } else if (kind == OP_LEAKY) {
            const float slope = k.params[arg];
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    f[j][e] = x[j][e] > 0.0f ? 1.0f : slope;
                    x[j][e] = round_store<DT>(x[j][e] > 0.0f ? x[j][e] : x[j][e] * slope);
                }
        } else {  // OP_CLAMP: the gradient passes where lo <= x <= hi
            const float lo = k.params[arg], hi = k.params[arg + 1];
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    f[j][e] = (x[j][e] >= lo && x[j][e] <= hi) ? 1.0f : 0.0f;
                    x[j][e] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[j][e], lo), hi));
                }
        }
#pragma unroll
        for (int j = 0; j < R; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                t[j][e] *= f[j][e];
#pragma unroll
                for (int n = 0; n < NR; ++n) r[n][j][e] *= f[j][e];
            }
    };
    if constexpr (CODE >= 0) {
#pragma unroll
        for (int q = 0; q < ew_code_len(CODE); ++q) one(ew_code_kind(CODE, q), k.ew[first + q].arg, q);
    } else {
#pragma clang loop unroll(disable)
        for (int32_t q = first; q < first + count; ++q) one(k.ew[q].kind, k.ew[q].arg, 0);
    }
    return adds;
}

template <int DT, int VEC, int R, bool CL = false, int NR = K_MAX_RES>
BS_DEV int32_t ew_sweep(const BwdK &k, const int32_t (&c)[R], const uint32_t (&off)[R], float (&x)[R][VEC], float (&t)[R][VEC],
                        float (&r)[NR ? NR : 1][R][VEC])
{
    const uint32_t none[R] = {};
    return ew_sweep_impl<DT, VEC, R, CL, NR, false>(k, c, off, x, t, r, none, 0, k.n_ew);
}

// Write grad_in = s * t and grad_residual[n] = s * r[n] for one register row.
// gin_shift: what the element's offset in g_in exceeds `off` by (channel slices).
template <int DT, int VEC, int R, int NR = K_MAX_RES>
BS_DEV void store_row(const BwdK &k, int j, uint32_t off, uint32_t gin_shift, int32_t adds, const float (&s)[VEC],
                      const float (&t)[R][VEC], const float (&r)[NR ? NR : 1][R][VEC])
{
    if (k.g_in) {
        float v[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = s[e] * t[j][e];
        store_elems<DT, VEC>(k.g_in, audited(k, 2, 23, off + gin_shift, VEC), v);
    }
#pragma unroll
    for (int n = 0; n < NR; ++n)
        if (n < adds && k.g_res[n]) {
            float v[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = s[e] * r[n][j][e];
            store_elems<DT, VEC>(k.g_res[n], off, v);
        }
}

// VEC consecutive int32 picks starting at element `off` (a multiple of VEC).
template <int VEC>
BS_DEV void load_picks(const int32_t *idx, uint32_t off, int32_t (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int q = 0; q < VEC / 4; ++q) {
            const int4 t = *reinterpret_cast<const int4 *>(idx + off + 4 * q);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = idx[off + e];
    }
}

// KH, KW, SH, SW, P: the pooling window, strides and padding (the same in both directions) when
// they are compiled in (KH == 0: read from the argument block).  With them the windows over a
// lane's cells are a fixed set -- NOH rows of NOW windows, and which cells each window holds is
// known at compile time -- so a row's gradients and picks are requested at once instead of one
// dependent round trip per window, and only the (window, cell) pairs that exist are summed.
template <int DT, int VEC, int KH, int KW, int SH, int SW, int P, int NR = K_MAX_RES>
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
    float x[1][VEC], t[1][VEC], r[NR ? NR : 1][1][VEC];
    unpack<DT, VEC>(load_raw<DT, VEC, true>(k.a, audited(k, 0, 1, off + img * k.a_extra, VEC)), x[0]);
    const uint32_t offs[1] = {off};
    const int32_t cs[1] = {c};
    const int32_t adds = ew_sweep<DT, VEC, 1, false, NR>(k, cs, offs, x, t, r);

    // ---- 2. gradient with respect to the list's output
    float s[VEC];
    const PoolK &p = k.pool;
    const uint32_t gsh = img * k.gout_extra;  // the upstream gradient's image starts this much later than a dense one's
    if (p.kind == 0) {
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.g_out, audited(k, 1, 8, off + gsh, VEC)), s);
    } else {
        const bool is_max = p.kind == OP_MAXPOOL;
        const int32_t kh = KH ? KH : p.kh, kw = KH ? KW : p.kw, sh = KH ? SH : p.sh, sw = KH ? SW : p.sw;
        // windows (oh, ow) whose rows hold ih: oh * sh - ph <= ih < oh * sh - ph + kh
        const int32_t th = ih + p.ph - kh + 1;
        const int32_t oh_lo = th <= 0 ? 0 : (th + sh - 1) / sh;
        const int32_t oh_hi = min((ih + p.ph) / sh, k.Ho - 1);
        const uint32_t obase = plane * (uint32_t)(k.Ho * k.Wo);
        // windows whose columns hold any of the lane's cells iw0 .. iw0 + VEC - 1: each is read once
        // and handed to the cells it holds, so a cell still sums its windows in row-major order
        const int32_t tw = iw0 + p.pw - kw + 1;
        const int32_t ow_lo = tw <= 0 ? 0 : (tw + sw - 1) / sw;
        const int32_t ow_hi = min((iw0 + VEC - 1 + p.pw) / sw, k.Wo - 1);
        const int32_t cell0 = ih * k.W + iw0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] = 0.0f;
        if constexpr (KH > 0) {
            // iw0 is a multiple of VEC and VEC of SW (checked at launch), so the first window over the
            // lane's cells is iw0 / SW + CQ with CQ = ceil((P - KW + 1) / SW), and window b of the row
            // begins W0(b) = (CQ + b) * SW - P cells after iw0: compile-time.  Windows left of the plane
            // (index < 0) or right of it are read at a clamped position and not used.
            constexpr int Q = P - KW + 1;
            constexpr int CQ = Q >= 0 ? (Q + SW - 1) / SW : -((-Q) / SW);
            constexpr int NOH = (KH - 1) / SH + 1, NOW = (VEC - 1 + P) / SW - CQ + 1;
            const int32_t ow0 = iw0 / SW + CQ;
#pragma unroll
            for (int a = 0; a < NOH; ++a) {
                float gv[NOW];
                int32_t pick[NOW];
                const int32_t oh = oh_lo + a;
                const uint32_t orow = obase + (uint32_t)(min(oh, k.Ho - 1) * k.Wo);
                if constexpr (SW == 1 && NOW == VEC + 2) {
                    // stride 1 (the output row is as long as the input row: checked at launch): windows
                    // iw0 - 1 .. iw0 + VEC; the middle VEC of them are one aligned vector
                    const Raw<DT, VEC> mid = load_raw<DT, VEC>(k.g_out, audited(k, 1, 9, gsh + orow + (uint32_t)iw0, VEC));
                    const Raw<DT, 1> left = load_raw<DT, 1>(k.g_out, audited(k, 1, 10, gsh + orow + (uint32_t)max(iw0 - 1, 0), 1));
                    const Raw<DT, 1> right = load_raw<DT, 1>(k.g_out, audited(k, 1, 11, gsh + orow + (uint32_t)min(iw0 + VEC, k.Wo - 1), 1));
                    if (is_max) {
                        int32_t pm[VEC];
                        load_picks<VEC>(k.idx, orow + (uint32_t)iw0, pm);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) pick[1 + e] = pm[e];
                        pick[0] = k.idx[orow + (uint32_t)max(iw0 - 1, 0)];
                        pick[VEC + 1] = k.idx[orow + (uint32_t)min(iw0 + VEC, k.Wo - 1)];
                    }
                    float gm[VEC], g1[1];
                    unpack<DT, VEC>(mid, gm);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) gv[1 + e] = gm[e];
                    unpack<DT, 1>(left, g1);
                    gv[0] = g1[0];
                    unpack<DT, 1>(right, g1);
                    gv[VEC + 1] = g1[0];
                } else if constexpr (SW == 2 && CQ == 0 && VEC >= 2 && NOW == VEC / 2 + 1) {
                    // stride 2 (the output row is half the input row: checked at launch): windows
                    // iw0 / 2 .. iw0 / 2 + VEC / 2; all but the last are one aligned vector
                    constexpr int HV = VEC / 2;
                    const Raw<DT, HV> mid = load_raw<DT, HV>(k.g_out, audited(k, 1, 12, gsh + orow + (uint32_t)ow0, HV));
                    const Raw<DT, 1> right = load_raw<DT, 1>(k.g_out, audited(k, 1, 13, gsh + orow + (uint32_t)min(ow0 + HV, k.Wo - 1), 1));
                    if (is_max) {
                        int32_t pm[HV];
                        load_picks<HV>(k.idx, orow + (uint32_t)ow0, pm);
#pragma unroll
                        for (int e = 0; e < HV; ++e) pick[e] = pm[e];
                        pick[HV] = k.idx[orow + (uint32_t)min(ow0 + HV, k.Wo - 1)];
                    }
                    float gm[HV], g1[1];
                    unpack<DT, HV>(mid, gm);
#pragma unroll
                    for (int e = 0; e < HV; ++e) gv[e] = gm[e];
                    unpack<DT, 1>(right, g1);
                    gv[HV] = g1[0];
                } else {
#pragma unroll
                    for (int b = 0; b < NOW; ++b) {
                        const uint32_t o = orow + (uint32_t)min(max(ow0 + b, 0), k.Wo - 1);
                        float g1[1];
                        unpack<DT, 1>(load_raw<DT, 1>(k.g_out, audited(k, 1, 14, gsh + o, 1)), g1);
                        gv[b] = g1[0];
                        pick[b] = is_max ? k.idx[o] : 0;
                    }
                }
#pragma unroll
                for (int b = 0; b < NOW; ++b) {
                    const int32_t ow = ow0 + b;
                    const bool in = oh <= oh_hi && ow >= 0 && ow < k.Wo;
                    const float g[1] = {gv[b]};
                    const int w0 = (CQ + b) * SW - P;  // a constant once the loop is unrolled
                    if (is_max) {
                        const int32_t d = pick[b] - cell0;
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (e >= w0 && e < w0 + KW) s[e] += (in && d == e) ? g[0] : 0.0f;
                    } else {
                        const float gi = in ? g[0] * bwd_avg_inv(p, k.H, k.W, min(oh, k.Ho - 1), min(max(ow, 0), k.Wo - 1)) : 0.0f;
#pragma unroll
                        for (int e = 0; e < VEC; ++e)
                            if (e >= w0 && e < w0 + KW) s[e] += gi;
                    }
                }
            }
        } else
        for (int32_t oh = oh_lo; oh <= oh_hi; ++oh)
            for (int32_t ow = ow_lo; ow <= ow_hi; ++ow) {
                const uint32_t o = obase + (uint32_t)(oh * k.Wo + ow);  // 0 <= oh < Ho, 0 <= ow < Wo
                float g[1];
                unpack<DT, 1>(load_raw<DT, 1>(k.g_out, audited(k, 1, 15, gsh + o, 1)), g);
                if (is_max) {
                    const int32_t d = k.idx[o] - cell0;  // the pick is one of the lane's cells if 0 <= d < VEC
#pragma unroll
                    for (int e = 0; e < VEC; ++e) s[e] += d == e ? g[0] : 0.0f;
                } else {
                    const float gi = g[0] * bwd_avg_inv(p, k.H, k.W, oh, ow);
                    const int32_t w0 = ow * p.sw - p.pw - iw0;  // the window's columns, relative to the lane's first
#pragma unroll
                    for (int e = 0; e < VEC; ++e) s[e] += (e >= w0 && e < w0 + p.kw) ? gi : 0.0f;
                }
            }
    }

    // ---- 3. results
    if (live) store_row<DT, VEC, 1, NR>(k, 0, off, img * k.gin_extra, adds, s, t, r);
}

// =============================================================================
// bwd_ew_kernel: a stage without pooling (BatchNorm -> Add -> ReLU of a residual block,
// BatchNorm -> ReLU of a dense layer) whose planes are whole vectors.  The tensor is one run of
// vectors; a work-group takes nthr * U consecutive ones, lane t the vectors t, t + nthr, ...:
// U independent loads of every operand in flight per lane.
// =============================================================================
// PRE: the kinds of the list as a compile-time code (ew_sweep_impl), or -1: read at run time.
template <int DT, int VEC, int U, int NR, int PRE = -1>
__global__ __launch_bounds__(256) void bwd_ew_kernel(const BwdK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t nvec = k.total;                      // vectors in the tensor
    bool live[U];
    uint32_t offs[U], nfirst[U], imgs[U];
    int32_t cs[U];
    Raw<DT, VEC> ar[U], gr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        live[u] = i < nvec;
        i = live[u] ? i : 0u;
        offs[u] = i * VEC;
        uint32_t plane;
        if (k.flat) {
            // vectors over the whole tensor: this one begins in `plane` and may end in the next one
            // (never further: a plane has at least VEC cells)
            plane = fdiv(offs[u], k.div_w);
            nfirst[u] = k.div_w.d - (offs[u] - plane * k.div_w.d);
        } else {
            plane = fdiv(fdiv(i, k.div_wv), k.div_h);  // i / (W / VEC) / H
            nfirst[u] = VEC;
        }
        imgs[u] = fdiv(plane, k.div_c);  // a vector lies in one image (checked at launch when the tensors are slices)
        cs[u] = (int32_t)(plane - imgs[u] * (uint32_t)k.C);
        ar[u] = load_raw<DT, VEC, true>(k.a, audited(k, 0, 2, offs[u] + imgs[u] * k.a_extra, VEC));
        gr[u] = load_raw<DT, VEC, true>(k.g_out, audited(k, 1, 16, offs[u] + imgs[u] * k.gout_extra, VEC));
    }
    float x[U][VEC], t[U][VEC], r[NR ? NR : 1][U][VEC], s[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        unpack<DT, VEC>(ar[u], x[u]);
        unpack<DT, VEC>(gr[u], s[u]);
    }
    const int32_t adds = k.flat ? ew_sweep_impl<DT, VEC, U, false, NR, true, PRE>(k, cs, offs, x, t, r, nfirst, 0, k.n_ew)
                                : ew_sweep_impl<DT, VEC, U, false, NR, false, PRE>(k, cs, offs, x, t, r, nfirst, 0, k.n_ew);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) store_row<DT, VEC, U, NR>(k, u, offs[u], imgs[u] * k.gin_extra, adds, s[u], t, r);
}

// =============================================================================
// bwd_direct2_kernel: a stage whose pooling has disjoint 2 x 2 windows that tile the plane
// (2 x 2 / stride 2, no padding, even H, whole vectors per row): BatchNorm -> ReLU -> MaxPool of
// the VGG stacks, the average pooling of a DenseNet transition.  Every input cell lies in exactly
// one window, so a lane takes whole windows -- two input rows of VEC cells, VEC / 2 windows -- runs
// the element-wise list on them, finds each max-pooling pick itself (first maximum in row-major
// order, as the forward kernels do) and writes the gradients of all its cells.  No recorded
// picks, no recomputation pass: the stage input and the gradient with respect to it move once.
// =============================================================================
// PRE: the kinds of the stage's element-wise list as a compile-time code (ew_sweep_impl), or -1: read at run time.
template <int DT, int VEC, int NR, int PRE = -1>
__global__ __launch_bounds__(256) void bwd_direct2_kernel(const BwdK k)
{
    constexpr int NO = VEC / 2;
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t rowo = fdiv(i, k.div_wv);          // plane * Ho + oh
    const uint32_t cv = i - rowo * k.div_wv.d;
    const uint32_t plane = fdiv(rowo, k.div_h);       // div_h divides by Ho here
    const uint32_t oh = rowo - plane * (uint32_t)k.Ho;
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c = (int32_t)(plane - img * (uint32_t)k.C);
    // rows 2 * oh and 2 * oh + 1 < H = 2 * Ho, columns cv * VEC .. + VEC - 1 < W
    const uint32_t offs[2] = {(plane * (uint32_t)k.H + 2 * oh) * (uint32_t)k.W + cv * VEC,
                              (plane * (uint32_t)k.H + 2 * oh + 1) * (uint32_t)k.W + cv * VEC};
    const uint32_t out_off = rowo * (uint32_t)k.Wo + cv * NO;  // Wo = W / 2: NO outputs of row oh

    const uint32_t ash = img * k.a_extra;
    const Raw<DT, VEC> a0 = load_raw<DT, VEC, true>(k.a, audited(k, 0, 3, offs[0] + ash, VEC)), a1 = load_raw<DT, VEC, true>(k.a, audited(k, 0, 4, offs[1] + ash, VEC));
    const Raw<DT, NO> gr = load_raw<DT, NO, true>(k.g_out, audited(k, 1, 17, out_off + img * k.gout_extra, NO));
    float x[2][VEC], t[2][VEC], r[NR ? NR : 1][2][VEC], g[NO];
    unpack<DT, VEC>(a0, x[0]);
    unpack<DT, VEC>(a1, x[1]);
    unpack<DT, NO>(gr, g);
    const int32_t cs[2] = {c, c};
    const uint32_t whole[2] = {};
    const int32_t adds = ew_sweep_impl<DT, VEC, 2, false, NR, false, PRE>(k, cs, offs, x, t, r, whole, 0, k.n_ew);

    float s[2][VEC];
    if (k.pool.kind == OP_MAXPOOL) {
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            float best = -INFINITY;
            int pick = 0;
#pragma unroll
            for (int dh = 0; dh < 2; ++dh)
#pragma unroll
                for (int dw = 0; dw < 2; ++dw) {
                    const bool more = x[dh][2 * j + dw] > best;
                    best = more ? x[dh][2 * j + dw] : best;
                    pick = more ? dh * 2 + dw : pick;
                }
#pragma unroll
            for (int dh = 0; dh < 2; ++dh)
#pragma unroll
                for (int dw = 0; dw < 2; ++dw) s[dh][2 * j + dw] = pick == dh * 2 + dw ? g[j] : 0.0f;
        }
    } else {
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            const float gi = g[j] * k.pool.inv_kk;  // every window lies inside the plane: the divisor is 4
#pragma unroll
            for (int dh = 0; dh < 2; ++dh)
#pragma unroll
                for (int dw = 0; dw < 2; ++dw) s[dh][2 * j + dw] = gi;
        }
    }
    if (!live) return;
    store_row<DT, VEC, 2, NR>(k, 0, offs[0], img * k.gin_extra, adds, s[0], t, r);
    store_row<DT, VEC, 2, NR>(k, 1, offs[1], img * k.gin_extra, adds, s[1], t, r);
}

// =============================================================================
// bwd_rows_kernel: a stage whose pooling has overlapping 3 x 3 windows (padding 1, stride S = 1 or
// 2; BatchNorm -> ReLU -> MaxPool of the ResNet stem, the stacked pooling blocks of Section 4.4)
// on planes whose rows fit one wave.  No recorded picks and no recomputation pass: the stage
// input, the upstream gradient and the gradient with respect to the input move once.
//
// The lanes of a plane's row sit side by side in one wave (a lane owns one column block of VEC
// cells, as in the forward sliding-window kernels) and walk down a chunk of rows.  A lane keeps
// the three input rows of the current window row in registers: the values after the element-wise
// list (with its neighbours' edge columns, one lane-shift each), the list's derivative factors,
// and the gradient sums collected so far.  Per window row it reads S new input rows and its VO =
// VEC / S upstream gradients and writes the S rows no later window touches.
//   Max pooling: the lane finds each of its windows' first maximum (row-major, as the forward
//   kernels do) and adds the window's gradient to the picked cell -- a pick in a neighbour's
//   column travels there by one lane-shift.  Element-wise operations behind the pooling
//   (k.n_post of them) are differentiated at the window maximum, which is the pooling's output.
//   Average pooling: every window's gradient, times the reciprocal of the divisor the forward
//   pass used, goes to all of the window's cells; the windows of the neighbouring lanes that
//   reach into the block arrive by lane-shift.
// A cell sums its windows in row-major window order (earlier window rows first; within a row the
// left neighbour's window, the lane's own windows from left to right, the right neighbour's
// window): no atomics, the same bits on every run.
//
// Chunks overlap: the rows a chunk writes are [rc * S * chunk, rc * S * (chunk + 1)) (to the end
// of the plane for the last one); it also visits the window row above and the one below, whose
// other rows belong to the neighbouring chunks.  Every lane of a wave runs the same number of
// iterations whether or not its windows exist.
// =============================================================================
// PRE: the kinds of the stage's element-wise list as a compile-time code (ew_sweep_impl), or -1: read at run time.
template <int DT, int VEC, int S, int NR, bool MAX, int PRE = -1>
__global__ __launch_bounds__(256) void bwd_rows_kernel(const BwdK k)
{
    constexpr int K = 3, P = 1, VO = VEC / S, NL = P, NX = K - S - P, CW = NL + VEC + NX;
    constexpr int KEEP = K - S;  // rows two consecutive window rows share
    static_assert(VEC % S == 0 && (S == 1 || S == 2), "strides of the compiled windows");
    const XLane L = xrows_lane(k);
    const int32_t col0 = L.j * VEC;
    const bool has_left = L.j > 0, has_right = L.j + 1 < k.cbs;
    const uint32_t plane_off = L.plane * (uint32_t)(k.H * k.W), oplane = L.plane * (uint32_t)(k.Ho * k.Wo);
    // rows this chunk writes
    const int32_t r_lo = L.chunk * k.rc * S, r_hi = L.chunk + 1 == k.chunks ? k.H : min(r_lo + k.rc * S, k.H);
    // window rows it visits: the first that holds row r_lo .. the last that holds a row below r_lo + rc * S
    constexpr int OFIRST = -((K - 1 - P) / S);  // ceil((P - K + 1) / S)
    constexpr int OEND = (P + S - 1) / S;
    const int32_t oh_first = L.chunk * k.rc + OFIRST;
    // the last chunk goes on until every row of the plane is written (rows below the last window get zeros)
    const int32_t n_iter = max(k.rc, (k.H - (k.chunks - 1) * k.rc * S + S - 1) / S) + OEND - OFIRST;  // the same for every lane

    float y[K][CW], t[K][VEC], r[NR ? NR : 1][K][VEC], s[K][VEC];
    int32_t adds = 0;
    // rows [first, first + N) of the plane -> ring slots [slot, slot + N): element-wise list, padding, edge columns
    auto take_rows = [&](auto n_tag, int slot, int32_t first) {
        constexpr int N = decltype(n_tag)::value;
        float xs[N][VEC], ts[N][VEC], rs[NR ? NR : 1][N][VEC];
        uint32_t offs[N];
        int32_t cs[N];
        Raw<DT, VEC> raw[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            offs[j] = plane_off + (uint32_t)(min(max(first + j, 0), k.H - 1) * k.W + col0);  // outside the plane: a safe row, replaced below
            cs[j] = L.c;
            raw[j] = load_raw<DT, VEC, true>(k.a, audited(k, 0, 5, offs[j] + L.img * k.a_extra, VEC));
        }
#pragma unroll
        for (int j = 0; j < N; ++j) unpack<DT, VEC>(raw[j], xs[j]);
        const uint32_t whole[N] = {};
        adds = ew_sweep_impl<DT, VEC, N, false, NR, false, PRE>(k, cs, offs, xs, ts, rs, whole, 0, k.n_ew);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const bool ok = first + j >= 0 && first + j < k.H;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                xs[j][e] = ok ? xs[j][e] : -INFINITY;
                t[slot + j][e] = ts[j][e];
                s[slot + j][e] = 0.0f;
#pragma unroll
                for (int n = 0; n < NR; ++n) r[n][slot + j][e] = rs[n][j][e];
            }
            with_neighbours<VEC, NL, NX>(xs[j], y[slot + j], has_left, has_right, -INFINITY);
        }
    };
    if constexpr (KEEP > 0) take_rows(std::integral_constant<int, KEEP>{}, 0, oh_first * S - P);

    for (int32_t it = 0; it < n_iter; ++it) {
        const int32_t oh = oh_first + it, hA = oh * S - P;
        take_rows(std::integral_constant<int, S>{}, KEEP, hA + KEEP);
        // upstream gradients of the lane's windows of this row; windows that do not exist give nothing
        const bool row_ok = oh >= 0 && oh < k.Ho;
        float g[VO];
        unpack<DT, VO>(load_raw<DT, VO>(k.g_out, audited(k, 1, 18, L.img * k.gout_extra + oplane + (uint32_t)(min(max(oh, 0), k.Ho - 1) * k.Wo + L.j * VO), VO)), g);
#pragma unroll
        for (int e = 0; e < VO; ++e) g[e] = row_ok ? g[e] : 0.0f;
        if constexpr (MAX) {
            // first maximum of every window: code = window row * K + window column
            int32_t pick[VO];
            float best[1][VO];
#pragma unroll
            for (int e = 0; e < VO; ++e) {
                best[0][e] = -INFINITY;
                pick[e] = -1;
#pragma unroll
                for (int dh = 0; dh < K; ++dh)
#pragma unroll
                    for (int dw = 0; dw < K; ++dw) {
                        const float v = y[dh][e * S + dw];
                        const bool more = v > best[0][e];
                        best[0][e] = more ? v : best[0][e];
                        pick[e] = more ? dh * K + dw : pick[e];
                    }
            }
            // element-wise operations behind the pooling: their derivative at the window's maximum (the pooling's
            // output, as the forward pass rounded it) scales the window's gradient
            if (k.n_post > 0) {
                float tp[1][VO], none[1][1][VO];
                const uint32_t no_off[1] = {0}, all[1] = {VO};
                const int32_t cs[1] = {L.c};
#pragma unroll
                for (int e = 0; e < VO; ++e) best[0][e] = row_ok ? best[0][e] : 0.0f;  // windows that do not exist: any finite value
                ew_sweep_impl<DT, VO, 1, false, 0, false>(k, cs, no_off, best, tp, none, all, k.n_ew, k.n_post);
#pragma unroll
                for (int e = 0; e < VO; ++e) g[e] *= tp[0][e];
            }
            // gradients into the picked cells, in the order a cell's windows have in the plane
#pragma unroll
            for (int dh = 0; dh < K; ++dh) {
                // picks in the neighbours' columns: the first window's first column lies in the left lane's block,
                // the last window's last column (stride 1) in the right lane's
                const float to_left = pick[0] == dh * K ? g[0] : 0.0f;
                const float from_right = from_right_lane(to_left);
                if constexpr (NX > 0) {
                    const float to_right = pick[VO - 1] == dh * K + K - 1 ? g[VO - 1] : 0.0f;
                    const float from_left = from_left_lane(to_right);
                    s[dh][0] += has_left ? from_left : 0.0f;
                }
#pragma unroll
                for (int e = 0; e < VO; ++e)
#pragma unroll
                    for (int dw = 0; dw < K; ++dw) {
                        const int col = e * S + dw - NL;  // the window cell's column in the lane's block
                        if (col >= 0 && col < VEC) s[dh][col] += pick[e] == dh * K + dw ? g[e] : 0.0f;
                    }
                s[dh][VEC - 1] += has_right ? from_right : 0.0f;
            }
        } else {
            // every window hands its gradient times the reciprocal of its divisor to all its cells: the same
            // per-column sums for the K rows of this window row, in the plane's window order
#pragma unroll
            for (int e = 0; e < VO; ++e)
                g[e] *= bwd_avg_inv(k.pool, k.H, k.W, min(max(oh, 0), k.Ho - 1), L.j * VO + e);
            float add[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) add[e] = 0.0f;
            const float from_right = from_right_lane(g[0]);  // the right lane's first window holds this lane's last column
            if constexpr (NX > 0) {
                const float from_left = from_left_lane(g[VO - 1]);  // stride 1: the left lane's last window holds the first
                add[0] += has_left ? from_left : 0.0f;
            }
#pragma unroll
            for (int e = 0; e < VO; ++e)
#pragma unroll
                for (int dw = 0; dw < K; ++dw) {
                    const int col = e * S + dw - NL;
                    if (col >= 0 && col < VEC) add[col] += g[e];
                }
            add[VEC - 1] += has_right ? from_right : 0.0f;
#pragma unroll
            for (int dh = 0; dh < K; ++dh)
#pragma unroll
                for (int e = 0; e < VEC; ++e) s[dh][e] += add[e];
        }
        // the S rows no later window row holds are complete
#pragma unroll
        for (int d = 0; d < S; ++d) {
            const int32_t row = hA + d;
            if (L.live && row >= r_lo && row < r_hi)
                store_row<DT, VEC, K, NR>(k, d, plane_off + (uint32_t)(row * k.W + col0), L.img * k.gin_extra, adds, s[d], t, r);
        }
#pragma unroll
        for (int d = 0; d < KEEP; ++d) {
#pragma unroll
            for (int e = 0; e < CW; ++e) y[d][e] = y[d + S][e];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                t[d][e] = t[d + S][e];
                s[d][e] = s[d + S][e];
#pragma unroll
                for (int n = 0; n < NR; ++n) r[n][d][e] = r[n][d + S][e];
            }
        }
    }
}

// =============================================================================
// bwd_rows2_kernel: two stages in one kernel -- element-wise list, average pooling 3 x 3 (stride 1,
// padding 1), then max pooling 3 x 3 (stride 2, padding 1) with element-wise operations behind it
// (the stacked pooling of Section 4.4 with its activation) -- on planes whose rows fit one wave.
// The stack's input and the upstream gradient are read once and the input gradient is written
// once; nothing is recomputed by another kernel and nothing passes through the workspace.
//
// As in bwd_rows_kernel the lanes of a row sit side by side in one wave and walk down a chunk of
// rows; per window row `oh` of the max pooling a lane
//   1. reads two new input rows (2 oh + 1, 2 oh + 2), applies the leading list (values y, derivative T),
//   2. forms the two new rows (2 oh, 2 oh + 1) of the average pooling's output `a` in the forward
//      kernels' arithmetic (row-major sum from +0, times the divisor's reciprocal, rounded to storage),
//   3. finds the picks of its max windows over a rows 2 oh - 1 .. 2 oh + 1, scales the upstream
//      gradients by the trailing list's derivative at the maxima and adds them to the picked cells
//      (sums per a row; a pick in the left neighbour's column travels there by a lane shift),
//   4. a rows 2 oh - 1 and 2 oh can get nothing more: their gradients, times the reciprocal of the
//      average's divisor, are summed over the three windows of the row that hold a cell (the
//      neighbours' edge columns by lane shifts): rows of `hs`,
//   5. writes the input gradient of rows 2 oh - 2 and 2 oh - 1: hs of the rows above, at and below, times T.
// Rings: y rows 2 oh - 1 .. 2 oh + 2, T rows 2 oh - 2 .. 2 oh + 2, a rows 2 oh - 1 .. 2 oh + 1 and their
// gradient sums, hs rows 2 oh - 3 .. 2 oh.  A chunk of rc window rows writes input rows
// [2 rc chunk, 2 rc (chunk + 1)) and visits window rows rc chunk - 1 .. rc (chunk + 1); every lane of
// a wave runs the same number of iterations.  Sums have a fixed order: the same bits on every run.
// The gradient between the two poolings stays in float32 registers (it is not rounded to the
// storage type as it is between stages that run as separate kernels).
// =============================================================================
// PRE, POST: the kinds of the leading and the trailing list as compile-time codes (ew_sweep_impl), or -1: read at run time.
// Waves per SIMD the register allocator is held to (measured on MI355X, halo_stress float32: 3 -> 146 us, 4 -> 134 us, 5 -> 151 us).
#if !defined(BS_ROWS2_WAVES)
#define BS_ROWS2_WAVES 4
#endif
template <int DT, int VEC, int PRE, int POST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(BS_ROWS2_WAVES, BS_ROWS2_WAVES))) void bwd_rows2_kernel(const BwdK k)
{
    constexpr int K = 3, S = 2, VO = VEC / S;
    constexpr int YW = VEC + 2, AW = VEC + 1;  // a row with both neighbours' edge columns / with the left one
    static_assert(VEC % S == 0, "whole windows per lane");
    const XLane L = xrows_lane(k);
    const int32_t col0 = L.j * VEC;
    const bool has_left = L.j > 0, has_right = L.j + 1 < k.cbs;
    const uint32_t plane_off = L.plane * (uint32_t)(k.H * k.W), oplane = L.plane * (uint32_t)(k.Ho * k.Wo);
    const int32_t r_lo = L.chunk * k.rc * S, r_hi = L.chunk + 1 == k.chunks ? k.H : min(r_lo + k.rc * S, k.H);
    // a chunk starts one window row early (that row's windows reach into the chunk's first row) -- not when the chunk is
    // the whole plane: there is no window row above the first
    const int32_t lead = k.chunks > 1 ? 1 : 0;
    const int32_t oh_first = L.chunk * k.rc - lead;
    const int32_t n_iter = max(k.rc, (k.H - (k.chunks - 1) * k.rc * S + S - 1) / S) + 1 + lead;  // the same for every lane

    float yf[4][YW], T[5][VEC], af[3][AW], gt[3][VEC], hs[4][VEC];
    const int32_t cs1[1] = {L.c};
    // both lists' BatchNorm parameters of the lane's channel
    float pre_par[2 * (ew_code_len(PRE) > 0 ? ew_code_len(PRE) : 1)], post_par[2 * (ew_code_len(POST) > 0 ? ew_code_len(POST) : 1)];
    if constexpr (PRE >= 0) ew_load_cache<PRE>(k, L.c, 0, pre_par);
    if constexpr (POST >= 0) ew_load_cache<POST>(k, L.c, k.n_ew, post_par);

    // rows [first, first + N) of the plane: leading element-wise list -> y with edge columns (padding +0: the
    // average's) into yf[slot ..], derivative factors into T[tslot ..]
    auto take_rows = [&](auto n_tag, int slot, int tslot, int32_t first) {
        constexpr int N = decltype(n_tag)::value;
        float xs[N][VEC], ts[N][VEC], none[1][N][VEC];
        uint32_t offs[N];
        int32_t cs[N];
        Raw<DT, VEC> raw[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            offs[j] = plane_off + (uint32_t)(min(max(first + j, 0), k.H - 1) * k.W + col0);  // outside the plane: a safe row, replaced below
            cs[j] = L.c;
            raw[j] = load_raw<DT, VEC, true>(k.a, audited(k, 0, 30, offs[j] + L.img * k.a_extra, VEC));
        }
#pragma unroll
        for (int j = 0; j < N; ++j) unpack<DT, VEC>(raw[j], xs[j]);
        const uint32_t whole[N] = {};
        ew_sweep_impl<DT, VEC, N, false, 0, false, PRE>(k, cs, offs, xs, ts, none, whole, 0, k.n_ew, PRE >= 0 ? pre_par : nullptr);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const bool ok = first + j >= 0 && first + j < k.H;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                xs[j][e] = ok ? xs[j][e] : 0.0f;
                T[tslot + j][e] = ts[j][e];
            }
            with_neighbours<VEC, 1, 1>(xs[j], yf[slot + j], has_left, has_right, 0.0f);
        }
    };
    // row `row` of the average pooling's output from y rows yf[slot .. slot + 2] -> af[aslot] (outside the
    // plane: the max pooling's padding)
    auto average_row = [&](int slot, int aslot, int32_t row) {
        float v[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = xrows_window_sum<K, K, false, YW>(yf + slot, e);
        xrows_normalise<DT, VEC, K, K, 1, 1, 1>(v, k.pool, row - 1, col0 - 1, k.H, k.W);
        const bool ok = row >= 0 && row < k.H;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = ok ? v[e] : -INFINITY;
        with_neighbours<VEC, 1, 0>(v, af[aslot], has_left, has_right, -INFINITY);
    };

#pragma unroll
    for (int d = 0; d < 3; ++d)
#pragma unroll
        for (int e = 0; e < VEC; ++e) gt[d][e] = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int e = 0; e < VEC; ++e) hs[d][e] = 0.0f;
    // y rows 2 oh - 2 .. 2 oh of the first window row -> a row 2 oh - 1; y rows 2 oh - 1, 2 oh stay
    take_rows(std::integral_constant<int, 3>{}, 0, 0, oh_first * S - 2);
    average_row(0, 0, oh_first * S - 1);
#pragma unroll
    for (int e = 0; e < YW; ++e) {
        yf[0][e] = yf[1][e];
        yf[1][e] = yf[2][e];
    }

    for (int32_t it = 0; it < n_iter; ++it) {
        const int32_t oh = oh_first + it, hA = oh * S - 1;  // a rows hA .. hA + 2 under this window row
        take_rows(std::integral_constant<int, 2>{}, 2, 3, hA + 2);
        // upstream gradients of the lane's windows of this row; windows that do not exist give nothing
        const bool row_ok = oh >= 0 && oh < k.Ho;
        float g[VO];
        unpack<DT, VO>(load_raw<DT, VO>(k.g_out, audited(k, 1, 31, L.img * k.gout_extra + oplane + (uint32_t)(min(max(oh, 0), k.Ho - 1) * k.Wo + L.j * VO), VO)), g);
#pragma unroll
        for (int e = 0; e < VO; ++e) g[e] = row_ok ? g[e] : 0.0f;
        average_row(0, 1, hA + 1);
        average_row(1, 2, hA + 2);
        // first maximum of every window: code = window row * K + window column
        int32_t pick[VO];
        float best[1][VO];
#pragma unroll
        for (int e = 0; e < VO; ++e) {
            best[0][e] = -INFINITY;
            pick[e] = -1;
#pragma unroll
            for (int dh = 0; dh < K; ++dh)
#pragma unroll
                for (int dw = 0; dw < K; ++dw) {
                    const float v = af[dh][e * S + dw];
                    const bool more = v > best[0][e];
                    best[0][e] = more ? v : best[0][e];
                    pick[e] = more ? dh * K + dw : pick[e];
                }
        }
        // element-wise operations behind the max pooling: their derivative at the window's maximum
        if (k.n_post > 0) {
            float tp[1][VO], none[1][1][VO];
            const uint32_t no_off[1] = {0}, all[1] = {VO};
#pragma unroll
            for (int e = 0; e < VO; ++e) best[0][e] = row_ok ? best[0][e] : 0.0f;  // windows that do not exist: any finite value
            ew_sweep_impl<DT, VO, 1, false, 0, false, POST>(k, cs1, no_off, best, tp, none, all, k.n_ew, k.n_post,
                                                            POST >= 0 ? post_par : nullptr);
#pragma unroll
            for (int e = 0; e < VO; ++e) g[e] *= tp[0][e];
        }
        // gradients into the picked cells of the a rows, in the order a cell's windows have in the plane
#pragma unroll
        for (int dh = 0; dh < K; ++dh) {
            const float to_left = pick[0] == dh * K ? g[0] : 0.0f;  // the first window's first column is the left lane's last
            const float from_right = from_right_lane(to_left);
#pragma unroll
            for (int e = 0; e < VO; ++e)
#pragma unroll
                for (int dw = 0; dw < K; ++dw) {
                    const int col = e * S + dw - 1;
                    if (col >= 0 && col < VEC) gt[dh][col] += pick[e] == dh * K + dw ? g[e] : 0.0f;
                }
            gt[dh][VEC - 1] += has_right ? from_right : 0.0f;
        }
        // a rows hA and hA + 1 are complete: times the reciprocal of the average's divisor; per cell the sum over the
        // three windows of that row that hold it (the neighbours' edge columns by lane shifts)
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int32_t row = min(max(hA + d, 0), k.H - 1);  // rows outside the plane hold zeros
            float w[VEC], wf[YW];
#pragma unroll
            for (int e = 0; e < VEC; ++e) w[e] = gt[d][e] * bwd_avg_inv(k.pool, k.H, k.W, row, col0 + e);
            with_neighbours<VEC, 1, 1>(w, wf, has_left, has_right, 0.0f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) hs[2 + d][e] = (wf[e] + wf[e + 1]) + wf[e + 2];
        }
        // input rows hA - 1 and hA: the window rows above, at and below the cell, times the list's derivative
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int32_t row = hA - 1 + d;
            float v[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = ((hs[d][e] + hs[d + 1][e]) + hs[d + 2][e]) * T[d][e];
            if (L.live && row >= r_lo && row < r_hi && k.g_in)
                store_elems<DT, VEC>(k.g_in, audited(k, 2, 32, plane_off + (uint32_t)(row * k.W + col0) + L.img * k.gin_extra, VEC), v);
        }
        // next window row: two rows down
#pragma unroll
        for (int e = 0; e < YW; ++e) {
            yf[0][e] = yf[2][e];
            yf[1][e] = yf[3][e];
        }
#pragma unroll
        for (int e = 0; e < AW; ++e) af[0][e] = af[2][e];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            T[0][e] = T[2][e];
            T[1][e] = T[3][e];
            T[2][e] = T[4][e];
            hs[0][e] = hs[2][e];
            hs[1][e] = hs[3][e];
            gt[0][e] = gt[2][e];
            gt[1][e] = 0.0f;
            gt[2][e] = 0.0f;
        }
    }
}

// =============================================================================
// Channels-last tensors (N, H, W, C in memory).  A lane owns VEC consecutive channels of one
// pixel: the same three steps as bwd_stage_kernel, with BatchNorm parameters as per-lane
// vectors and a window's gradient and picks as one vector each (the VEC channels of the output
// pixel), so every access of a wave is contiguous.
// =============================================================================
// NOH, NOW: compile-time bounds on the windows over one pixel (ceil(kh / sh) x ceil(kw / sw)),
// 0 = loops with run-time bounds.  With them all windows' gradients and picks are requested at once.
template <int DT, int VEC, int NOH, int NOW, int NR = K_MAX_RES>
__global__ __launch_bounds__(256) void bwd_stage_nhwc_kernel(const BwdK k)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t pix = fdiv(i, k.div_wv);            // (n * H + ih) * W + iw
    const uint32_t cv = i - pix * k.div_wv.d;
    const uint32_t row = fdiv(pix, k.div_w);           // n * H + ih
    const int32_t iw = (int32_t)(pix - row * (uint32_t)k.W);
    const uint32_t n = fdiv(row, k.div_h);
    const int32_t ih = (int32_t)(row - n * (uint32_t)k.H);
    const int32_t c0 = (int32_t)(cv * VEC);
    const uint32_t off = pix * (uint32_t)k.C + (uint32_t)c0;  // < N*H*W*C: i < total, or 0

    float x[1][VEC], t[1][VEC], r[NR ? NR : 1][1][VEC];
    unpack<DT, VEC>(load_raw<DT, VEC, true>(k.a, audited(k, 0, 6, off + pix * k.a_extra, VEC)), x[0]);
    const uint32_t offs[1] = {off};
    const int32_t cs[1] = {c0};
    const int32_t adds = ew_sweep<DT, VEC, 1, true, NR>(k, cs, offs, x, t, r);

    float s[VEC];
    const PoolK &p = k.pool;
    if (p.kind == 0) {
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.g_out, audited(k, 1, 19, off + pix * k.gout_extra, VEC)), s);
    } else {
        const bool is_max = p.kind == OP_MAXPOOL;
        // windows (oh, ow) that hold the pixel
        const int32_t th = ih + p.ph - p.kh + 1, tw = iw + p.pw - p.kw + 1;
        const int32_t oh_lo = th <= 0 ? 0 : (th + p.sh - 1) / p.sh, ow_lo = tw <= 0 ? 0 : (tw + p.sw - 1) / p.sw;
        const int32_t oh_hi = min((ih + p.ph) / p.sh, k.Ho - 1), ow_hi = min((iw + p.pw) / p.sw, k.Wo - 1);
        const uint32_t obase = n * (uint32_t)(k.Ho * k.Wo);
        const int32_t cell = ih * k.W + iw;
#pragma unroll
        for (int e = 0; e < VEC; ++e) s[e] = 0.0f;
        if constexpr (NOH > 0) {
            Raw<DT, VEC> graw[NOH][NOW];
            int32_t pick[NOH][NOW][VEC];
#pragma unroll
            for (int a = 0; a < NOH; ++a)
#pragma unroll
                for (int b = 0; b < NOW; ++b) {
                    // windows beyond the range are read at a clamped (valid) pixel and not used
                    const uint32_t opix = obase + (uint32_t)(min(oh_lo + a, k.Ho - 1) * k.Wo + min(ow_lo + b, k.Wo - 1));
                    const uint32_t o = opix * (uint32_t)k.C + (uint32_t)c0;
                    graw[a][b] = load_raw<DT, VEC>(k.g_out, audited(k, 1, 20, o + opix * k.gout_extra, VEC));
                    if (is_max) load_picks<VEC>(k.idx, o, pick[a][b]);
                }
#pragma unroll
            for (int a = 0; a < NOH; ++a)
#pragma unroll
                for (int b = 0; b < NOW; ++b) {
                    const int32_t oh = oh_lo + a, ow = ow_lo + b;
                    const bool in = oh <= oh_hi && ow <= ow_hi;
                    float g[VEC];
                    unpack<DT, VEC>(graw[a][b], g);
                    if (is_max) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) s[e] += (in && pick[a][b][e] == cell) ? g[e] : 0.0f;
                    } else {
                        const float inv = in ? bwd_avg_inv(p, k.H, k.W, min(oh, k.Ho - 1), min(ow, k.Wo - 1)) : 0.0f;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) s[e] += g[e] * inv;
                    }
                }
        } else
        for (int32_t oh = oh_lo; oh <= oh_hi; ++oh)
            for (int32_t ow = ow_lo; ow <= ow_hi; ++ow) {
                // 0 <= oh < Ho, 0 <= ow < Wo: an output pixel; its VEC channels c0 .. c0 + VEC - 1
                const uint32_t opix = obase + (uint32_t)(oh * k.Wo + ow);
                const uint32_t o = opix * (uint32_t)k.C + (uint32_t)c0;
                float g[VEC];
                unpack<DT, VEC>(load_raw<DT, VEC>(k.g_out, audited(k, 1, 21, o + opix * k.gout_extra, VEC)), g);
                if (is_max) {
                    int32_t pick[VEC];
                    load_picks<VEC>(k.idx, o, pick);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) s[e] += pick[e] == cell ? g[e] : 0.0f;
                } else {
                    const float inv = bwd_avg_inv(p, k.H, k.W, oh, ow);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) s[e] += g[e] * inv;
                }
            }
    }
    if (live) store_row<DT, VEC, 1, NR>(k, 0, off, pix * k.gin_extra, adds, s, t, r);
}

// Disjoint 2 x 2 windows that tile the plane, channels-last: a lane owns VEC channels of one
// window's four pixels (row-major window order: the order of the first-maximum rule).
template <int DT, int VEC, int NR>
__global__ __launch_bounds__(256) void bwd_direct2_nhwc_kernel(const BwdK k)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t opix = fdiv(i, k.div_wv);           // (n * Ho + oh) * Wo + ow
    const uint32_t cv = i - opix * k.div_wv.d;
    const uint32_t orow = fdiv(opix, k.div_w);         // n * Ho + oh   (div_w divides by Wo here)
    const uint32_t ow = opix - orow * (uint32_t)k.Wo;
    const uint32_t n = fdiv(orow, k.div_h);            // div_h divides by Ho here
    const uint32_t oh = orow - n * (uint32_t)k.Ho;
    const int32_t c0 = (int32_t)(cv * VEC);
    // input pixels (2 oh + dh, 2 ow + dw): H = 2 Ho, W = 2 Wo
    const uint32_t p00 = (n * (uint32_t)k.H + 2 * oh) * (uint32_t)k.W + 2 * ow;
    const uint32_t offs[4] = {p00 * (uint32_t)k.C + (uint32_t)c0, (p00 + 1) * (uint32_t)k.C + (uint32_t)c0,
                              (p00 + (uint32_t)k.W) * (uint32_t)k.C + (uint32_t)c0,
                              (p00 + (uint32_t)k.W + 1) * (uint32_t)k.C + (uint32_t)c0};
    const uint32_t out_off = opix * (uint32_t)k.C + (uint32_t)c0;

    const uint32_t pixels[4] = {p00, p00 + 1, p00 + (uint32_t)k.W, p00 + (uint32_t)k.W + 1};
    Raw<DT, VEC> raw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) raw[j] = load_raw<DT, VEC, true>(k.a, audited(k, 0, 7, offs[j] + pixels[j] * k.a_extra, VEC));
    const Raw<DT, VEC> gr = load_raw<DT, VEC, true>(k.g_out, audited(k, 1, 22, out_off + opix * k.gout_extra, VEC));
    float x[4][VEC], t[4][VEC], r[NR ? NR : 1][4][VEC], g[VEC];
#pragma unroll
    for (int j = 0; j < 4; ++j) unpack<DT, VEC>(raw[j], x[j]);
    unpack<DT, VEC>(gr, g);
    const int32_t cs[4] = {c0, c0, c0, c0};
    const int32_t adds = ew_sweep<DT, VEC, 4, true, NR>(k, cs, offs, x, t, r);

    float s[4][VEC];
    if (k.pool.kind == OP_MAXPOOL) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float best = -INFINITY;
            int pick = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool more = x[j][e] > best;
                best = more ? x[j][e] : best;
                pick = more ? j : pick;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j][e] = pick == j ? g[e] : 0.0f;
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float gi = g[e] * k.pool.inv_kk;
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j][e] = gi;
        }
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) store_row<DT, VEC, 4, NR>(k, j, offs[j], pixels[j] * k.gin_extra, adds, s[j], t, r);
}

static void set_error(hipError_t e) { set_hip_error((int32_t)e); }

constexpr int K_BWD_EW_U = 1;  // vectors per lane in bwd_ew_kernel (2 measured no faster in float32 and 70 % slower with 16-bit storage: registers)

// The instance compiled for the stage's window, or the one that reads it from the argument block.
template <int DT, int VEC>
static void launch_stage(const BwdK &k, dim3 g, dim3 b, hipStream_t st)
{
    const PoolK &p = k.pool;
    bool has_add = false;
    for (int32_t j = 0; j < k.n_ew; ++j) has_add = has_add || k.ew[j].kind == OP_ADD;
    // the compiled-in instances assume whole vectors per row and VEC a multiple of the stride
    const bool w33p1 = p.kind != 0 && p.kh == 3 && p.kw == 3 && p.ph == 1 && p.pw == 1 && VEC > 1;
    if (w33p1 && p.sh == 2 && p.sw == 2 && 2 * k.Wo == k.W) {
        if (has_add) bwd_stage_kernel<DT, VEC, 3, 3, 2, 2, 1><<<g, b, 0, st>>>(k);
        else bwd_stage_kernel<DT, VEC, 3, 3, 2, 2, 1, 0><<<g, b, 0, st>>>(k);
    } else if (w33p1 && p.sh == 1 && p.sw == 1 && k.Wo == k.W) {
        if (has_add) bwd_stage_kernel<DT, VEC, 3, 3, 1, 1, 1><<<g, b, 0, st>>>(k);
        else bwd_stage_kernel<DT, VEC, 3, 3, 1, 1, 1, 0><<<g, b, 0, st>>>(k);
    }
    else bwd_stage_kernel<DT, VEC, 0, 0, 0, 0, 0><<<g, b, 0, st>>>(k);
}

bs_status launch_backward_stage(const BwdK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t full = dtype == BS_F32 ? 4 : 8;
    // the launch must cover exactly the lanes the argument block describes
    if (grid < 1 || grid > 0x7fffffffll || threads != 256) return BS_ERR_UNSUPPORTED;
    if (k.n_ew < 0 || k.n_ew > K_BWD_EW) return BS_ERR_UNSUPPORTED;
    const dim3 g((uint32_t)grid), b((uint32_t)threads);
    // a stage without Add gets the instances that keep no residual gradients in registers
    int32_t n_add = 0;
    for (int32_t j = 0; j < k.n_ew; ++j) n_add += k.ew[j].kind == OP_ADD;
    if (k.nhwc) {
        // a lane per (pixel or window, channel vector): the divisors must be the ones the kernels assume
        if ((vec != 1 && vec != full) || k.C % vec != 0 || (int64_t)k.div_wv.d * vec != k.C ||
            (int64_t)k.div_h.d != (k.direct ? k.Ho : k.H) || (int64_t)k.div_w.d != (k.direct ? k.Wo : k.W) ||
            (int64_t)grid * threads < (int64_t)k.total)
            return BS_ERR_UNSUPPORTED;
        const PoolK &p = k.pool;
        if (k.direct && ((p.kind != OP_MAXPOOL && p.kind != OP_AVGSUM) || p.kh != 2 || p.kw != 2 || p.sh != 2 || p.sw != 2 ||
                         p.ph != 0 || p.pw != 0 || k.H != 2 * k.Ho || k.W != 2 * k.Wo))
            return BS_ERR_UNSUPPORTED;
        if (k.direct && n_add > 1) return BS_ERR_UNSUPPORTED;  // planned for the gathering kernel instead
        if (!k.direct && p.kind == OP_MAXPOOL && !k.idx) return BS_ERR_NULL;
        // windows over one pixel: at most ceil(kh / sh) x ceil(kw / sw); 2 x 2 and 3 x 3 are compiled in
        const int32_t noh = p.kind != 0 ? (p.kh + p.sh - 1) / p.sh : 0, now = p.kind != 0 ? (p.kw + p.sw - 1) / p.sw : 0;
#define BS_LAUNCH_NHWC(DT, V)                                                          \
    do {                                                                               \
        if (k.direct && n_add == 0) bwd_direct2_nhwc_kernel<DT, V, 0><<<g, b, 0, st>>>(k); \
        else if (k.direct) bwd_direct2_nhwc_kernel<DT, V, 1><<<g, b, 0, st>>>(k); \
        else if (noh == 2 && now == 2 && n_add == 0) bwd_stage_nhwc_kernel<DT, V, 2, 2, 0><<<g, b, 0, st>>>(k); \
        else if (noh == 2 && now == 2) bwd_stage_nhwc_kernel<DT, V, 2, 2><<<g, b, 0, st>>>(k); \
        else if (noh == 3 && now == 3 && n_add == 0) bwd_stage_nhwc_kernel<DT, V, 3, 3, 0><<<g, b, 0, st>>>(k); \
        else if (noh == 3 && now == 3) bwd_stage_nhwc_kernel<DT, V, 3, 3><<<g, b, 0, st>>>(k); \
        else if (n_add == 0) bwd_stage_nhwc_kernel<DT, V, 0, 0, 0><<<g, b, 0, st>>>(k); \
        else if (n_add == 1) bwd_stage_nhwc_kernel<DT, V, 0, 0, 1><<<g, b, 0, st>>>(k); \
        else bwd_stage_nhwc_kernel<DT, V, 0, 0><<<g, b, 0, st>>>(k);                   \
    } while (0)
        if (dtype == BS_F32) { if (vec == 4) BS_LAUNCH_NHWC(DT_F32, 4); else BS_LAUNCH_NHWC(DT_F32, 1); }
        else if (dtype == BS_BF16) { if (vec == 8) BS_LAUNCH_NHWC(DT_BF16, 8); else BS_LAUNCH_NHWC(DT_BF16, 1); }
        else if (dtype == BS_F16) { if (vec == 8) BS_LAUNCH_NHWC(DT_F16, 8); else BS_LAUNCH_NHWC(DT_F16, 1); }
        else return BS_ERR_UNSUPPORTED;
#undef BS_LAUNCH_NHWC
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error(e);
            return BS_ERR_HIP;
        }
        return BS_OK;
    }
    if (k.flat && (k.a_extra || k.gin_extra || k.gout_extra) && ((int64_t)k.C * k.H * k.W) % vec != 0)
        return BS_ERR_UNSUPPORTED;  // a vector would run from one image of a slice into the next
    if (k.flat) {
        // vectors that run over plane boundaries: no pooling, whole vectors, a plane of at least one vector
        if (k.pool.kind != 0 || vec != full || (int64_t)k.div_w.d != (int64_t)k.H * k.W || (int64_t)k.H * k.W < vec ||
            (int64_t)k.div_c.d != k.C || (int64_t)grid * threads < (int64_t)k.total)
            return BS_ERR_UNSUPPORTED;
    } else if ((vec != 1 && vec != full && !(dtype != BS_F32 && vec == 4)) || k.W % vec != 0 || (int64_t)k.div_wv.d * vec != k.W ||
               (int64_t)k.div_h.d != (k.direct ? k.Ho : k.H) || (int64_t)k.div_c.d != k.C ||
               (int64_t)grid * threads < (int64_t)k.total) {
        return BS_ERR_UNSUPPORTED;
    }
    if (k.wave_rows == 2) {
        // what the two-level kernel assumes: average 3 x 3 / 1 / 1 that keeps the plane's size, then max 3 x 3 / 2 / 1;
        // no Add anywhere; 4 cells per lane; a row's column blocks in one wave; chunks that cover the plane
        const PoolK &p = k.pool, &q = k.pool2;
        for (int32_t j = 0; j < k.n_ew + k.n_post; ++j)
            if (j >= K_BWD_EW || k.ew[j].kind == OP_ADD) return BS_ERR_UNSUPPORTED;
        if (k.n_post < 0 || k.n_ew + k.n_post > K_BWD_EW) return BS_ERR_UNSUPPORTED;
        if (k.direct || p.kind != OP_AVGSUM || p.kh != 3 || p.kw != 3 || p.ph != 1 || p.pw != 1 || p.sh != 1 || p.sw != 1 ||
            q.kind != OP_MAXPOOL || q.kh != 3 || q.kw != 3 || q.ph != 1 || q.pw != 1 || q.sh != 2 || q.sw != 2 || vec != 4 ||
            k.W % 4 != 0 || k.cbs != k.W / 4 || k.cbs < 1 || k.cbs > 64 || k.spw != 64 / k.cbs || k.Wo * 2 != k.W ||
            k.Ho != (k.H + 2 - 3) / 2 + 1 || k.rc < 1 || k.chunks < 1 || (int64_t)(k.chunks - 1) * k.rc * 2 >= k.H ||
            (int64_t)k.div_cbs.d != k.cbs || (int64_t)k.div_chunks.d != k.chunks || (int64_t)k.div_c.d != k.C ||
            (uint64_t)grid * 4 * k.spw < k.units)
            return BS_ERR_UNSUPPORTED;
        // lists whose kinds are compiled in (BatchNorm, ReLU on both sides); any other goes through the run-time loops
        auto code = [&](int32_t first, int32_t n) {
            int32_t c = 0, digit = 1;
            if (n > 6) return -1;
            for (int32_t j = 0; j < n; ++j, digit *= K_EW_BASE) c += k.ew[first + j].kind * digit;
            return c;
        };
        constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE;
        const bool compiled = code(0, k.n_ew) == BN_RELU && code(k.n_ew, k.n_post) == BN_RELU;
#define BS_LAUNCH_ROWS2(DT)                                                                     \
    do {                                                                                        \
        if (compiled) bwd_rows2_kernel<DT, 4, BN_RELU, BN_RELU><<<g, b, 0, st>>>(k);            \
        else bwd_rows2_kernel<DT, 4, -1, -1><<<g, b, 0, st>>>(k);                               \
    } while (0)
        if (dtype == BS_F32) BS_LAUNCH_ROWS2(DT_F32);
        else if (dtype == BS_BF16) BS_LAUNCH_ROWS2(DT_BF16);
        else if (dtype == BS_F16) BS_LAUNCH_ROWS2(DT_F16);
        else return BS_ERR_UNSUPPORTED;
#undef BS_LAUNCH_ROWS2
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error(e);
            return BS_ERR_HIP;
        }
        return BS_OK;
    }
    if (k.wave_rows) {
        const PoolK &p = k.pool;
        // what the kernel assumes: 3 x 3 max windows, padding 1, stride 1 or 2 that divides the row exactly;
        // a row's column blocks in one wave; chunks that cover the plane
        for (int32_t j = k.n_ew; j < k.n_ew + k.n_post; ++j)
            if (k.ew[j].kind == OP_ADD) return BS_ERR_UNSUPPORTED;
        if (k.n_post < 0 || k.n_ew + k.n_post > K_BWD_EW) return BS_ERR_UNSUPPORTED;
        const bool is_max = p.kind == OP_MAXPOOL;
        if (!is_max && k.n_post != 0) return BS_ERR_UNSUPPORTED;
        if (k.direct || (p.kind != OP_MAXPOOL && p.kind != OP_AVGSUM) || p.kh != 3 || p.kw != 3 || p.ph != 1 || p.pw != 1 || p.sh != p.sw ||
            (p.sh != 1 && p.sh != 2) || vec != full || k.W % vec != 0 || k.cbs != k.W / vec || k.cbs < 1 || k.cbs > 64 ||
            k.spw != 64 / k.cbs || k.Wo * p.sw != k.W || k.Ho != (k.H + 2 - 3) / p.sh + 1 || k.rc < 1 || k.chunks < 1 ||
            (int64_t)(k.chunks - 1) * k.rc * p.sh >= k.H || (int64_t)k.div_cbs.d != k.cbs || (int64_t)k.div_chunks.d != k.chunks ||
            (int64_t)k.div_c.d != k.C || (uint64_t)grid * 4 * k.spw < k.units)
            return BS_ERR_UNSUPPORTED;
        // BatchNorm, ReLU in front of a max pooling with stride 2 (the ResNet stem): the kinds of the list compiled in
        constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE;
        const bool bn_relu = k.n_ew == 2 && k.ew[0].kind == OP_BN && k.ew[1].kind == OP_RELU;
#define BS_LAUNCH_MAXROWS(DT, V)                                                               \
    do {                                                                                       \
        if (is_max && p.sh == 2 && bn_relu && k.n_post == 0) bwd_rows_kernel<DT, V, 2, 0, true, BN_RELU><<<g, b, 0, st>>>(k); \
        else if (is_max && p.sh == 2 && n_add == 0) bwd_rows_kernel<DT, V, 2, 0, true><<<g, b, 0, st>>>(k);     \
        else if (is_max && p.sh == 2) bwd_rows_kernel<DT, V, 2, K_MAX_RES, true><<<g, b, 0, st>>>(k);           \
        else if (is_max && n_add == 0) bwd_rows_kernel<DT, V, 1, 0, true><<<g, b, 0, st>>>(k);                  \
        else if (is_max) bwd_rows_kernel<DT, V, 1, K_MAX_RES, true><<<g, b, 0, st>>>(k);                        \
        else if (p.sh == 2 && n_add == 0) bwd_rows_kernel<DT, V, 2, 0, false><<<g, b, 0, st>>>(k);              \
        else if (p.sh == 2) bwd_rows_kernel<DT, V, 2, K_MAX_RES, false><<<g, b, 0, st>>>(k);                    \
        else if (n_add == 0) bwd_rows_kernel<DT, V, 1, 0, false><<<g, b, 0, st>>>(k);                           \
        else bwd_rows_kernel<DT, V, 1, K_MAX_RES, false><<<g, b, 0, st>>>(k);                                   \
    } while (0)
        if (dtype == BS_F32) BS_LAUNCH_MAXROWS(DT_F32, 4);
        else if (dtype == BS_BF16) BS_LAUNCH_MAXROWS(DT_BF16, 8);
        else if (dtype == BS_F16) BS_LAUNCH_MAXROWS(DT_F16, 8);
        else return BS_ERR_UNSUPPORTED;
#undef BS_LAUNCH_MAXROWS
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error(e);
            return BS_ERR_HIP;
        }
        return BS_OK;
    }
    if (k.direct) {
        const PoolK &p = k.pool;
        // what the kernel assumes: 2 x 2 windows, stride 2, no padding, tiling the plane; whole vectors
        if ((p.kind != OP_MAXPOOL && p.kind != OP_AVGSUM) || p.kh != 2 || p.kw != 2 || p.sh != 2 || p.sw != 2 || p.ph != 0 ||
            p.pw != 0 || k.H != 2 * k.Ho || k.W != 2 * k.Wo || vec < 2)
            return BS_ERR_UNSUPPORTED;
        // BatchNorm, ReLU in front of the pooling (the VGG stacks, the DenseNet transition): the kinds of the list compiled in
        const bool bn_relu2 = k.n_ew == 2 && k.ew[0].kind == OP_BN && k.ew[1].kind == OP_RELU;
#define BS_LAUNCH_DIRECT(DT, V)                                                                \
    do {                                                                                       \
        if (n_add == 0 && bn_relu2) bwd_direct2_kernel<DT, V, 0, OP_BN + OP_RELU * K_EW_BASE><<<g, b, 0, st>>>(k); \
        else if (n_add == 0) bwd_direct2_kernel<DT, V, 0><<<g, b, 0, st>>>(k);                 \
        else if (n_add == 1) bwd_direct2_kernel<DT, V, 1><<<g, b, 0, st>>>(k);                 \
        else bwd_direct2_kernel<DT, V, K_MAX_RES><<<g, b, 0, st>>>(k);                         \
    } while (0)
        if (dtype == BS_F32) BS_LAUNCH_DIRECT(DT_F32, 4);
        else if (dtype == BS_BF16) { if (vec == 8) BS_LAUNCH_DIRECT(DT_BF16, 8); else BS_LAUNCH_DIRECT(DT_BF16, 4); }
        else if (dtype == BS_F16) { if (vec == 8) BS_LAUNCH_DIRECT(DT_F16, 8); else BS_LAUNCH_DIRECT(DT_F16, 4); }
        else return BS_ERR_UNSUPPORTED;
#undef BS_LAUNCH_DIRECT
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error(e);
            return BS_ERR_HIP;
        }
        return BS_OK;
    }
    if (k.pool.kind == OP_MAXPOOL && !k.idx) return BS_ERR_NULL;
    if (k.pool.kind == 0 && vec == full) {
        // no pooling, whole vectors: K_BWD_EW_U vectors per lane (the grid was sized for one per lane)
        const dim3 gu((uint32_t)((grid + K_BWD_EW_U - 1) / K_BWD_EW_U));
        // instances that keep 0, 1 or K_MAX_RES residual gradients in registers, by the stage's Adds
        // the lists of the common networks with their kinds compiled in: BatchNorm, ReLU (a DenseNet layer) and
        // BatchNorm, Add, ReLU (the tail of a residual block; 16-bit storage only: measured on MI355X 3.5 % faster there, 1 %
        // slower in float32, where the kernel waits for memory either way)
        constexpr int C_BN_RELU = OP_BN + OP_RELU * K_EW_BASE, C_BN_ADD_RELU = OP_BN + OP_ADD * K_EW_BASE + OP_RELU * K_EW_BASE * K_EW_BASE;
        int32_t ew_code = 0;
        for (int32_t j = 0, digit = 1; j < k.n_ew; ++j, digit *= K_EW_BASE) ew_code = j < 6 ? ew_code + k.ew[j].kind * digit : -1;
#define BS_LAUNCH_EW(DT, V)                                                                        \
    do {                                                                                           \
        if (ew_code == C_BN_RELU) bwd_ew_kernel<DT, V, K_BWD_EW_U, 0, C_BN_RELU><<<gu, b, 0, st>>>(k); \
        else if (ew_code == C_BN_ADD_RELU && DT != DT_F32) bwd_ew_kernel<DT, V, K_BWD_EW_U, 1, C_BN_ADD_RELU><<<gu, b, 0, st>>>(k); \
        else if (n_add == 0) bwd_ew_kernel<DT, V, K_BWD_EW_U, 0><<<gu, b, 0, st>>>(k);             \
        else if (n_add == 1) bwd_ew_kernel<DT, V, K_BWD_EW_U, 1><<<gu, b, 0, st>>>(k);             \
        else bwd_ew_kernel<DT, V, K_BWD_EW_U, K_MAX_RES><<<gu, b, 0, st>>>(k);                     \
    } while (0)
        if (dtype == BS_F32) BS_LAUNCH_EW(DT_F32, 4);
        else if (dtype == BS_BF16) BS_LAUNCH_EW(DT_BF16, 8);
        else if (dtype == BS_F16) BS_LAUNCH_EW(DT_F16, 8);
        else return BS_ERR_UNSUPPORTED;
#undef BS_LAUNCH_EW
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error(e);
            return BS_ERR_HIP;
        }
        return BS_OK;
    }
    if (dtype == BS_F32) {
        if (vec == 4) launch_stage<DT_F32, 4>(k, g, b, st);
        else launch_stage<DT_F32, 1>(k, g, b, st);
    } else if (dtype == BS_BF16) {
        if (vec == 8) launch_stage<DT_BF16, 8>(k, g, b, st);
        else if (vec == 4) launch_stage<DT_BF16, 4>(k, g, b, st);
        else launch_stage<DT_BF16, 1>(k, g, b, st);
    } else if (dtype == BS_F16) {
        if (vec == 8) launch_stage<DT_F16, 8>(k, g, b, st);
        else if (vec == 4) launch_stage<DT_F16, 4>(k, g, b, st);
        else launch_stage<DT_F16, 1>(k, g, b, st);
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
