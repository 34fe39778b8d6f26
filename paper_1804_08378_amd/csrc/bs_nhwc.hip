// Channels-last (NHWC) kernels.  The tensor is N x H x W x C in memory: the channels of one
// pixel are contiguous, so a lane takes one 128-bit vector of VEC consecutive channels of one
// pixel and consecutive lanes take consecutive vectors: every access of a wave is one
// contiguous run, for element-wise layers and for pooling windows alike (a window cell is a
// pixel, i.e. the same channel vector W * C elements or C elements further on).  BatchNorm
// parameters are per-lane vectors here (one 128-bit load of scale and of shift per lane).
//
//   nhwc_stream_kernel  element-wise only sequence, U vectors per lane.
//   nhwc_pool_kernel    [element-wise]* pool [element-wise]* for the common windows (2x2/2,
//                       3x3/2, 3x3/1): a lane produces VEC channels of a small block of
//                       neighbouring output pixels, so cells shared by overlapping windows are
//                       loaded, and taken through the element-wise operations, once per block.
//   nhwc_pool_any_kernel  the same for any window, one output pixel per lane.
//
// The arithmetic and its order are those of the NCHW kernels (float32, BatchNorm one fused
// multiply-add, window cells visited row-major, first maximum wins, the average's sum taken
// over the in-range cells from +0 and multiplied by a float32 reciprocal, every layer's
// output rounded to the storage type), so the results are the same numbers in another
// memory order.  Index outputs hold ih * W + iw like the NCHW ones and are laid out like
// the output tensor.
#include "bs_nhwc_device.h"
#include <algorithm>

#include "bs_internal.h"

namespace bs {

// Element-wise only.  A work-group takes nthr * U consecutive vectors; lane t handles vectors
// t, t + nthr, ...  CODE: the kinds of the list's operations as a compile-time code (apply_ew_nhwc), or -1.
template <int DT, int VEC, int U, int CODE = -1>
__global__ __launch_bounds__(512) void nhwc_stream_kernel(const NhwcK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t cvn = k.div_cv.d;
    if (nthr % cvn == 0) {
        // the lane's U vectors lie a multiple of the channel count apart: the same channels, one
        // set of BatchNorm parameters for all of them
        const uint32_t c0 = (base - fdiv(base, k.div_cv) * cvn) * VEC;
        bool valid[U];
        uint32_t off[U], pixel[U];
        Raw<DT, VEC> raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = base + u * nthr;
            valid[u] = i < k.total;
            i = valid[u] ? i : base % cvn;  // a vector of the same channels at the start of the tensor
            off[u] = i * VEC;
            pixel[u] = fdiv(i, k.div_cv);
            raw[u] = load_raw<DT, VEC, true>(k.in, off[u] + pixel[u] * k.in_xp);
        }
        float x[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) unpack<DT, VEC>(raw[u], x[u]);
        apply_ew_nhwc<DT, VEC, U, CODE>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (valid[u]) store_elems<DT, VEC>(k.out, off[u] + pixel[u] * k.out_xp, x[u]);
        return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        const bool valid = i < k.total;
        i = valid ? i : 0u;
        const uint32_t off1[1] = {i * VEC};
        const uint32_t pixel = fdiv(i, k.div_cv);
        const uint32_t c0 = (i - pixel * cvn) * VEC;
        float x[1][VEC];
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.in, off1[0] + pixel * k.in_xp), x[0]);
        apply_ew_nhwc<DT, VEC, 1, CODE>(x, c0, off1, k.pre, k.n_pre, k.params, k.C, k.res);
        if (valid) store_elems<DT, VEC>(k.out, off1[0] + pixel * k.out_xp, x[0]);
    }
}

// What a lane adds to its running maximum / sum for one window cell.
template <int VEC, bool IDX>
BS_DEV void take_cell(bool is_max, const float (&v)[VEC], int32_t cell_index, float (&acc)[VEC], int32_t (&bi)[VEC])
{
    if (is_max) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if constexpr (IDX) {
                const bool g = v[e] > acc[e];
                acc[e] = g ? v[e] : acc[e];
                bi[e] = g ? cell_index : bi[e];
            } else {
                acc[e] = __builtin_fmaxf(acc[e], v[e]);  // the same value as the first maximum
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = acc[e] + v[e];
    }
}

// One pooling operation with a compile-time window KH x KW and strides SH x SW.  A lane
// produces VEC channels of a block of OHB x OWB neighbouring output pixels: the
// ((OHB-1)*SH + KH) x ((OWB-1)*SW + KW) input cells under the block are requested at once,
// the element-wise operations before the pool run once per cell (not once per window that
// holds it), then every output of the block takes its window from the registers.
// IDX: keep the argmax (only when an index output was asked for).
// PRE, POST: the kinds of the lists in front of and behind the pooling as compile-time codes (apply_ew_nhwc), or -1.
template <int DT, int VEC, int KH, int KW, int SH, int SW, int OHB, int OWB, bool IDX, int PRE = -1, int POST = -1>
__global__ __launch_bounds__(256) void nhwc_pool_kernel(const NhwcK k)
{
    constexpr int CR = (OHB - 1) * SH + KH, CC = (OWB - 1) * SW + KW, NCELL = CR * CC, NOUT = OHB * OWB;
    constexpr bool OVERLAP = KH > SH || KW > SW;
    uint32_t i = (OVERLAP ? xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x) * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    // lane -> (image n, block row, block column, channel vector cv), cv fastest
    const uint32_t blk = fdiv(i, k.div_cv);
    const uint32_t c0 = (i - blk * k.div_cv.d) * VEC;
    const uint32_t t = fdiv(blk, k.div_wo);
    const int32_t ow0 = (int32_t)(blk - t * k.div_wo.d) * OWB;
    const uint32_t n = fdiv(t, k.div_ho);
    const int32_t oh0 = (int32_t)(t - n * k.div_ho.d) * OHB;
    const PoolK &p = k.pool;
    const int32_t hb = oh0 * SH - p.ph, wb = ow0 * SW - p.pw;  // plane position of cell (0, 0)
    const uint32_t img = n * (uint32_t)(k.H * k.W);            // first pixel of the image
    const bool is_max = p.kind == OP_MAXPOOL;
    const bool interior = hb >= 0 && hb + CR <= k.H && wb >= 0 && wb + CC <= k.W;

    // One output per lane and many cell registers (3 x 3 windows of 8-channel vectors): the cells are
    // still requested at once, but unpacked, run through the element-wise list and folded into the
    // window one window row at a time -- 24 live values instead of 72, twice the waves per SIMD.
    constexpr bool ROWWISE = NOUT == 1 && NCELL * VEC >= 64;
    if constexpr (ROWWISE) {
        Raw<DT, VEC> raw[NCELL];
        uint32_t off[NCELL];
#pragma unroll
        for (int r = 0; r < CR; ++r)
#pragma unroll
            for (int c = 0; c < CC; ++c) {
                const int32_t ih = min(max(hb + r, 0), k.H - 1), iw = min(max(wb + c, 0), k.W - 1);
                const uint32_t pixel = img + (uint32_t)(ih * k.W + iw);
                off[r * CC + c] = pixel * (uint32_t)k.C + c0;
                raw[r * CC + c] = load_raw<DT, VEC>(k.in, off[r * CC + c] + pixel * k.in_xp);
            }
        const bool oin = oh0 < k.Ho && ow0 < k.Wo;
        const uint32_t opix = (n * (uint32_t)k.Ho + (uint32_t)min(oh0, k.Ho - 1)) * (uint32_t)k.Wo + (uint32_t)min(ow0, k.Wo - 1);
        const uint32_t ooff[1] = {opix * (uint32_t)k.C + c0};
        const int32_t hlo = max(hb, 0), hhi = min(hb + KH, k.H), wlo = max(wb, 0), whi = min(wb + KW, k.W);
        float acc[VEC];
        int32_t bi[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            acc[e] = is_max ? -INFINITY : 0.0f;
            bi[e] = hlo * k.W + wlo;  // first in-range cell
        }
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) {
            float xr[KW][VEC];
            uint32_t offr[KW];
#pragma unroll
            for (int dw = 0; dw < KW; ++dw) {
                unpack<DT, VEC>(raw[dh * CC + dw], xr[dw]);
                offr[dw] = off[dh * CC + dw];
            }
            apply_ew_nhwc<DT, VEC, KW, PRE>(xr, c0, offr, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
            for (int dw = 0; dw < KW; ++dw)
                if (interior || (hb + dh >= hlo && hb + dh < hhi && wb + dw >= wlo && wb + dw < whi))
                    take_cell<VEC, IDX>(is_max, xr[dw], (hb + dh) * k.W + wb + dw, acc, bi);
        }
        float y[1][VEC];
        if (is_max) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) y[0][e] = acc[e];
        } else {
            const float inv = avg_inv(p, KH, KW, k.H, k.W, hb, wb, hlo, hhi, wlo, whi);
#pragma unroll
            for (int e = 0; e < VEC; ++e) y[0][e] = round_store<DT>(acc[e] * inv);
        }
        apply_ew_nhwc<DT, VEC, 1, POST>(y, c0, ooff, k.post, k.n_post, k.params, k.C, k.res);
        if (live && oin) {
            store_elems<DT, VEC>(k.out, ooff[0] + opix * k.out_xp, y[0]);
            if constexpr (IDX) {
                if (is_max) store_indices<VEC>(k.idx + ooff[0], bi);
            }
        }
        return;
    }

    float x[NCELL][VEC];
    uint32_t off[NCELL];
    {
        Raw<DT, VEC> raw[NCELL];
#pragma unroll
        for (int r = 0; r < CR; ++r)
#pragma unroll
            for (int c = 0; c < CC; ++c) {
                // a cell outside the plane is padding: requested from the nearest cell inside
                // (a safe address) and never used
                const int32_t ih = min(max(hb + r, 0), k.H - 1), iw = min(max(wb + c, 0), k.W - 1);
                const uint32_t pixel = img + (uint32_t)(ih * k.W + iw);
                off[r * CC + c] = pixel * (uint32_t)k.C + c0;
                raw[r * CC + c] = load_raw<DT, VEC>(k.in, off[r * CC + c] + pixel * k.in_xp);
            }
#pragma unroll
        for (int cell = 0; cell < NCELL; ++cell) unpack<DT, VEC>(raw[cell], x[cell]);
    }
    apply_ew_nhwc<DT, VEC, NCELL, PRE>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);

    float y[NOUT][VEC];
    int32_t yi[NOUT][VEC];
    uint32_t ooff[NOUT], opix[NOUT];
    bool oin[NOUT];
#pragma unroll
    for (int a = 0; a < OHB; ++a)
#pragma unroll
        for (int b = 0; b < OWB; ++b) {
            const int o = a * OWB + b;
            const int32_t oh = oh0 + a, ow = ow0 + b;
            oin[o] = oh < k.Ho && ow < k.Wo;
            // outputs beyond the plane's edge (ragged blocks) are computed at a safe address and dropped
            opix[o] = (n * (uint32_t)k.Ho + (uint32_t)min(oh, k.Ho - 1)) * (uint32_t)k.Wo + (uint32_t)min(ow, k.Wo - 1);
            ooff[o] = opix[o] * (uint32_t)k.C + c0;
            const int32_t h0 = hb + a * SH, w0 = wb + b * SW;
            const int32_t hlo = max(h0, 0), hhi = min(h0 + KH, k.H), wlo = max(w0, 0), whi = min(w0 + KW, k.W);
            float acc[VEC];
            int32_t bi[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                acc[e] = is_max ? -INFINITY : 0.0f;
                bi[e] = hlo * k.W + wlo;  // first in-range cell
            }
            if (interior) {
#pragma unroll
                for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw)
                        take_cell<VEC, IDX>(is_max, x[(a * SH + dh) * CC + b * SW + dw], (h0 + dh) * k.W + w0 + dw, acc, bi);
            } else {
#pragma unroll
                for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw)
                        if (h0 + dh >= hlo && h0 + dh < hhi && w0 + dw >= wlo && w0 + dw < whi)
                            take_cell<VEC, IDX>(is_max, x[(a * SH + dh) * CC + b * SW + dw], (h0 + dh) * k.W + w0 + dw, acc, bi);
            }
            if (is_max) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[o][e] = acc[e];
            } else {
                const float inv = avg_inv(p, KH, KW, k.H, k.W, h0, w0, hlo, hhi, wlo, whi);
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[o][e] = round_store<DT>(acc[e] * inv);
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) yi[o][e] = bi[e];
        }
    apply_ew_nhwc<DT, VEC, NOUT, POST>(y, c0, ooff, k.post, k.n_post, k.params, k.C, k.res);
#pragma unroll
    for (int o = 0; o < NOUT; ++o)
        if (live && oin[o]) {
            store_elems<DT, VEC>(k.out, ooff[o] + opix[o] * k.out_xp, y[o]);
            if constexpr (IDX) {
                if (is_max) store_indices<VEC>(k.idx + ooff[o], yi[o]);
            }
        }
}

// Any window: one output pixel per lane, a few cells of a window row at a time.
template <int DT, int VEC>
__global__ __launch_bounds__(256) void nhwc_pool_any_kernel(const NhwcK k)
{
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = i < k.total;
    i = live ? i : 0u;
    const uint32_t pix = fdiv(i, k.div_cv);
    const uint32_t c0 = (i - pix * k.div_cv.d) * VEC;
    const uint32_t t = fdiv(pix, k.div_wo);
    const int32_t ow = (int32_t)(pix - t * (uint32_t)k.Wo);
    const uint32_t n = fdiv(t, k.div_ho);
    const int32_t oh = (int32_t)(t - n * (uint32_t)k.Ho);
    const PoolK &p = k.pool;
    const int32_t h0 = oh * p.sh - p.ph, w0 = ow * p.sw - p.pw;
    // in-range part of the window; never empty (the padding is at most half the window)
    const int32_t hlo = max(h0, 0), hhi = min(h0 + p.kh, k.H), wlo = max(w0, 0), whi = min(w0 + p.kw, k.W);
    const uint32_t img = n * (uint32_t)(k.H * k.W);
    const bool is_max = p.kind == OP_MAXPOOL;
    float acc[VEC];
    int32_t bi[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        acc[e] = is_max ? -INFINITY : 0.0f;
        bi[e] = hlo * k.W + wlo;
    }
    // row by row, U cells of a row requested at once (cells past the row's end repeat its last
    // cell and are not taken), taken in row-major order
    constexpr int U = VEC >= 8 ? 4 : 8;
    for (int32_t ih = hlo; ih < hhi; ++ih)
        for (int32_t iw0 = wlo; iw0 < whi; iw0 += U) {
            uint32_t off[U];
            Raw<DT, VEC> raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t pixel = img + (uint32_t)(ih * k.W + min(iw0 + u, whi - 1));
                off[u] = pixel * (uint32_t)k.C + c0;
                raw[u] = load_raw<DT, VEC>(k.in, off[u] + pixel * k.in_xp);
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) unpack<DT, VEC>(raw[u], x[u]);
            apply_ew_nhwc<DT, VEC, U>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (iw0 + u < whi) take_cell<VEC, true>(is_max, x[u], ih * k.W + iw0 + u, acc, bi);
        }
    float y[1][VEC];
    if (is_max) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[0][e] = acc[e];
    } else {
        const float inv = avg_inv(p, p.kh, p.kw, k.H, k.W, h0, w0, hlo, hhi, wlo, whi);
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[0][e] = round_store<DT>(acc[e] * inv);
    }
    const uint32_t ooff[1] = {pix * (uint32_t)k.C + c0};
    apply_ew_nhwc<DT, VEC, 1>(y, c0, ooff, k.post, k.n_post, k.params, k.C, k.res);
    if (live) {
        store_elems<DT, VEC>(k.out, ooff[0] + pix * k.out_xp, y[0]);
        if (k.idx && is_max) store_indices<VEC>(k.idx + ooff[0], bi);
    }
}

// Pooling over the whole plane (the global pooling at the end of a network) for planes of more
// than a few cells.  A lane of the kernel above would walk the plane one memory round trip
// after the other.  Here a work-group takes one image and k.cv_group channel vectors: all its
// lanes fetch the plane's cells of those channels together (at most U per lane, one round
// trip), take them through the element-wise operations in front of the pool and leave them in
// LDS; then one lane per channel walks its cells in LDS in row-major order.
template <int DT, int VEC>
__global__ __launch_bounds__(256) void nhwc_plane_pool_kernel(const NhwcK k)
{
    extern __shared__ float staged[];
    constexpr int U = 8;
    const uint32_t CV = (uint32_t)k.cv_group, cvn = k.div_cv.d, hw = (uint32_t)(k.H * k.W);
    const uint32_t n = fdiv(blockIdx.x, k.div_wo);
    const uint32_t cv0 = (blockIdx.x - n * k.div_wo.d) * CV;  // first channel vector of this group
    const uint32_t ncv = min(CV, cvn - cv0);
    const uint32_t cl = threadIdx.x / CV, cv = threadIdx.x - cl * CV;  // cell lane, channel vector
    const uint32_t cells_per_pass = blockDim.x / CV;
    const uint32_t img = n * hw;
    if (cv < ncv && cl < cells_per_pass) {
        const uint32_t c0 = (cv0 + cv) * VEC;
        for (uint32_t t0 = cl; t0 < hw; t0 += cells_per_pass * U) {
            uint32_t off[U];
            Raw<DT, VEC> raw[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t t = min(t0 + u * cells_per_pass, hw - 1);  // past the end: the last cell again, not stored
                off[u] = (img + t) * (uint32_t)k.C + c0;
                raw[u] = load_raw<DT, VEC>(k.in, off[u] + (img + t) * k.in_xp);
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) unpack<DT, VEC>(raw[u], x[u]);
            apply_ew_nhwc<DT, VEC, U>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t t = t0 + u * cells_per_pass;
                if (t < hw) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) staged[(t * CV + cv) * VEC + e] = x[u][e];
                }
            }
        }
    }
    __syncthreads();
    if (threadIdx.x >= ncv * VEC) return;
    // lane -> one channel; its cells lie CV * VEC floats apart in LDS
    const bool is_max = k.pool.kind == OP_MAXPOOL;
    float acc = is_max ? -INFINITY : 0.0f;
    int32_t bi = 0;
    const float *cells = staged + threadIdx.x;
    const uint32_t pitch = CV * VEC;
    for (uint32_t t0 = 0; t0 < hw; t0 += U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = cells[min(t0 + u, hw - 1) * pitch];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (t0 + u < hw) {
                if (is_max) {
                    const bool g = v[u] > acc;
                    acc = g ? v[u] : acc;
                    bi = g ? (int32_t)(t0 + u) : bi;
                } else {
                    acc = acc + v[u];
                }
            }
    }
    const uint32_t c = cv0 * VEC + threadIdx.x;  // the lane's channel
    float y[1][1] = {{is_max ? acc : round_store<DT>(acc * k.pool.inv_kk)}};
    const uint32_t ooff[1] = {n * (uint32_t)k.C + c};
    apply_ew_nhwc<DT, 1, 1>(y, c, ooff, k.post, k.n_post, k.params, k.C, k.res);
    store_elems<DT, 1>(k.out, ooff[0] + n * k.out_xp, y[0]);
    if (k.idx && is_max) k.idx[ooff[0]] = bi;
}

// Channel vectors per work-group of nhwc_plane_pool_kernel for a plane of hw cells (0: the plane
// is small enough for the one-pixel-per-lane kernel): at most 48 KiB of LDS, at most 32 vectors,
// a divisor of the work-group size.
int32_t nhwc_plane_group(int64_t hw, int32_t vec, const PoolK &p, int32_t H, int32_t W, int32_t Ho, int32_t Wo)
{
    if (hw <= 16 || p.kh != H || p.kw != W || p.ph != 0 || p.pw != 0 || Ho != 1 || Wo != 1) return 0;
    int32_t cv = 32;
    while (cv > 1 && hw * cv * vec * 4 > 48 * 1024) cv /= 2;
    return hw * cv * vec * 4 > 48 * 1024 ? 0 : cv;
}

// Output block (rows x columns of output pixels per lane) of the compiled windows.  Measured on
// MI355X: sharing cells between the outputs of a block pays for stride 1 (3x3/1: 2 x 2 outputs
// from 4 x 4 cells with float32 vectors, 2 x 1 from 4 x 3 with the twice as long 16-bit
// vectors), not for stride 2 (3x3/2: 1 x 2 was 20..60 % slower than 1 x 1: registers).
// The 16-bit 3x3/1 instance with its 2 x 1 block holds 241 registers (two waves per SIMD); with a 1 x 1 block it holds
// fewer and is slower all the same (halo_stress channels-last step by step, both steps: 162 -> 180 us).
// The planner sizes the grid with it, the launcher picks the instance.
void nhwc_block(const PoolK &p, int32_t vec, int32_t dtype, int32_t &ohb, int32_t &owb)
{
    (void)dtype;
    ohb = owb = 1;
    if (p.kh == 3 && p.kw == 3 && p.sh == 1 && p.sw == 1) {
        ohb = 2;
        owb = vec <= 4 ? 2 : 1;
    }
}

// code of an element-wise list (-1: too long for a code)
static int32_t list_code(const EwOp *ew, int32_t n)
{
    int32_t c = 0, digit = 1;
    if (n > 6) return -1;
    for (int32_t j = 0; j < n; ++j, digit *= K_EW_BASE) c += ew[j].kind * digit;
    return c;
}

// COMMON: also the instances with the lists of the common networks compiled in -- BatchNorm, ReLU behind the pooling
// (where the plan moved the list behind a max pooling: VGG, the ResNet stem) or in front of it (the DenseNet transition).
template <int DT, int VEC, int KH, int KW, int SH, int SW, int OHB, int OWB, bool COMMON = false>
static void launch_block(const NhwcK &k, dim3 grid, dim3 block, hipStream_t st)
{
    constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE;
    const bool idx = k.idx && k.pool.kind == OP_MAXPOOL;
    if constexpr (COMMON) {
        const int32_t pre = list_code(k.pre, k.n_pre), post = list_code(k.post, k.n_post);
        if (!idx && pre == 0 && post == BN_RELU) {
            nhwc_pool_kernel<DT, VEC, KH, KW, SH, SW, OHB, OWB, false, 0, BN_RELU><<<grid, block, 0, st>>>(k);
            return;
        }
        if (!idx && pre == BN_RELU && post == 0) {
            nhwc_pool_kernel<DT, VEC, KH, KW, SH, SW, OHB, OWB, false, BN_RELU, 0><<<grid, block, 0, st>>>(k);
            return;
        }
    }
    if (idx) nhwc_pool_kernel<DT, VEC, KH, KW, SH, SW, OHB, OWB, true><<<grid, block, 0, st>>>(k);
    else nhwc_pool_kernel<DT, VEC, KH, KW, SH, SW, OHB, OWB, false><<<grid, block, 0, st>>>(k);
}

template <int DT, int VEC>
static bs_status launch_nhwc_t(const NhwcK &k, int32_t dtype, dim3 grid, dim3 block, uint64_t lds_bytes, hipStream_t st)
{
    const PoolK &p = k.pool;
    if (p.kind == 0) {
        // the lists of the common networks compiled in: BatchNorm, ReLU (DenseNet) and BatchNorm, Add, ReLU (ResNet)
        constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE, BN_ADD_RELU = OP_BN + (OP_ADD + OP_RELU * K_EW_BASE) * K_EW_BASE;
        if constexpr (VEC > 1) {
            const int32_t code = list_code(k.pre, k.n_pre);
            if (code == BN_RELU) {
                nhwc_stream_kernel<DT, VEC, K_STREAM_U, BN_RELU><<<grid, block, 0, st>>>(k);
                return BS_OK;
            }
            if (code == BN_ADD_RELU) {
                nhwc_stream_kernel<DT, VEC, K_STREAM_U, BN_ADD_RELU><<<grid, block, 0, st>>>(k);
                return BS_OK;
            }
        }
        nhwc_stream_kernel<DT, VEC, K_STREAM_U><<<grid, block, 0, st>>>(k);
        return BS_OK;
    }
    if (k.cv_group > 0) {
        // the plan must be the one this kernel assumes: group size, work-groups per image, LDS
        const int64_t hw = (int64_t)k.H * k.W;
        const int32_t cv = nhwc_plane_group(hw, VEC, p, k.H, k.W, k.Ho, k.Wo);
        const int64_t groups = ((int64_t)k.div_cv.d + cv - 1) / std::max(cv, 1);
        if (cv != k.cv_group || (int64_t)k.div_wo.d != groups || block.x != 256 || 256 % cv != 0 ||
            lds_bytes < (uint64_t)hw * cv * VEC * 4)
            return BS_ERR_UNSUPPORTED;
        nhwc_plane_pool_kernel<DT, VEC><<<grid, block, (size_t)lds_bytes, st>>>(k);
        return BS_OK;
    }
    int32_t ohb, owb;
    nhwc_block(p, VEC, dtype, ohb, owb);
    // the plan's lane grid must be the one the kernel's block shape implies
    if ((int32_t)k.div_wo.d != (k.Wo + owb - 1) / owb || (int32_t)k.div_ho.d != (k.Ho + ohb - 1) / ohb)
        return BS_ERR_UNSUPPORTED;
    constexpr bool WIDE = VEC <= 4;
    if (p.kh == 2 && p.kw == 2 && p.sh == 2 && p.sw == 2) {
        launch_block<DT, VEC, 2, 2, 2, 2, 1, 1, (VEC > 1)>(k, grid, block, st);
    } else if (p.kh == 3 && p.kw == 3 && p.sh == 2 && p.sw == 2) {
        if (ohb != 1 || owb != 1) return BS_ERR_UNSUPPORTED;
        launch_block<DT, VEC, 3, 3, 2, 2, 1, 1, (VEC > 1)>(k, grid, block, st);
    } else if (p.kh == 3 && p.kw == 3 && p.sh == 1 && p.sw == 1) {
        if (ohb != 2 || owb != (WIDE ? 2 : 1)) return BS_ERR_UNSUPPORTED;
        launch_block<DT, VEC, 3, 3, 1, 1, 2, WIDE ? 2 : 1>(k, grid, block, st);
    } else {
        nhwc_pool_any_kernel<DT, VEC><<<grid, block, 0, st>>>(k);
    }
    return BS_OK;
}

bs_status launch_nhwc(const NhwcK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, uint64_t lds_bytes,
                      void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (grid < 1 || grid > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    const int32_t full = dtype == BS_F32 ? 4 : 8;
    // the vector width the plan was made for must be one the kernels exist for and must divide C
    if ((vec != 1 && vec != full) || k.C % vec != 0 || (int64_t)k.div_cv.d * vec != k.C) return BS_ERR_UNSUPPORTED;
    const dim3 g((uint32_t)grid), b((uint32_t)threads);
    if (dtype == BS_F32) return vec == 4 ? launch_nhwc_t<DT_F32, 4>(k, dtype, g, b, lds_bytes, st) : launch_nhwc_t<DT_F32, 1>(k, dtype, g, b, lds_bytes, st);
    if (dtype == BS_BF16) return vec == 8 ? launch_nhwc_t<DT_BF16, 8>(k, dtype, g, b, lds_bytes, st) : launch_nhwc_t<DT_BF16, 1>(k, dtype, g, b, lds_bytes, st);
    if (dtype == BS_F16) return vec == 8 ? launch_nhwc_t<DT_F16, 8>(k, dtype, g, b, lds_bytes, st) : launch_nhwc_t<DT_F16, 1>(k, dtype, g, b, lds_bytes, st);
    return BS_ERR_UNSUPPORTED;
}

}  // namespace bs
