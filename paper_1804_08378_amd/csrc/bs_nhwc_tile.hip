// Channels-last (NHWC) sequences of two pooling steps in one kernel: the depth-first execution
// of Section 3.1 (Figure 3) for tensors whose channels are contiguous -- the stacked pooling
// building block of Section 4.4 (values pass from step to step through on-chip buffers, a
// barrier between the steps) with lanes over channel vectors instead of over a plane's columns.
//
// A work-group owns a tile of TH x TW output pixels of one image and CVB consecutive channel
// vectors (VEC channels each, one 128-bit access).  For the tile it keeps, in LDS, the
// rectangle of the plane between the two pools that the tile's windows cover and, under that,
// the rectangle of the input plane (after the leading element-wise operations) those cover in
// turn: origin[level - 1] = origin[level] * stride - padding, so the rectangles have the same
// extents for every tile.  A cell outside its plane holds the padding value of the pooling
// operation that reads it (-inf for max, +0 for average) and is never computed from earlier
// layers, which keeps the window loops free of bounds tests.  Every value is stored in LDS in
// the storage type: a level's values are a layer's output, already rounded to it.
//
// A lane is (pixel lane, channel vector): the CVB lanes of one pixel are consecutive, so every
// global access of a wave is a run of whole pixels' channels and every LDS access a contiguous
// run of 16-byte vectors.  The arithmetic and its order are those of every other kernel of the
// library (see bs_nhwc.hip): the result is bit-identical to the two-kernel plan.
#include "bs_nhwc_device.h"

#include "bs_internal.h"

namespace bs {
namespace {

// VEC values -> one 16-byte register block in the storage type (float32: VEC = 4; 16-bit: VEC = 8)
template <int DT, int VEC>
BS_DEV uint4 pack16(const float (&v)[VEC])
{
    if constexpr (DT == DT_F32) {
        static_assert(VEC == 4, "one 128-bit vector");
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    } else {
        static_assert(VEC == 8, "one 128-bit vector");
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)half_bits<DT>(v[2 * i]) | ((uint32_t)half_bits<DT>(v[2 * i + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int DT, int VEC>
BS_DEV void unpack16(const uint4 &q, float (&v)[VEC])
{
    Raw<DT, VEC> r;
    r.q = q;
    unpack<DT, VEC>(r, v);
}

// K x K window (row-major) of one pooling operation over an LDS rectangle whose rows are `pitch`
// vectors apart, first cell at `cell`: maximum (with the first maximum's plane index when IDX)
// or sum.  (h0, w0): the window's first cell in the plane the rectangle is cut from, of width Wp.
template <int DT, int VEC, int K, bool IDX>
BS_DEV void window_reduce(const uint4 *lds, uint32_t cell, uint32_t pitch, uint32_t cvb, bool is_max, int32_t h0, int32_t w0,
                          int32_t Hp, int32_t Wp, float (&acc)[VEC], int32_t (&bi)[VEC])
{
    const int32_t first = max(h0, 0) * Wp + max(w0, 0);  // first in-range cell
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        acc[e] = is_max ? -INFINITY : 0.0f;
        bi[e] = first;
    }
    (void)Hp;
#pragma unroll
    for (int dh = 0; dh < K; ++dh)
#pragma unroll
        for (int dw = 0; dw < K; ++dw) {
            float v[VEC];
            unpack16<DT, VEC>(lds[cell + ((uint32_t)dh * pitch + (uint32_t)dw) * cvb], v);
            if (is_max) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    if constexpr (IDX) {
                        const bool g = v[e] > acc[e];
                        acc[e] = g ? v[e] : acc[e];
                        bi[e] = g ? (h0 + dh) * Wp + w0 + dw : bi[e];
                    } else {
                        acc[e] = __builtin_fmaxf(acc[e], v[e]);
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = acc[e] + v[e];  // padding cells hold +0: the sum keeps its bits
            }
        }
}

template <int DT, int VEC, int K1, int S1, int K2, int S2>
__global__ __launch_bounds__(256) void nhwc_tile2_kernel(const NhwcTile2K k)
{
    extern __shared__ uint4 lds[];
    uint4 *lds0 = lds, *lds1 = lds + (uint32_t)(k.r0h * k.r0w * k.cvb);

    // work-group -> (image, tile row, tile column, channel-vector group), the group fastest
    const uint32_t g0 = blockIdx.x;
    const uint32_t t0 = fdiv(g0, k.div_cvgs);
    const uint32_t cvg = g0 - t0 * k.div_cvgs.d;
    const uint32_t t1 = fdiv(t0, k.div_tiles_w);
    const int32_t tc = (int32_t)(t0 - t1 * k.div_tiles_w.d);
    const uint32_t n = fdiv(t1, k.div_tiles_h);
    const int32_t tr = (int32_t)(t1 - n * k.div_tiles_h.d);
    // lane -> (pixel lane, channel vector of the group)
    const uint32_t pl = fdiv(threadIdx.x, k.div_cvb);
    const uint32_t cvl = threadIdx.x - pl * k.div_cvb.d;
    const bool lane_on = pl < (uint32_t)k.pl;
    const uint32_t c0 = (cvg * (uint32_t)k.cvb + cvl) * VEC;
    const uint32_t cvb = (uint32_t)k.cvb;

    const int32_t oh0 = tr * k.TH, ow0 = tc * k.TW;                              // tile origin in the output plane
    const int32_t h10 = oh0 * S2 - k.pool2.ph, w10 = ow0 * S2 - k.pool2.pw;      // in the plane between the pools
    const int32_t h00 = h10 * S1 - k.pool1.ph, w00 = w10 * S1 - k.pool1.pw;      // in the input plane
    const bool max1 = k.pool1.kind == OP_MAXPOOL, max2 = k.pool2.kind == OP_MAXPOOL;
    const float pad0 = max1 ? -INFINITY : 0.0f, pad1 = max2 ? -INFINITY : 0.0f;

    // ---- phase 0: input rectangle -> leading element-wise operations -> LDS
    if (lane_on) {
        const uint32_t cells = (uint32_t)(k.r0h * k.r0w);
        for (uint32_t cell = pl; cell < cells; cell += 2u * (uint32_t)k.pl) {
            float x[2][VEC];
            uint32_t off[2];
            bool in[2];
            Raw<DT, VEC> raw[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t cu = min(cell + (uint32_t)u * (uint32_t)k.pl, cells - 1u);
                const uint32_t r = fdiv(cu, k.div_r0w);
                const int32_t ih = h00 + (int32_t)r, iw = w00 + (int32_t)(cu - r * k.div_r0w.d);
                in[u] = ih >= 0 && ih < k.H && iw >= 0 && iw < k.W;
                const uint32_t pixel = (n * (uint32_t)k.H + (uint32_t)min(max(ih, 0), k.H - 1)) * (uint32_t)k.W +
                                       (uint32_t)min(max(iw, 0), k.W - 1);
                off[u] = pixel * (uint32_t)k.C + c0;
                raw[u] = load_raw<DT, VEC>(k.in, off[u] + pixel * k.in_xp);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) unpack<DT, VEC>(raw[u], x[u]);
            apply_ew_nhwc<DT, VEC, 2>(x, c0, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t cu = cell + (uint32_t)u * (uint32_t)k.pl;
                if (cu < cells) {
                    if (!in[u]) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) x[u][e] = pad0;
                    }
                    lds0[cu * cvb + cvl] = pack16<DT, VEC>(x[u]);
                }
            }
        }
    }
    __syncthreads();

    // ---- phase 1: first pool, middle element-wise operations -> LDS
    if (lane_on) {
        const uint32_t cells = (uint32_t)(k.r1h * k.r1w);
        for (uint32_t cell = pl; cell < cells; cell += (uint32_t)k.pl) {
            const uint32_t r = fdiv(cell, k.div_r1w);
            const uint32_t c = cell - r * k.div_r1w.d;
            const int32_t h1 = h10 + (int32_t)r, w1 = w10 + (int32_t)c;
            const int32_t hw = h1 * S1 - k.pool1.ph, ww = w1 * S1 - k.pool1.pw;  // window origin in the input plane
            float y[1][VEC];
            int32_t unused[VEC];
            window_reduce<DT, VEC, K1, false>(lds0, (r * S1 * (uint32_t)k.r0w + c * S1) * cvb + cvl, (uint32_t)k.r0w, cvb, max1, hw, ww,
                                              k.H, k.W, y[0], unused);
            if (!max1) {
                const float inv = avg_inv(k.pool1, K1, K1, k.H, k.W, hw, ww, max(hw, 0), min(hw + K1, k.H), max(ww, 0),
                                          min(ww + K1, k.W));
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[0][e] = round_store<DT>(y[0][e] * inv);
            }
            const bool in = h1 >= 0 && h1 < k.H1 && w1 >= 0 && w1 < k.W1;
            const uint32_t pixel = (n * (uint32_t)k.H1 + (uint32_t)min(max(h1, 0), k.H1 - 1)) * (uint32_t)k.W1 +
                                   (uint32_t)min(max(w1, 0), k.W1 - 1);
            const uint32_t off[1] = {pixel * (uint32_t)k.C + c0};
            apply_ew_nhwc<DT, VEC, 1>(y, c0, off, k.mid, k.n_mid, k.params, k.C, k.res);
            if (!in) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[0][e] = pad1;
            }
            lds1[cell * cvb + cvl] = pack16<DT, VEC>(y[0]);
        }
    }
    __syncthreads();

    // ---- phase 2: second pool, trailing element-wise operations -> output
    if (lane_on) {
        const uint32_t cells = (uint32_t)(k.TH * k.TW);
        const bool want_idx = k.idx != nullptr && max2;  // the same for every lane
        for (uint32_t cell = pl; cell < cells; cell += (uint32_t)k.pl) {
            const uint32_t a = fdiv(cell, k.div_tw);
            const uint32_t b = cell - a * k.div_tw.d;
            const int32_t oh = oh0 + (int32_t)a, ow = ow0 + (int32_t)b;
            const int32_t hw = oh * S2 - k.pool2.ph, ww = ow * S2 - k.pool2.pw;  // window origin in the plane between the pools
            float y[1][VEC];
            int32_t bi[VEC];
            const uint32_t first = (a * S2 * (uint32_t)k.r1w + b * S2) * cvb + cvl;
            if (want_idx) window_reduce<DT, VEC, K2, true>(lds1, first, (uint32_t)k.r1w, cvb, max2, hw, ww, k.H1, k.W1, y[0], bi);
            else window_reduce<DT, VEC, K2, false>(lds1, first, (uint32_t)k.r1w, cvb, max2, hw, ww, k.H1, k.W1, y[0], bi);
            if (!max2) {
                const float inv = avg_inv(k.pool2, K2, K2, k.H1, k.W1, hw, ww, max(hw, 0), min(hw + K2, k.H1), max(ww, 0),
                                          min(ww + K2, k.W1));
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[0][e] = round_store<DT>(y[0][e] * inv);
            }
            const bool in = oh < k.Ho && ow < k.Wo;
            const uint32_t pixel = (n * (uint32_t)k.Ho + (uint32_t)min(oh, k.Ho - 1)) * (uint32_t)k.Wo + (uint32_t)min(ow, k.Wo - 1);
            const uint32_t off[1] = {pixel * (uint32_t)k.C + c0};
            apply_ew_nhwc<DT, VEC, 1>(y, c0, off, k.post, k.n_post, k.params, k.C, k.res);
            if (in) {
                store_elems<DT, VEC>(k.out, off[0] + pixel * k.out_xp, y[0]);
                if (want_idx) store_indices<VEC>(k.idx + off[0], bi);
            }
        }
    }
}

template <int DT, int VEC, int K1, int S1>
bool launch_second(const NhwcTile2K &k, dim3 grid, dim3 block, size_t lds, hipStream_t st)
{
    const PoolK &p = k.pool2;
    if (p.kh != p.kw || p.sh != p.sw) return false;
    if (p.kh == 3 && p.sh == 1) nhwc_tile2_kernel<DT, VEC, K1, S1, 3, 1><<<grid, block, lds, st>>>(k);
    else if (p.kh == 3 && p.sh == 2) nhwc_tile2_kernel<DT, VEC, K1, S1, 3, 2><<<grid, block, lds, st>>>(k);
    else if (p.kh == 2 && p.sh == 2) nhwc_tile2_kernel<DT, VEC, K1, S1, 2, 2><<<grid, block, lds, st>>>(k);
    else return false;
    return true;
}

template <int DT, int VEC>
bool launch_first(const NhwcTile2K &k, dim3 grid, dim3 block, size_t lds, hipStream_t st)
{
    const PoolK &p = k.pool1;
    if (p.kh != p.kw || p.sh != p.sw) return false;
    if (p.kh == 3 && p.sh == 1) return launch_second<DT, VEC, 3, 1>(k, grid, block, lds, st);
    if (p.kh == 3 && p.sh == 2) return launch_second<DT, VEC, 3, 2>(k, grid, block, lds, st);
    if (p.kh == 2 && p.sh == 2) return launch_second<DT, VEC, 2, 2>(k, grid, block, lds, st);
    return false;
}

bool window_in_table(const PoolK &p)
{
    return p.kh == p.kw && p.sh == p.sw && ((p.kh == 3 && (p.sh == 1 || p.sh == 2)) || (p.kh == 2 && p.sh == 2));
}

}  // namespace

// Are both windows among the compiled ones (3 x 3 stride 1 or 2, 2 x 2 stride 2)?
bool nhwc_tile2_supported(const PoolK &pool1, const PoolK &pool2) { return window_in_table(pool1) && window_in_table(pool2); }

// LDS bytes of a tile of th x tw outputs with cvb channel vectors per work-group, and the extents of its two rectangles.
uint64_t nhwc_tile2_lds(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t cvb, int32_t (&r0)[2], int32_t (&r1)[2])
{
    r1[0] = (th - 1) * p2.sh + p2.kh;
    r1[1] = (tw - 1) * p2.sw + p2.kw;
    r0[0] = (r1[0] - 1) * p1.sh + p1.kh;
    r0[1] = (r1[1] - 1) * p1.sw + p1.kw;
    return ((uint64_t)r0[0] * r0[1] + (uint64_t)r1[0] * r1[1]) * (uint64_t)cvb * 16;
}

bs_status launch_nhwc_tile2(const NhwcTile2K &k, int32_t dtype, int32_t vec, int64_t grid_n, int32_t threads, uint64_t lds_bytes,
                            void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the argument block must describe what the kernel assumes
    int32_t r0[2], r1[2];
    if (k.TH < 1 || k.TW < 1 || k.cvb < 1 || k.pl < 1 || threads != 256 || k.cvb * k.pl > threads) return BS_ERR_UNSUPPORTED;
    if (vec != (dtype == BS_F32 ? 4 : 8) || k.C % vec != 0 || (k.C / vec) % k.cvb != 0 || k.cvgs != (k.C / vec) / k.cvb) return BS_ERR_UNSUPPORTED;
    if (nhwc_tile2_lds(k.pool1, k.pool2, k.TH, k.TW, k.cvb, r0, r1) > lds_bytes || lds_bytes > 64 * 1024) return BS_ERR_UNSUPPORTED;
    if (r0[0] != k.r0h || r0[1] != k.r0w || r1[0] != k.r1h || r1[1] != k.r1w) return BS_ERR_UNSUPPORTED;
    if (k.div_cvb.d != (uint32_t)k.cvb || k.div_r0w.d != (uint32_t)k.r0w || k.div_r1w.d != (uint32_t)k.r1w || k.div_tw.d != (uint32_t)k.TW ||
        k.div_cvgs.d != (uint32_t)k.cvgs || k.div_tiles_w.d != (uint32_t)k.tiles_w || k.div_tiles_h.d != (uint32_t)k.tiles_h)
        return BS_ERR_UNSUPPORTED;
    if ((int64_t)k.tiles_h * k.TH < k.Ho || (int64_t)k.tiles_w * k.TW < k.Wo) return BS_ERR_UNSUPPORTED;
    if (grid_n < 1 || grid_n > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const size_t lds = (size_t)lds_bytes;
    bool ok = false;
    if (dtype == BS_F32) ok = launch_first<DT_F32, 4>(k, grid, block, lds, st);
    else if (dtype == BS_BF16) ok = launch_first<DT_BF16, 8>(k, grid, block, lds, st);
    else if (dtype == BS_F16) ok = launch_first<DT_F16, 8>(k, grid, block, lds, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
