// Channels-last (NHWC) sequences of two pooling steps in one kernel: the depth-first execution
// of Section 3.1 (Figure 3) for tensors whose channels are contiguous -- the stacked pooling
// building block of Section 4.4 (values pass from step to step through on-chip buffers, a
// barrier between the steps) with lanes over channel vectors instead of over a plane's columns.
//
// A tile is TH x TW output pixels of one image and CVB consecutive channel vectors (VEC
// channels each, one 128-bit access).  For a tile the work-group keeps, in LDS, the rectangle
// of the plane between the two pools that the tile's windows cover and, under that, the
// rectangle of the input plane (after the leading element-wise operations) those cover in
// turn: origin[level - 1] = origin[level] * stride - padding, so the rectangles have the same
// extents for every tile.  A cell outside its plane holds the padding value of the pooling
// operation that reads it (-inf for max, +0 for average) and is never computed from earlier
// layers, which keeps the window loops free of bounds tests.  Every value is stored in LDS in
// the storage type: a level's values are a layer's output, already rounded to it.
//
// A lane is (pixel lane, channel vector): the CVB lanes of one pixel are consecutive, so every
// global access of a wave is a run of whole pixels' channels.  A lane has at most K_TILE_U0
// cells of the input rectangle, one block of the rectangle between the pools and one block of
// outputs (the planner only picks tiles for which that holds), at the same places in every
// tile: everything that depends on the lane alone is computed once.
//
// A work-group walks a run of consecutive tiles.  The input cells of the next tile are
// requested before the two pooling levels of the current one run and are consumed after them,
// so the memory round trip is hidden behind arithmetic; BatchNorm parameters of the lane's
// channels are staged in LDS once per run.  Columns of both rectangles are stored even
// columns first, odd columns behind them: all windows start at even columns, so the lanes of a
// wave read consecutive vectors (no bank conflicts between neighbouring blocks).
//
// The arithmetic and its order are those of every other kernel of the library (see
// bs_nhwc.hip): the result is bit-identical to the two-kernel plan.
#include "bs_nhwc_device.h"

#include <algorithm>
#include <map>
#include <mutex>
#include <tuple>

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

// Maximum of values that come straight from memory.  The compiler's fmaxf first re-encodes such
// an operand (v_max_f32 x, x: signalling NaNs must come out quiet), one more instruction per
// value; the instruction itself already returns the other operand for any NaN, and finite values
// are all these kernels promise anything for.
BS_DEV float max_of(float a, float b)
{
    float d;
    asm("v_max_f32_e32 %0, %1, %2" : "=v"(d) : "v"(a), "v"(b));
    return d;
}
BS_DEV float max_of(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// n / f.d without the branch fdiv takes for a divisor of 1 (mul is 0 then: the product is 0 and the mask lets n through)
BS_DEV uint32_t fdiv_flat(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.mul) >> f.shift) | (n & (f.d == 1 ? ~0u : 0u)); }

// a * b + c for operands below 2^24 (cell counts, plane extents, channel counts): one full-rate instruction
BS_DEV uint32_t mad24(uint32_t a, uint32_t b, uint32_t c) { return __umul24(a, b) + c; }

// Place of column c in a rectangle row of w cells: even columns first, odd columns behind them.
BS_DEV uint32_t column_place(uint32_t c, uint32_t w) { return (c >> 1) + (c & 1u) * ((w + 1u) >> 1); }

// The windows of a block of BH x BW neighbouring cells of one pooling operation (K x K, stride S),
// taken from an LDS rectangle of w cells per row, cvb vectors per cell; `first`: the vector of the
// block's first window's first cell (an even column).  The ((BH-1)*S + K) x ((BW-1)*S + K) cells
// under the block are read once, row by row; a row goes to every window that holds it, so each
// window still sees its cells in row-major order (the order of the sum, and of the first
// maximum).  (h0, w0): origin of the first window in the plane the rectangle is cut from (width
// Wp): cell indices for the picks.
template <int DT, int VEC, int K, int S, int BH, int BW, bool MAX, bool IDX>
BS_DEV void pool_block(const uint4 *src, uint32_t first, uint32_t w, uint32_t cvb, int32_t h0, int32_t w0, int32_t Wp,
                       float (&acc)[BH * BW][VEC], int32_t (&bi)[BH * BW][VEC])
{
    constexpr int RR = (BH - 1) * S + K, CC = (BW - 1) * S + K;
    const uint32_t pitch = w * cvb, odd = ((w + 1u) >> 1) * cvb;  // vectors from row to row, from the even columns to the odd ones
#pragma unroll
    for (int a = 0; a < BH; ++a)
#pragma unroll
        for (int b = 0; b < BW; ++b)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                acc[a * BW + b][e] = MAX ? -INFINITY : 0.0f;
                if constexpr (IDX) bi[a * BW + b][e] = max(h0 + a * S, 0) * Wp + max(w0 + b * S, 0);  // first in-range cell
            }
#pragma unroll
    for (int rr = 0; rr < RR; ++rr) {
        float v[CC][VEC];
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
            unpack16<DT, VEC>(src[first + (uint32_t)rr * pitch + (uint32_t)(cc >> 1) * cvb + (uint32_t)(cc & 1) * odd], v[cc]);
#pragma unroll
        for (int a = 0; a < BH; ++a) {
            const int dh = rr - a * S;  // row of window row a's windows this is
            if (dh < 0 || dh >= K) continue;
            if constexpr (MAX && !IDX) {
                // the value of the maximum does not depend on the order: a row's cells first, then the rows
#pragma unroll
                for (int b = 0; b < BW; ++b)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        float t = v[b * S][e];
                        if constexpr (K == 2) t = max_of(t, v[b * S + 1][e]);
                        if constexpr (K == 3) t = max_of(t, v[b * S + 1][e], v[b * S + 2][e]);
                        static_assert(K == 2 || K == 3, "windows of the table");
                        float &m = acc[a * BW + b][e];
                        m = dh == 0 ? t : max_of(m, t);
                    }
                continue;
            }
#pragma unroll
            for (int b = 0; b < BW; ++b)
#pragma unroll
                for (int dw = 0; dw < K; ++dw) {
                    const float(&c)[VEC] = v[b * S + dw];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        float &m = acc[a * BW + b][e];
                        if constexpr (!MAX) {
                            m = m + c[e];  // padding cells hold +0: the sum keeps its bits
                        } else {
                            const bool g = c[e] > m;
                            m = g ? c[e] : m;
                            bi[a * BW + b][e] = g ? (h0 + a * S + dh) * Wp + w0 + b * S + dw : bi[a * BW + b][e];
                        }
                    }
                }
        }
    }
}

// Block of neighbouring cells a lane produces: 2 x 2 for 3 x 3 windows of stride 1 (16 cells read
// for 36 window cells), one cell otherwise.
constexpr int block_edge(int K, int S) { return K == 3 && S == 1 ? 2 : 1; }

// An element-wise list on U register vectors of the lane's channels, BatchNorm scale and shift
// vectors taken from the copies staged in LDS (`par`: the lane's vector of the list's first
// BatchNorm scale; scale and shift of one operation, and operations, `stride` floats apart).
//   off[u]  element offset of vector u inside its image, res_base: the image's first element (residual operands)
// CODE >= 0: the kinds of the list's operations are known at compile time (a code of base-K_EW_BASE digits; n_ew is
// ignored) and the list unrolls into straight code; arguments still come from `ew`.

template <int DT, int VEC, int U, int CODE = -1>
BS_DEV void apply_ew_tile(float (&x)[U][VEC], const uint32_t (&off)[U], const EwOp *ew, int32_t n_ew, const float *par, uint32_t stride,
                          const float *__restrict__ params, const void *const *res, uint32_t res_base)
{
    auto one = [&](const int32_t kind, const int32_t arg) {
        if (kind == OP_BN) {
            float sc[VEC], sh[VEC];
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                const float4 a = *reinterpret_cast<const float4 *>(par + 4 * q), b = *reinterpret_cast<const float4 *>(par + stride + 4 * q);
                sc[4 * q] = a.x; sc[4 * q + 1] = a.y; sc[4 * q + 2] = a.z; sc[4 * q + 3] = a.w;
                sh[4 * q] = b.x; sh[4 * q + 1] = b.y; sh[4 * q + 2] = b.z; sh[4 * q + 3] = b.w;
            }
            par += 2 * stride;
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
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[u][i], lo), hi));
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

// What a lane keeps of one pooling level: its block's place in the destination rectangle and
// where the block's first window starts in the source rectangle.
struct LaneBlock {
    bool on;          // the lane has a block
    int32_t r, c;     // the block's first cell in the destination rectangle
    uint32_t first;   // vector of the first window's first cell in the source rectangle
};

template <int K, int S>
BS_DEV LaneBlock lane_block(uint32_t pl, bool lane_on, const FastDiv &div_bw, int32_t dst_h, uint32_t src_w, uint32_t cvb, uint32_t cvl)
{
    constexpr int B = block_edge(K, S);
    LaneBlock lb;
    const uint32_t bw = div_bw.d, nblocks = (uint32_t)((dst_h + B - 1) / B) * bw;
    lb.on = lane_on && pl < nblocks;
    const uint32_t blk = min(pl, nblocks - 1u);  // lanes without a block shadow the last one (in-bounds reads, nothing stored)
    const uint32_t br = fdiv_flat(blk, div_bw);
    lb.r = (int32_t)br * B;
    lb.c = (int32_t)(blk - __umul24(br, bw)) * B;
    lb.first = mad24(mad24((uint32_t)(lb.r * S), src_w, (uint32_t)(lb.c * S) >> 1), cvb, cvl);  // an even column
    return lb;
}

// One pooling level for the lane's block: source rectangle in LDS -> windows -> normalisation ->
// element-wise list -> destination (the next rectangle in LDS, or the output tensor).
//   dst_h x dst_w   cells of the destination rectangle (the tile's share of the output for the second level)
//   dst_pitch       cells per row the destination rectangle is stored with
//   (dh0, dw0)      plane position of its cell (0, 0); destination plane Hd x Wd, source plane Hs x Ws
//   pad_next        what cells outside the destination plane hold (the next pool's padding)
//   img             the image: residual operands and index outputs are dense tensors
// CODE: the kinds of the level's element-wise list at compile time, or -1 (read at run time); KIND: the pooling
// operation's kind, and no index output, or 0 (read at run time).
template <int DT, int VEC, int K, int S, bool TO_LDS, int CODE = -1, int KIND = 0>
BS_DEV void pool_level(const NhwcTile2K &k, const PoolK &p, const LaneBlock &lb, const uint4 *src, uint32_t src_w, uint4 *dst_lds,
                       int32_t dst_h, int32_t dst_w, uint32_t dst_pitch, int32_t dh0, int32_t dw0, int32_t Hs, int32_t Ws, int32_t Hd,
                       int32_t Wd, const EwOp *ew, int32_t n_ew, const float *par, uint32_t par_stride, float pad_next, uint32_t img,
                       uint32_t cvl, uint32_t c0)
{
    constexpr int B = block_edge(K, S), NB = B * B;
    constexpr uint32_t ES = DT == DT_F32 ? 4 : 2;
    const uint32_t cvb = (uint32_t)k.cvb;
    const bool is_max = KIND != 0 ? KIND == OP_MAXPOOL : p.kind == OP_MAXPOOL;
    const bool want_idx = KIND == 0 && !TO_LDS && is_max && k.idx != nullptr;  // the same for every lane
    const int32_t r = lb.r, c = lb.c;
    const int32_t hd = dh0 + r, wd = dw0 + c;              // the block's first cell in the destination plane
    const int32_t hs = hd * S - p.ph, ws = wd * S - p.pw;  // first window's origin in the source plane
    float y[NB][VEC];
    int32_t bi[NB][VEC];
    if (!is_max) pool_block<DT, VEC, K, S, B, B, false, false>(src, lb.first, src_w, cvb, hs, ws, Ws, y, bi);
    else if (want_idx) pool_block<DT, VEC, K, S, B, B, true, true>(src, lb.first, src_w, cvb, hs, ws, Ws, y, bi);
    else pool_block<DT, VEC, K, S, B, B, true, false>(src, lb.first, src_w, cvb, hs, ws, Ws, y, bi);
    if (!is_max) {
        if (p.count_include_pad == 1) {  // every window counts K * K cells
#pragma unroll
            for (int o = 0; o < NB; ++o)
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[o][e] = round_store<DT>(y[o][e] * p.inv_kk);
        } else {
#pragma unroll
            for (int o = 0; o < NB; ++o) {
                const int32_t h0 = hs + (o / B) * S, w0 = ws + (o % B) * S;
                const float inv = avg_inv(p, K, K, Hs, Ws, h0, w0, max(h0, 0), min(h0 + K, Hs), max(w0, 0), min(w0 + K, Ws));
#pragma unroll
                for (int e = 0; e < VEC; ++e) y[o][e] = round_store<DT>(y[o][e] * inv);
            }
        }
    }
    // which cells of the block lie inside the destination plane, and inside the rectangle (blocks at its edge hang over)
    bool in[NB], cell[NB];
#pragma unroll
    for (int o = 0; o < NB; ++o) {
        in[o] = (uint32_t)(hd + o / B) < (uint32_t)Hd && (uint32_t)(wd + o % B) < (uint32_t)Wd;
        cell[o] = lb.on && r + o / B < dst_h && c + o % B < dst_w;
    }
    // their pixels in the destination plane (clamped to it: safe addresses for the residual operands of cells outside)
    uint32_t pixel[NB], off[NB];
    const uint32_t img_off = img * (uint32_t)(Hd * Wd) * (uint32_t)k.C;  // the image's first element in a dense tensor
    const bool has_list = CODE >= 0 ? ew_code_len(CODE) > 0 : n_ew > 0;
    if (has_list || !TO_LDS) {
#pragma unroll
        for (int o = 0; o < NB; ++o) {
            pixel[o] = mad24((uint32_t)min(max(hd + o / B, 0), Hd - 1), (uint32_t)Wd, (uint32_t)min(max(wd + o % B, 0), Wd - 1));
            off[o] = mad24(pixel[o], (uint32_t)k.C, c0);
        }
    }
    if (has_list) apply_ew_tile<DT, VEC, NB, CODE>(y, off, ew, n_ew, par, par_stride, k.params, k.res, img_off);
    if constexpr (TO_LDS) {
#pragma unroll
        for (int o = 0; o < NB; ++o) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) y[o][e] = in[o] ? y[o][e] : pad_next;
            if (cell[o])
                dst_lds[mad24(mad24((uint32_t)(r + o / B), dst_pitch, column_place((uint32_t)(c + o % B), dst_pitch)), cvb, cvl)] =
                    pack16<DT, VEC>(y[o]);
        }
    } else {
        char *out_img = static_cast<char *>(k.out) + (size_t)img * (size_t)(Hd * Wd) * (k.C + k.out_xp) * ES;
#pragma unroll
        for (int o = 0; o < NB; ++o)
            if (cell[o] && in[o]) {
                store_elems<DT, VEC>(out_img, mad24(pixel[o], k.out_xp, off[o]), y[o]);
                if (want_idx) store_indices<VEC>(k.idx + img_off + off[o], bi[o]);
            }
    }
}

// Input cells a lane holds.
constexpr int K_TILE_U0 = 4;

// Where a tile is: image, channel-vector group, origins of the tile in the three planes.  The same for all lanes.
struct TilePlace {
    uint32_t n, cvg;
    int32_t oh0, ow0, h10, w10, h00, w00;
};

template <int S1, int S2>
BS_DEV TilePlace tile_place(const NhwcTile2K &k, uint32_t t)
{
    // tiles are numbered (channel-vector group, image, tile row, tile column), the column fastest
    TilePlace tp;
    const uint32_t t0 = fdiv(t, k.div_tiles_w);
    const int32_t tc = (int32_t)(t - t0 * k.div_tiles_w.d);
    const uint32_t t1 = fdiv(t0, k.div_tiles_h);
    const int32_t tr = (int32_t)(t0 - t1 * k.div_tiles_h.d);
    tp.cvg = fdiv(t1, k.div_n);
    tp.n = t1 - tp.cvg * k.div_n.d;
    tp.oh0 = tr * k.TH;
    tp.ow0 = tc * k.TW;
    tp.h10 = tp.oh0 * S2 - k.pool2.ph;
    tp.w10 = tp.ow0 * S2 - k.pool2.pw;
    tp.h00 = tp.h10 * S1 - k.pool1.ph;
    tp.w00 = tp.w10 * S1 - k.pool1.pw;
    return tp;
}

// Waves per SIMD the register allocator is held to: one more than it would choose by itself where that costs no
// scratch memory; a second pooling step with stride 1 keeps a 4 x 4 block of cells per lane and gets one wave less.
constexpr int tile_waves(int dt, int k2, int s2) { return (dt == DT_F32 ? 4 : 3) - (k2 == 3 && s2 == 1 ? 1 : 0); }

// What an instance knows of the stack beyond its windows: the kinds of the three element-wise lists as codes (-1: read at run
// time) and the kinds of the two pooling operations (0: read at run time; given, the instance writes no index output).
// Measured on MI355X (stacked pooling of 128 x 128 x 56 x 56, microseconds, float32 / bfloat16 / binary16): nothing known
// 89 / 108 / 106; lists known 77 / 98 / 94; lists and kinds known 94 / 87 / 83 -- with the kinds compiled in the scheduler
// takes 155 registers for float32 (three waves per SIMD instead of four), while the 16-bit instances, at two to three
// waves either way, gain from the shorter code.
template <int PRE_, int MID_, int POST_, int KIND1_, int KIND2_>
struct TileSig {
    static constexpr int PRE = PRE_, MID = MID_, POST = POST_, KIND1 = KIND1_, KIND2 = KIND2_;
    static constexpr int FEWER_WAVES = KIND1_ != 0 ? 1 : 0;  // instances that know the kinds may use one wave per SIMD less
};
using AnySig = TileSig<-1, -1, -1, 0, 0>;
constexpr int K_CODE_BN_RELU = OP_BN + OP_RELU * K_EW_BASE;
// BatchNorm, ReLU in front of the first pooling, nothing between the two, BatchNorm, ReLU behind the second (the stacked
// pooling of Section 4.4 with its activations); the second also with average pooling first and max pooling second compiled in
using BnReluSig = TileSig<K_CODE_BN_RELU, 0, K_CODE_BN_RELU, 0, 0>;
using BnReluAvgMaxSig = TileSig<K_CODE_BN_RELU, 0, K_CODE_BN_RELU, OP_AVGSUM, OP_MAXPOOL>;
template <int DT, int VEC, int K1, int S1, int K2, int S2, class SIG = AnySig>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(tile_waves(DT, K2, S2) - SIG::FEWER_WAVES, tile_waves(DT, K2, S2)))) void nhwc_tile2_kernel(const NhwcTile2K k)
{
    extern __shared__ uint4 lds[];
    uint4 *lds0 = lds, *lds1 = lds + k.lds1_off;
    float *par = reinterpret_cast<float *>(lds + k.par_off);
    constexpr int U = K_TILE_U0;
    constexpr uint32_t ES = DT == DT_F32 ? 4 : 2;

    // the work-group's run of tiles
    const uint32_t per = (k.total_tiles + gridDim.x - 1) / gridDim.x;
    uint32_t t = blockIdx.x * per;
    const uint32_t t_end = min(t + per, k.total_tiles);
    if (t >= t_end) return;

    // lane -> (pixel lane, channel vector of the group), and what follows from the lane alone
    const uint32_t pl = fdiv(threadIdx.x, k.div_cvb);
    const uint32_t cvl = threadIdx.x - pl * k.div_cvb.d;
    const bool lane_on = pl < (uint32_t)k.pl;
    const uint32_t cvb = (uint32_t)k.cvb;
    const uint32_t cells0 = (uint32_t)(k.r0h * k.r0w);
    int32_t cell_r[U], cell_c[U];  // the lane's cells of the input rectangle
    uint32_t cell_at[U];           // ... and their vectors in LDS
    bool cell_on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t cu = pl + (uint32_t)u * (uint32_t)k.pl;
        cell_on[u] = lane_on && cu < cells0;
        const uint32_t cc = min(cu, cells0 - 1u);  // no such cell: the last one again (a safe address), not stored
        const uint32_t r = __umulhi(cc, k.div_r0w.mul) >> k.div_r0w.shift;  // a rectangle has at least two columns
        const uint32_t c = cc - __umul24(r, (uint32_t)k.r0w);
        cell_r[u] = (int32_t)r;
        cell_c[u] = (int32_t)c;
        cell_at[u] = mad24(mad24(r, (uint32_t)k.r0w, column_place(c, (uint32_t)k.r0w)), cvb, cvl);
    }
    const LaneBlock lb1 = lane_block<K1, S1>(pl, lane_on, k.div_bw1, k.r1h, (uint32_t)k.r0w, cvb, cvl);
    const LaneBlock lb2 = lane_block<K2, S2>(pl, lane_on, k.div_bw2, k.TH, (uint32_t)k.r1w, cvb, cvl);
    const float pad0 = (SIG::KIND1 != 0 ? SIG::KIND1 == OP_MAXPOOL : k.pool1.kind == OP_MAXPOOL) ? -INFINITY : 0.0f;
    const float pad1 = (SIG::KIND2 != 0 ? SIG::KIND2 == OP_MAXPOOL : k.pool2.kind == OP_MAXPOOL) ? -INFINITY : 0.0f;
    const uint32_t pitch_b = ((uint32_t)k.C + k.in_xp) * ES;  // bytes from pixel to pixel of the input
    const uint32_t par_stride = cvb * VEC;                    // floats from one staged parameter vector set to the next
    const float *par_lane = par + cvl * VEC;

    // request the lane's input cells of a tile; pixel[u]: their pixels inside the image (clamped to the plane)
    Raw<DT, VEC> raw[U];
    uint32_t pixel[U];
    uint32_t inside = 0;  // bit u: cell u lies inside the plane
    auto request = [&](const TilePlace &tp) {
        const char *in_img = static_cast<const char *>(k.in) + (size_t)tp.n * (size_t)(k.H * k.W) * (k.C + k.in_xp) * ES;
        const uint32_t c0_b = (tp.cvg * cvb + cvl) * VEC * ES;
        inside = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int32_t ih = tp.h00 + cell_r[u], iw = tp.w00 + cell_c[u];
            inside |= ((uint32_t)ih < (uint32_t)k.H && (uint32_t)iw < (uint32_t)k.W) ? 1u << u : 0u;
            // a cell outside the plane is padding: requested from the nearest cell inside (a safe address)
            pixel[u] = mad24((uint32_t)min(max(ih, 0), k.H - 1), (uint32_t)k.W, (uint32_t)min(max(iw, 0), k.W - 1));
            raw[u].q = *reinterpret_cast<const typename Raw<DT, VEC>::type *>(in_img + mad24(pixel[u], pitch_b, c0_b));
        }
    };

    TilePlace tp = tile_place<S1, S2>(k, t);
    request(tp);
    uint32_t staged_cvg = ~0u;
    for (;;) {
        const uint32_t c0 = (tp.cvg * cvb + cvl) * VEC;
        if (tp.cvg != staged_cvg) {
            // BatchNorm scale and shift vectors of this group's channels -> LDS (runs of tiles rarely cross groups)
            if (staged_cvg != ~0u) __syncthreads();
            for (uint32_t h = 0; h < 2u * (uint32_t)k.n_bn; ++h) {  // h: 2 * operation + (0: scale, 1: shift)
                const float *src = k.params + k.bn_arg[h >> 1] + (h & 1u) * (uint32_t)k.C + tp.cvg * par_stride;
                for (uint32_t e = threadIdx.x; e < par_stride; e += 256) par[h * par_stride + e] = src[e];
            }
            staged_cvg = tp.cvg;
            __syncthreads();
        }
        // ---- the tile's input cells (requested one tile ahead) -> leading element-wise operations -> LDS
        {
            float x[U][VEC];
            uint32_t off[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                unpack<DT, VEC>(raw[u], x[u]);
                off[u] = mad24(pixel[u], (uint32_t)k.C, c0);
            }
            if (SIG::PRE >= 0 ? ew_code_len(SIG::PRE) > 0 : k.n_pre > 0)
                apply_ew_tile<DT, VEC, U, SIG::PRE>(x, off, k.pre, k.n_pre, par_lane, par_stride, k.params, k.res,
                                                    tp.n * (uint32_t)(k.H * k.W) * (uint32_t)k.C);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool real = inside >> u & 1u;
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[u][e] = real ? x[u][e] : pad0;
                if (cell_on[u]) lds0[cell_at[u]] = pack16<DT, VEC>(x[u]);
            }
        }
        __syncthreads();
        // ---- first pool, middle element-wise operations -> LDS
        pool_level<DT, VEC, K1, S1, true, SIG::MID, SIG::KIND1>(k, k.pool1, lb1, lds0, (uint32_t)k.r0w, lds1, k.r1h, k.r1w, (uint32_t)k.r1w, tp.h10, tp.w10, k.H,
                                          k.W, k.H1, k.W1, k.mid, k.n_mid, par_lane + 2u * (uint32_t)k.bn_base[1] * par_stride, par_stride,
                                          pad1, tp.n, cvl, c0);
        __syncthreads();
        // ---- request the next tile's cells; they arrive while the second pooling level runs (requested before the
        // first level: measured 4 % slower in float32, registers)
        const uint32_t t_next = t + 1;
        TilePlace tp_next = tp;
        if (t_next < t_end) {
            tp_next = tile_place<S1, S2>(k, t_next);
            request(tp_next);
        }
        // ---- second pool, trailing element-wise operations -> output
        pool_level<DT, VEC, K2, S2, false, SIG::POST, SIG::KIND2>(k, k.pool2, lb2, lds1, (uint32_t)k.r1w, nullptr, min(k.TH, k.Ho - tp.oh0),
                                           min(k.TW, k.Wo - tp.ow0), 0u, tp.oh0, tp.ow0, k.H1, k.W1, k.Ho, k.Wo, k.post, k.n_post,
                                           par_lane + 2u * (uint32_t)k.bn_base[2] * par_stride, par_stride, 0.0f, tp.n, cvl, c0);
        if (t_next >= t_end) break;
        t = t_next;
        tp = tp_next;
    }
}

template <int DT, int VEC, int K1, int S1>
const void *instance_second(const PoolK &p)
{
    if (p.kh == 3 && p.sh == 1) return reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT, VEC, K1, S1, 3, 1>);
    if (p.kh == 3 && p.sh == 2) return reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT, VEC, K1, S1, 3, 2>);
    if (p.kh == 2 && p.sh == 2) return reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT, VEC, K1, S1, 2, 2>);
    return nullptr;
}

template <int DT, int VEC>
const void *instance_first(const PoolK &p1, const PoolK &p2)
{
    if (p1.kh == 3 && p1.sh == 1) return instance_second<DT, VEC, 3, 1>(p2);
    if (p1.kh == 3 && p1.sh == 2) return instance_second<DT, VEC, 3, 2>(p2);
    if (p1.kh == 2 && p1.sh == 2) return instance_second<DT, VEC, 2, 2>(p2);
    return nullptr;
}

bool window_in_table(const PoolK &p)
{
    return p.kh == p.kw && p.sh == p.sw && ((p.kh == 3 && (p.sh == 1 || p.sh == 2)) || (p.kh == 2 && p.sh == 2));
}

}  // namespace

// Are both windows among the compiled ones (3 x 3 stride 1 or 2, 2 x 2 stride 2)?
bool nhwc_tile2_supported(const PoolK &pool1, const PoolK &pool2) { return window_in_table(pool1) && window_in_table(pool2); }

// The kernel multiplies pixel numbers inside an image, channel counts and cell numbers with
// 24-bit multipliers and addresses an image with 32-bit byte offsets.
bool nhwc_tile2_sizes_ok(int64_t H, int64_t W, int64_t C, int64_t extra_per_pixel, int32_t dtype)
{
    const int64_t es = dtype == BS_F32 ? 4 : 2, lim24 = 1 << 24;
    return H * W < lim24 && (C + extra_per_pixel) * es < lim24 && H * W * (C + extra_per_pixel) * es < (1ll << 32);
}

// Extents of the two rectangles of a tile of th x tw outputs, the LDS cells each takes, and the
// blocks per rectangle row of the two pooling levels.  A lane produces a whole block: blocks at
// a rectangle's edge may hang over it, and their windows then read (and drop) cells behind the
// source rectangle's end -- each rectangle is followed by enough spare cells for that.
void nhwc_tile2_shape(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t (&r0)[2], int32_t (&r1)[2], int32_t (&cells)[2],
                      int32_t (&bw)[2])
{
    r1[0] = (th - 1) * p2.sh + p2.kh;
    r1[1] = (tw - 1) * p2.sw + p2.kw;
    r0[0] = (r1[0] - 1) * p1.sh + p1.kh;
    r0[1] = (r1[1] - 1) * p1.sw + p1.kw;
    const int32_t b1 = block_edge(p1.kh, p1.sh), b2 = block_edge(p2.kh, p2.sh);
    cells[0] = (r0[0] + p1.sh * (b1 - 1) + 1) * r0[1];
    cells[1] = (r1[0] + p2.sh * (b2 - 1) + 1) * r1[1];
    bw[0] = (r1[1] + b1 - 1) / b1;
    bw[1] = (tw + b2 - 1) / b2;
}

// Can a work-group of pl pixel lanes take that tile: at most K_TILE_U0 input cells and one block of either level per lane?
bool nhwc_tile2_fits(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t pl)
{
    int32_t r0[2], r1[2], cells[2], bw[2];
    nhwc_tile2_shape(p1, p2, th, tw, r0, r1, cells, bw);
    const int32_t b1 = block_edge(p1.kh, p1.sh), b2 = block_edge(p2.kh, p2.sh);
    return (int64_t)r0[0] * r0[1] <= (int64_t)pl * K_TILE_U0 && (int64_t)((r1[0] + b1 - 1) / b1) * bw[0] <= pl &&
           (int64_t)((th + b2 - 1) / b2) * bw[1] <= pl;
}

// LDS bytes of that tile with cvb channel vectors per work-group and n_bn staged BatchNorm operations (vec channels per vector).
uint64_t nhwc_tile2_lds(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t cvb, int32_t n_bn, int32_t vec)
{
    int32_t r0[2], r1[2], cells[2], bw[2];
    nhwc_tile2_shape(p1, p2, th, tw, r0, r1, cells, bw);
    return ((uint64_t)cells[0] + (uint64_t)cells[1]) * (uint64_t)cvb * 16 + (uint64_t)n_bn * 2 * cvb * vec * 4;
}

bs_status launch_nhwc_tile2(const NhwcTile2K &k, int32_t dtype, int32_t vec, int64_t grid_n, int32_t threads, uint64_t lds_bytes,
                            void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the argument block must describe what the kernel assumes
    int32_t r0[2], r1[2], cells[2], bw[2];
    if (k.TH < 1 || k.TW < 1 || k.cvb < 1 || k.pl < 1 || threads != 256 || k.cvb * k.pl > threads) return BS_ERR_UNSUPPORTED;
    if (vec != (dtype == BS_F32 ? 4 : 8) || k.C % vec != 0 || (k.C / vec) % k.cvb != 0 || k.cvgs != (k.C / vec) / k.cvb) return BS_ERR_UNSUPPORTED;
    if (!nhwc_tile2_supported(k.pool1, k.pool2) || !nhwc_tile2_fits(k.pool1, k.pool2, k.TH, k.TW, k.pl)) return BS_ERR_UNSUPPORTED;
    nhwc_tile2_shape(k.pool1, k.pool2, k.TH, k.TW, r0, r1, cells, bw);
    if (k.n_bn < 0 || k.n_bn > K_TILE_MAX_BN || k.bn_base[0] != 0 || k.bn_base[1] < 0 || k.bn_base[2] < k.bn_base[1] || k.bn_base[2] > k.n_bn)
        return BS_ERR_UNSUPPORTED;
    if (nhwc_tile2_lds(k.pool1, k.pool2, k.TH, k.TW, k.cvb, k.n_bn, vec) > lds_bytes || lds_bytes > 64 * 1024) return BS_ERR_UNSUPPORTED;
    if (r0[0] != k.r0h || r0[1] != k.r0w || r1[0] != k.r1h || r1[1] != k.r1w || k.lds1_off != (uint32_t)(cells[0] * k.cvb) ||
        k.par_off != (uint32_t)((cells[0] + cells[1]) * k.cvb))
        return BS_ERR_UNSUPPORTED;
    if (k.div_cvb.d != (uint32_t)k.cvb || k.div_r0w.d != (uint32_t)k.r0w || k.div_bw1.d != (uint32_t)bw[0] || k.div_bw2.d != (uint32_t)bw[1] ||
        k.div_tiles_w.d != (uint32_t)k.tiles_w || k.div_tiles_h.d != (uint32_t)k.tiles_h || k.div_n.d < 1)
        return BS_ERR_UNSUPPORTED;
    if ((int64_t)k.tiles_h * k.TH < k.Ho || (int64_t)k.tiles_w * k.TW < k.Wo || (int64_t)(k.tiles_h - 1) * k.TH >= k.Ho ||
        (int64_t)(k.tiles_w - 1) * k.TW >= k.Wo)
        return BS_ERR_UNSUPPORTED;
    if ((uint64_t)k.total_tiles != (uint64_t)k.div_n.d * k.tiles_h * k.tiles_w * k.cvgs) return BS_ERR_UNSUPPORTED;
    if (grid_n < 1 || grid_n > (int64_t)k.total_tiles) return BS_ERR_UNSUPPORTED;
    // offsets inside an image are products of 24-bit factors and fit 32 bits, in elements and in bytes
    if (!nhwc_tile2_sizes_ok(k.H, k.W, k.C, k.in_xp, dtype) || !nhwc_tile2_sizes_ok(k.Ho, k.Wo, k.C, k.out_xp, dtype) ||
        !nhwc_tile2_sizes_ok(k.H1, k.W1, k.C, 0, dtype))
        return BS_ERR_UNSUPPORTED;
    const void *fn = dtype == BS_F32    ? instance_first<DT_F32, 4>(k.pool1, k.pool2)
                     : dtype == BS_BF16 ? instance_first<DT_BF16, 8>(k.pool1, k.pool2)
                     : dtype == BS_F16  ? instance_first<DT_F16, 8>(k.pool1, k.pool2)
                                        : nullptr;
    if (!fn) return BS_ERR_UNSUPPORTED;
    // the instance that knows the whole stack, where there is one
    {
        auto code = [](const EwOp *ew, int32_t n) {
            int32_t c = 0, digit = 1;
            if (n > 6) return -1;
            for (int32_t j = 0; j < n; ++j, digit *= K_EW_BASE) c += ew[j].kind * digit;
            return c;
        };
        const PoolK &a = k.pool1, &b = k.pool2;
        if (a.kh == 3 && a.sh == 1 && b.kh == 3 && b.sh == 2 && code(k.pre, k.n_pre) == K_CODE_BN_RELU && k.n_mid == 0 &&
            code(k.post, k.n_post) == K_CODE_BN_RELU) {
            const bool avg_max = a.kind == OP_AVGSUM && b.kind == OP_MAXPOOL && !k.idx;
            if (dtype == BS_F32) fn = reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT_F32, 4, 3, 1, 3, 2, BnReluSig>);
            else if (dtype == BS_BF16 && avg_max) fn = reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT_BF16, 8, 3, 1, 3, 2, BnReluAvgMaxSig>);
            else if (dtype == BS_F16 && avg_max) fn = reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT_F16, 8, 3, 1, 3, 2, BnReluAvgMaxSig>);
            else if (dtype == BS_BF16) fn = reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT_BF16, 8, 3, 1, 3, 2, BnReluSig>);
            else fn = reinterpret_cast<const void *>(&nhwc_tile2_kernel<DT_F16, 8, 3, 1, 3, 2, BnReluSig>);
        }
    }
    // no more work-groups than the device holds at once: each walks its run of tiles from start to end
    int64_t groups = grid_n;
    {
        static std::mutex mu;
        static std::map<std::tuple<int, const void *, uint64_t>, int64_t> resident;  // (device, instance, LDS bytes) -> work-groups
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        const auto key = std::make_tuple(dev, fn, lds_bytes);
        std::lock_guard<std::mutex> lock(mu);
        auto it = resident.find(key);
        if (it == resident.end()) {
            int per_cu = 0, cus = 0;
            if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, (size_t)lds_bytes);
            if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) {
                set_hip_error((int32_t)e);
                return BS_ERR_HIP;
            }
            it = resident.emplace(key, (int64_t)std::max(per_cu, 1) * std::max(cus, 1)).first;
        }
        groups = std::min(groups, it->second);
    }
    NhwcTile2K args = k;
    void *kargs[] = {&args};
    const hipError_t e = hipLaunchKernel(fn, dim3((uint32_t)groups), dim3((uint32_t)threads), kargs, (size_t)lds_bytes, st);
    if (e != hipSuccess) {
        set_hip_error((int32_t)e);
        return BS_ERR_HIP;
    }
    return BS_OK;
}

}  // namespace bs
