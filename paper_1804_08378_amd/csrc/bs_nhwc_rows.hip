// Channels-last tensors, two pooling steps in one kernel without LDS: nhwc_rows2_kernel.
//
// The row-major lane-exchange kernel (pool_xrows2_kernel) turned by ninety degrees.  A lane owns one
// pixel column w of the image and one vector of VEC consecutive channels; the lanes of a wave are the
// columns of one image row (W <= 64), the waves of a work-group are channel vectors of the same rows.
// A lane walks down a chunk of output rows with the rows of both pooling levels in registers; what a
// window needs from the columns left and right of it are the neighbouring lanes' values, read through
// data-parallel-primitive operands (the compiler folds a lane shift into the add that uses it; a
// maximum takes one v_mov_b32 with the padding value as its "old" operand).  Nothing goes through
// LDS; the waves of a work-group meet at a barrier after every row request, which only keeps them
// on the same rows (row_sync below); every input element is loaded once per chunk that needs it.
//
// Memory: a lane reads the 16 bytes of its channel vector, C * element size bytes from its neighbour's;
// the cache lines of a pixel are shared by the waves of the work-group (four: half a 128-byte line of a
// pixel; eight measured slower, see K_NHWC_ROWS_WAVES), which request the same rows at the same time.  Measured on
// MI355X, the rate of these 16-byte lane requests is what bounds the kernel (about 2.3 TB/s of algorithmic bytes).
//
// Compiled for 16-bit storage and the 3 x 3 windows with padding 1 the benchmark's stacks use: first pooling with
// stride 1 (average or maximum), second pooling a maximum with stride 1 or 2, no index output,
// averages that divide by nine (count_include_pad), lists of BatchNorm / ReLU / leaky ReLU / clamp.
// Everything else stays with the tile kernel (bs_nhwc_tile.hip).
#include "bs_xrows_device.h"
#include "bs_nhwc_device.h"

#include "bs_internal.h"

#if !defined(BS_NHWC_ROWS_SYNC)
#define BS_NHWC_ROWS_SYNC 1
#endif

namespace bs {
namespace {

// value of the same register in the lane to the left / right (beyond the wave's ends: +0)
BS_DEV float left0(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), 0x138, 0xf, 0xf, true));
}
BS_DEV float right0(float v)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), 0x130, 0xf, 0xf, true));
}
// ... beyond the wave's ends: pad
BS_DEV float left_or(float v, float pad)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp((int)__float_as_uint(pad), (int)__float_as_uint(v), 0x138, 0xf, 0xf, false));
}
BS_DEV float right_or(float v, float pad)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp((int)__float_as_uint(pad), (int)__float_as_uint(v), 0x130, 0xf, 0xf, false));
}

// Parameters of a compile-time list for the lane's VEC channels.
template <class EW, int VEC>
struct ColParams {
    float sc[EW::n > 0 ? EW::n : 1][VEC], sh[EW::n > 0 ? EW::n : 1][VEC];
};
template <class EW, int VEC>
BS_DEV void col_load_params(const EwOp *ew, const float *__restrict__ params, int32_t C, uint32_t c0, ColParams<EW, VEC> &p)
{
#pragma unroll
    for (int j = 0; j < EW::n; ++j) {
        if (EW::kind(j) == OP_BN) {
            load_params<VEC>(params, (uint32_t)ew[j].arg + c0, p.sc[j]);
            load_params<VEC>(params, (uint32_t)(ew[j].arg + C) + c0, p.sh[j]);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const bool two = EW::kind(j) == OP_LEAKY || EW::kind(j) == OP_CLAMP;  // [slope, -] / [lo, hi]
                p.sc[j][e] = two ? params[ew[j].arg] : 0.0f;
                p.sh[j][e] = two ? params[ew[j].arg + 1] : 0.0f;
            }
        }
    }
}
template <int DT, class EW, int VEC>
BS_DEV void col_apply(float (&x)[VEC], const ColParams<EW, VEC> &p)
{
#pragma unroll
    for (int j = 0; j < EW::n; ++j) {
        if (EW::kind(j) == OP_BN) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = __builtin_fmaf(x[e], p.sc[j][e], p.sh[j][e]);
            round_store_all<DT, VEC>(x);
        } else if (EW::kind(j) == OP_LEAKY) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(x[e] > 0.0f ? x[e] : x[e] * p.sc[j][e]);
        } else if (EW::kind(j) == OP_CLAMP) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[e], p.sc[j][e]), p.sh[j][e]));
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[e] = __builtin_fmaxf(x[e], 0.0f);  // NaN, -0 -> +0
        }
    }
}

// One 3 x 3 / padding 1 pooling of the rows a, b, c (above, at, below the output row) at the lane's column.
// Maximum: down the rows first, then across the three lanes.  Average: the row-major sum of the layer
// definition, from +0 (a padding cell adds +0, which leaves a sum that started at +0 as it is), times 1/9.
template <int DT, int KIND, int VEC, bool NONNEG>
BS_DEV void col_pool3(const float (&a)[VEC], const float (&b)[VEC], const float (&c)[VEC], float inv_kk, float (&y)[VEC])
{
    if constexpr (KIND == OP_MAXPOOL) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const float m = __builtin_fmaxf(__builtin_fmaxf(a[e], b[e]), c[e]);
            y[e] = __builtin_fmaxf(__builtin_fmaxf(left_or(m, -INFINITY), m), right_or(m, -INFINITY));
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float s = NONNEG ? left0(a[e]) : 0.0f + left0(a[e]);
            s = s + a[e];
            s = s + right0(a[e]);
            s = s + left0(b[e]);
            s = s + b[e];
            s = s + right0(b[e]);
            s = s + left0(c[e]);
            s = s + c[e];
            s = s + right0(c[e]);
            y[e] = s * inv_kk;
        }
        round_store_all<DT, VEC>(y);
    }
}

// KIND1, KIND2: the two poolings (3 x 3, padding 1; the first with stride 1, the second with stride S2).
// EW0, EW1, EW2: the lists in front of, between and behind them as compile-time codes (RowsEw).
template <int DT, int VEC, int KIND1, int KIND2, int S2, int EW0, int EW1, int EW2>
__global__ __launch_bounds__(64 * K_NHWC_ROWS_WAVES) void nhwc_rows2_kernel(const NhwcTile2K k)
{
    constexpr int K = 3, P = 1;
    constexpr int NS = S2;        // new input rows (= new rows of the plane between the poolings) per output row
    constexpr int KEEP1 = K - S2;  // rows of that plane two consecutive output rows share
    using E0 = RowsEw<EW0>;
    using E1 = RowsEw<EW1>;
    using E2 = RowsEw<EW2>;
    constexpr bool NONNEG0 = ends_in_relu<E0>();
    const float pad0 = KIND1 == OP_MAXPOOL ? -INFINITY : 0.0f;  // value of a cell outside the input plane
    const float pad1 = KIND2 == OP_MAXPOOL ? -INFINITY : 0.0f;  // ... outside the plane between the poolings

    // work-group -> (channel-vector group, chunk, image), numbered in that order.  The chip hands consecutive work-groups to
    // its eight XCDs in turn (work-group b runs on XCD b % 8), each with an L2 of its own: with a batch that divides by
    // eight, XCD x takes the images x, x + 8, ..., so that the groups that share a pixel's cache lines and the chunks
    // that share input rows meet in one L2 (halo_stress bfloat16: 110 MB fetched for 103 MB of input; numbered
    // straight through, the two groups of a cache line sat on different XCDs and each fetched it: 239 MB).
    uint32_t s = blockIdx.x, xcd = 0, n_step = 1;
    {
        const uint32_t n8 = fdiv(fdiv(gridDim.x >> 3, k.div_cvgs), k.div_chunks);  // images / 8, rounded down
        if (n8 * k.div_chunks.d * k.div_cvgs.d * 8u == gridDim.x) {
            xcd = s & 7u;
            s >>= 3;
            n_step = 8;
        }
    }
    const uint32_t t1 = fdiv(s, k.div_cvgs);
    const uint32_t cvg = s - t1 * k.div_cvgs.d;
    const uint32_t n_hi = fdiv(t1, k.div_chunks);
    const int32_t chunk = (int32_t)(t1 - n_hi * k.div_chunks.d);
    const uint32_t n = n_hi * n_step + xcd;
    const int32_t w = (int32_t)(threadIdx.x & 63u);
    const uint32_t c0 = (cvg * (uint32_t)k.cvb + (threadIdx.x >> 6)) * VEC;      // first channel of the lane
    const bool live = w < k.W;
    const uint32_t wc = live ? (uint32_t)w : 0u;

    ColParams<E0, VEC> p0;
    ColParams<E1, VEC> p1;
    ColParams<E2, VEC> p2;
    col_load_params<E0, VEC>(k.pre, k.params, k.C, c0, p0);
    col_load_params<E1, VEC>(k.mid, k.params, k.C, c0, p1);
    col_load_params<E2, VEC>(k.post, k.params, k.C, c0, p2);

    constexpr int ES = DT != DT_F32 ? 2 : 4;
    const uint32_t in_pitch = (uint32_t)k.C + k.in_xp, out_pitch = (uint32_t)k.C + k.out_xp;  // elements from pixel to pixel
    // the image's first element; offsets inside an image fit 32 bits (checked by the launcher)
    const char *inp = static_cast<const char *>(k.in) + (size_t)n * (size_t)(k.H * k.W) * in_pitch * ES;
    char *outp = static_cast<char *>(k.out) + (size_t)n * (size_t)(k.Ho * k.Wo) * out_pitch * ES;
    using Row = Raw<DT, VEC>;
    auto fetch = [&](int32_t ih) {  // the lane's vector of input row ih, clamped into the plane (a row outside is padding: replaced when settled)
        const uint32_t row = (uint32_t)min(max(ih, 0), k.H - 1);
        return load_raw<DT, VEC>(inp, (row * (uint32_t)k.W + wc) * in_pitch + c0);
    };
    // The waves of the work-group request a row together: a cache line of the row (one pixel's channels) is asked for
    // by all of them while it is on its way or freshly arrived, not again after the requests of faster waves for later
    // rows have pushed it out of the first-level cache.  Every wave reaches every call (the chunk length is the same
    // for all of them).
    auto row_sync = [&]() {
        if (BS_NHWC_ROWS_SYNC) __syncthreads();
    };
    // registers -> input row after the leading list, padding outside the plane and in the wave's idle lanes
    auto settle = [&](const Row &r, int32_t ih, float (&y)[VEC]) {
        unpack<DT, VEC>(r, y);
        col_apply<DT, E0, VEC>(y, p0);
        const bool ok = live && ih >= 0 && ih < k.H;
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[e] = ok ? y[e] : pad0;
    };
    // row r1 of the plane between the poolings from the input rows a, b, c: first pooling, middle list, padding
    auto level1 = [&](int32_t r1, const float (&a)[VEC], const float (&b)[VEC], const float (&c)[VEC], float (&y)[VEC]) {
        col_pool3<DT, KIND1, VEC, NONNEG0>(a, b, c, k.pool1.inv_kk, y);
        col_apply<DT, E1, VEC>(y, p1);
        const bool ok = live && r1 >= 0 && r1 < k.H1;
#pragma unroll
        for (int e = 0; e < VEC; ++e) y[e] = ok ? y[e] : pad1;
    };

    const int32_t oh0 = chunk * k.rc;
    float keep0[2][VEC];  // the two newest input rows
    float win1[K][VEC];   // the rows of the plane between the poolings under the current output row
    {
        const int32_t r1f = oh0 * S2 - P, h0f = r1f - P;
        Row r[5];
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            r[j] = fetch(h0f + j);
            row_sync();
        }
        float l0[5][VEC];
#pragma unroll
        for (int j = 0; j < 5; ++j) settle(r[j], h0f + j, l0[j]);
#pragma unroll
        for (int j = 0; j < K; ++j) level1(r1f + j, l0[j], l0[j + 1], l0[j + 2], win1[j]);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            keep0[0][e] = l0[3][e];
            keep0[1][e] = l0[4][e];
        }
    }
    auto reduce = [&](float (&y)[VEC]) {
        col_pool3<DT, KIND2, VEC, ends_in_relu<E1>()>(win1[0], win1[1], win1[2], k.pool2.inv_kk, y);
        col_apply<DT, E2, VEC>(y, p2);
    };
    auto put = [&](int32_t t, const float (&y)[VEC]) {
        const int32_t oh = oh0 + t;
        const int32_t ow = S2 == 2 ? w >> 1 : w;
        if (live && (S2 == 1 || (w & 1) == 0) && ow < k.Wo && oh < k.Ho)
            store_elems<DT, VEC>(outp, (uint32_t)(oh * k.Wo + ow) * out_pitch + c0, y);
    };
    // first row of the plane between the poolings / of the input that output row t adds
    auto new_l1 = [&](int32_t t) { return (oh0 + t - 1) * S2 - P + K; };
    auto new_l0 = [&](int32_t t) { return new_l1(t) + 1; };
    // One output row, and the windows slid down to the next: its new input rows are requested before this row is
    // reduced and used after; the store comes last (see pool_xrows2_kernel on how this shapes the compiler's waits).
    auto step = [&](int32_t t) {
        Row nr[NS];
        const int32_t r1n = new_l1(t + 1), h0n = new_l0(t + 1);
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            nr[j] = fetch(h0n + j);
            row_sync();
        }
        float y[VEC];
        reduce(y);
#pragma unroll
        for (int j = 0; j < KEEP1; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) win1[j][e] = win1[j + S2][e];
        float l0[2 + NS][VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            l0[0][e] = keep0[0][e];
            l0[1][e] = keep0[1][e];
        }
#pragma unroll
        for (int j = 0; j < NS; ++j) settle(nr[j], h0n + j, l0[2 + j]);
#pragma unroll
        for (int j = 0; j < S2; ++j) level1(r1n + j, l0[j], l0[j + 1], l0[j + 2], win1[KEEP1 + j]);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            keep0[0][e] = l0[NS][e];
            keep0[1][e] = l0[NS + 1][e];
        }
        put(t, y);
    };
    auto last = [&](int32_t t) {
        float y[VEC];
        reduce(y);
        put(t, y);
    };
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): nothing in flight at the loop's head
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

// signatures compiled in: (first pooling, stride of the second, list codes in front / behind); nothing between the poolings
constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE;
constexpr int BN_RELU_TWICE = BN_RELU + BN_RELU * K_EW_BASE * K_EW_BASE;

template <int DT, int VEC, int KIND1, int S2, int EW0, int EW2>
bool try_launch(const NhwcTile2K &k, int32_t c0, int32_t c2, dim3 grid, dim3 block, hipStream_t st)
{
    if (k.pool1.kind != KIND1 || k.pool2.sh != S2 || c0 != EW0 || c2 != EW2) return false;
    nhwc_rows2_kernel<DT, VEC, KIND1, OP_MAXPOOL, S2, EW0, 0, EW2><<<grid, block, 0, st>>>(k);
    return true;
}

template <int DT, int VEC, int KIND1, int S2>
bool launch_lists(const NhwcTile2K &k, int32_t c0, int32_t c2, dim3 grid, dim3 block, hipStream_t st)
{
    if constexpr (KIND1 == OP_AVGSUM) {
        return try_launch<DT, VEC, KIND1, S2, BN_RELU, BN_RELU>(k, c0, c2, grid, block, st) ||
               try_launch<DT, VEC, KIND1, S2, BN_RELU, 0>(k, c0, c2, grid, block, st) ||
               try_launch<DT, VEC, KIND1, S2, 0, BN_RELU>(k, c0, c2, grid, block, st) ||
               try_launch<DT, VEC, KIND1, S2, 0, 0>(k, c0, c2, grid, block, st);
    } else {  // lists in front of a maximum have moved behind it
        return try_launch<DT, VEC, KIND1, S2, 0, BN_RELU>(k, c0, c2, grid, block, st) ||
               try_launch<DT, VEC, KIND1, S2, 0, BN_RELU_TWICE>(k, c0, c2, grid, block, st) ||
               try_launch<DT, VEC, KIND1, S2, 0, 0>(k, c0, c2, grid, block, st);
    }
}

template <int DT, int VEC>
bool launch_t(const NhwcTile2K &k, dim3 grid, dim3 block, hipStream_t st)
{
    const int32_t c0 = rows_ew_code(k.pre, k.n_pre), c2 = rows_ew_code(k.post, k.n_post);
    return launch_lists<DT, VEC, OP_AVGSUM, 1>(k, c0, c2, grid, block, st) || launch_lists<DT, VEC, OP_AVGSUM, 2>(k, c0, c2, grid, block, st) ||
           launch_lists<DT, VEC, OP_MAXPOOL, 1>(k, c0, c2, grid, block, st) || launch_lists<DT, VEC, OP_MAXPOOL, 2>(k, c0, c2, grid, block, st);
}

bool lists_compiled(const NhwcTile2K &k)
{
    const int32_t c0 = rows_ew_code(k.pre, k.n_pre), c2 = rows_ew_code(k.post, k.n_post);
    if (k.n_mid != 0) return false;
    if (k.pool1.kind == OP_AVGSUM) return (c0 == BN_RELU || c0 == 0) && (c2 == BN_RELU || c2 == 0);
    return c0 == 0 && (c2 == BN_RELU || c2 == BN_RELU_TWICE || c2 == 0);
}

}  // namespace

// Is this pair of pooling steps (lists already in the places plan_nhwc_tile2 gives them) one the kernel is compiled for?
bool nhwc_rows2_supported(const NhwcTile2K &k, int32_t dtype)
{
    // 16-bit storage only.  Measured on MI355X (halo_stress, us): bfloat16 57 against the tile kernel's 86, binary16 55
    // against 83, float32 (eight waves per work-group) 91 against 77.
    if (dtype != BS_BF16 && dtype != BS_F16) return false;
    const PoolK &a = k.pool1, &b = k.pool2;
    auto is3p1 = [](const PoolK &p) { return p.kh == 3 && p.kw == 3 && p.ph == 1 && p.pw == 1 && p.sh == p.sw; };
    if (!is3p1(a) || !is3p1(b) || a.sh != 1 || (b.sh != 1 && b.sh != 2)) return false;
    if ((a.kind != OP_MAXPOOL && a.kind != OP_AVGSUM) || b.kind != OP_MAXPOOL || b.idx_slot >= 0 || a.idx_slot >= 0) return false;
    if (a.kind == OP_AVGSUM && a.count_include_pad != 1) return false;
    if (k.W < 1 || k.W > 64 || k.H1 != k.H || k.W1 != k.W) return false;
    if (k.Ho != (k.H1 + 2 - 3) / b.sh + 1 || k.Wo != (k.W1 + 2 - 3) / b.sw + 1) return false;  // floor mode
    return lists_compiled(k);
}

bs_status launch_nhwc_rows2(const NhwcTile2K &k, int32_t dtype, int32_t vec, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t full = dtype == BS_F32 ? 4 : 8;
    // what the kernel assumes of its argument block: whole channel vectors, one wave per vector of the group, a grid
    // that is exactly groups x chunks x images, chunks that cover the output rows
    if (vec != full || k.C % vec != 0 || !nhwc_rows2_supported(k, dtype)) return BS_ERR_UNSUPPORTED;
    const int32_t cvn = k.C / vec;
    if (k.cvb < 1 || k.cvb > K_NHWC_ROWS_WAVES || cvn % k.cvb != 0 || k.cvgs != cvn / k.cvb || threads != 64 * k.cvb) return BS_ERR_UNSUPPORTED;
    if (k.rc < 1 || k.chunks < 1 || (int64_t)k.chunks * k.rc < k.Ho || k.div_cvgs.d != (uint32_t)k.cvgs ||
        k.div_chunks.d != (uint32_t)k.chunks)
        return BS_ERR_UNSUPPORTED;
    // exactly one work-group per (image, chunk, group); images addressed with 32-bit offsets
    if (grid_n != (int64_t)k.div_n.d * k.chunks * k.cvgs || grid_n > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    if (!nhwc_tile2_sizes_ok(k.H, k.W, k.C, k.in_xp, dtype) || !nhwc_tile2_sizes_ok(k.Ho, k.Wo, k.C, k.out_xp, dtype))
        return BS_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    bool ok = false;
    if (dtype == BS_BF16) ok = launch_t<DT_BF16, 8>(k, grid, block, st);
    else if (dtype == BS_F16) ok = launch_t<DT_F16, 8>(k, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
