// HIP kernels (gfx950 / CDNA4, wave64) for depth-first execution of a sequence of
// steps, and their launchers.
//
// Three kernel families, following the two code-generation cases of Section 4.1
// (single-step sequence: values pass from operation to operation directly;
// multi-step sequence: cached buffer + synchronisation between steps) and the GPU
// building blocks of Section 4.4 (element-wise; non-stacked pooling; stacked
// pooling with two on-chip buffers swapped after each step):
//
//   stream_kernel       element-wise only.  128-bit loads/stores, everything in
//                       registers.
//   pool_direct_kernel  one pooling operation with disjoint windows (k == s, p == 0)
//                       plus element-wise operations before and after it.  Each lane
//                       owns whole windows: KH 128-bit row loads give VEC/KW outputs.
//   lds_tile_kernel     any sequence with pooling: a work-group takes a tile of the
//                       final output, loads the input region it depends on (tile +
//                       halo) into LDS, and runs step after step between two LDS
//                       buffers with a barrier in between; halo cells are recomputed
//                       per tile (Section 5.1 discusses this overlap).
//
// Arithmetic is float32 with one fixed operation order per layer so that results do
// not depend on the tiling: BatchNorm is one fused multiply-add with host-folded
// scale/shift, the average's sum runs row-major over the in-range cells from +0 and is
// multiplied by a float32 reciprocal, max takes the first maximum in row-major order.
// With bfloat16 storage every layer's output is rounded to bfloat16 (nearest-even).
// No MFMA: the path moves 5..12 bytes per element and does ~10 flops on them.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "bs_internal.h"

namespace bs {

#define BS_DEV __device__ __forceinline__

BS_DEV uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    return f.d == 1 ? n : (__umulhi(n, f.mul) >> f.shift);
}

// ------------------------------------------------------------------ bfloat16
BS_DEV float bf16_round(float f)
{
    // round-to-nearest-even through the compiler's bfloat16 type (v_cvt_pk_bf16_f32)
    return (float)(__bf16)f;
}
BS_DEV uint16_t bf16_bits(float f)
{
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}
BS_DEV float bf16_up(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <bool BF16>
BS_DEV float round_store(float v)
{
    if constexpr (BF16) return bf16_round(v);
    else return v;
}

// --------------------------------------------------------- vector load/store
// Raw register block of N consecutive elements (2, 4, 8 or 16 bytes, one load instruction).
template <int BYTES>
struct RawT;
template <>
struct RawT<16> { using type = uint4; };
template <>
struct RawT<8> { using type = uint2; };
template <>
struct RawT<4> { using type = uint32_t; };
template <>
struct RawT<2> { using type = uint16_t; };

template <bool BF16, int N>
struct Raw {
    using type = typename RawT<N * (BF16 ? 2 : 4)>::type;
    type q;
};

template <bool BF16, int N>
BS_DEV Raw<BF16, N> load_raw(const void *base, uint32_t elem)
{
    using T = typename Raw<BF16, N>::type;
    Raw<BF16, N> r;
    r.q = *reinterpret_cast<const T *>(static_cast<const char *>(base) + (size_t)elem * (BF16 ? 2 : 4));
    return r;
}

template <bool BF16, int N>
BS_DEV void unpack(const Raw<BF16, N> &r, float (&v)[N])
{
    constexpr int BYTES = N * (BF16 ? 2 : 4);
    if constexpr (BYTES == 2) {
        v[0] = __uint_as_float((uint32_t)r.q << 16);
    } else {
        constexpr int WORDS = BYTES / 4;
        uint32_t w[WORDS];
        if constexpr (BYTES == 16) { w[0] = r.q.x; w[1] = r.q.y; w[2] = r.q.z; w[3] = r.q.w; }
        else if constexpr (BYTES == 8) { w[0] = r.q.x; w[1] = r.q.y; }
        else w[0] = r.q;
        if constexpr (!BF16) {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) v[i] = __uint_as_float(w[i]);
        } else {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) {
                v[2 * i] = __uint_as_float(w[i] << 16);
                v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        }
    }
}

// Store N consecutive elements (N * element size is 2, 4, 8 or 16 bytes, naturally aligned).
template <bool BF16, int N>
BS_DEV void store_elems(void *base, uint32_t elem, const float (&v)[N])
{
    if constexpr (!BF16) {
        float *p = static_cast<float *>(base) + elem;
        if constexpr (N == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
        else if constexpr (N == 2) *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
        else {
#pragma unroll
            for (int i = 0; i < N; ++i) p[i] = v[i];
        }
    } else {
        uint16_t *p = static_cast<uint16_t *>(base) + elem;
        if constexpr (N == 8 || N == 4 || N == 2) {
            uint32_t w[N / 2];
#pragma unroll
            for (int i = 0; i < N / 2; ++i)
                w[i] = (uint32_t)bf16_bits(v[2 * i]) | ((uint32_t)bf16_bits(v[2 * i + 1]) << 16);
            if constexpr (N == 8) *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
            else if constexpr (N == 4) *reinterpret_cast<uint2 *>(p) = make_uint2(w[0], w[1]);
            else *reinterpret_cast<uint32_t *>(p) = w[0];
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) p[i] = bf16_bits(v[i]);
        }
    }
}

// ------------------------------------------------------ element-wise operations
// Apply a list of element-wise operations to U register vectors at once (the list is
// wave-uniform, so its interpretation costs scalar instructions only).
//   c[u]    channel of vector u (BatchNorm parameters)
//   off[u]  element offset of vector u in this level's tensors (residual loads)
template <bool BF16, int VEC, int U>
BS_DEV void apply_ew(float (&x)[U][VEC], const bool (&valid)[U], const int32_t (&c)[U],
                     const uint32_t (&off)[U], const EwOp *ew, int32_t n_ew, const float *params,
                     int32_t C, const void *const *res)
{
    for (int32_t j = 0; j < n_ew; ++j) {
        const int32_t kind = ew[j].kind, arg = ew[j].arg;
        if (kind == OP_BN) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!valid[u]) continue;
                const float sc = params[arg + c[u]], sh = params[arg + C + c[u]];
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<BF16>(__builtin_fmaf(x[u][i], sc, sh));
            }
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = x[u][i] > 0.0f ? x[u][i] : 0.0f;
        } else {  // OP_ADD
            const void *rp = res[arg];
            Raw<BF16, VEC> rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (valid[u]) rr[u] = load_raw<BF16, VEC>(rp, off[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!valid[u]) continue;
                float r[VEC];
                unpack<BF16, VEC>(rr[u], r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<BF16>(x[u][i] + r[i]);
            }
        }
    }
}

// =============================================================================
// stream_kernel: element-wise only sequence.
// =============================================================================
template <bool BF16, int VEC>
__global__ __launch_bounds__(512) void stream_kernel(const StreamK k)
{
    constexpr int U = 4;
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    Raw<BF16, VEC> raw[U];
    bool valid[U];
    uint32_t off[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        off[u] = i * VEC;
        if (valid[u]) raw[u] = load_raw<BF16, VEC>(k.in, off[u]);
    }
    float x[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = base + u * nthr;
        const uint32_t plane = fdiv(i, k.div_plane);
        c[u] = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);
        if (valid[u]) unpack<BF16, VEC>(raw[u], x[u]);
        else {
            c[u] = 0;
#pragma unroll
            for (int i2 = 0; i2 < VEC; ++i2) x[u][i2] = 0.0f;
        }
    }
    apply_ew<BF16, VEC, U>(x, valid, c, off, k.ew, k.n_ew, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (valid[u]) store_elems<BF16, VEC>(k.out, off[u], x[u]);
}

// =============================================================================
// pool_direct_kernel: [element-wise]* pool(k == s, p == 0) [element-wise]*,
// windows disjoint, one 128-bit column block (VEC input columns) per unit.
// unit = (plane, output row oh, column block cv); it reads KH rows x VEC columns and
// produces VEC / KW outputs.
// =============================================================================
template <bool BF16, int VEC, int KH, int KW>
__global__ __launch_bounds__(512) void pool_direct_kernel(const PoolDirectK k)
{
    constexpr int U = 2;
    constexpr int NO = VEC / KW;  // outputs per unit
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t wv = k.div_wv.d;

    Raw<BF16, VEC> raw[U][KH];
    bool valid[U];
    uint32_t in_off[U], out_off[U], oh[U], cv[U], plane[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        const uint32_t t = fdiv(i, k.div_wv);
        cv[u] = i - t * wv;
        plane[u] = fdiv(t, k.div_ho);
        oh[u] = t - plane[u] * (uint32_t)k.Ho;
        c[u] = (int32_t)(plane[u] - fdiv(plane[u], k.div_c) * (uint32_t)k.C);
        in_off[u] = (plane[u] * (uint32_t)k.H + oh[u] * KH) * (uint32_t)k.W + cv[u] * VEC;
        out_off[u] = (plane[u] * (uint32_t)k.Ho + oh[u]) * (uint32_t)k.Wo + cv[u] * NO;
        if (!valid[u]) c[u] = 0;
#pragma unroll
        for (int dh = 0; dh < KH; ++dh)
            if (valid[u]) raw[u][dh] = load_raw<BF16, VEC>(k.in, in_off[u] + dh * (uint32_t)k.W);
    }

    float y[U][NO];
    int32_t yi[U][NO];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float x[KH][VEC];
        bool v1[KH];
        int32_t c1[KH];
        uint32_t o1[KH];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) {
            v1[dh] = valid[u];
            c1[dh] = c[u];
            o1[dh] = in_off[u] + dh * (uint32_t)k.W;
            if (valid[u]) unpack<BF16, VEC>(raw[u][dh], x[dh]);
            else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[dh][i] = 0.0f;
            }
        }
        apply_ew<BF16, VEC, KH>(x, v1, c1, o1, k.pre, k.n_pre, k.params, k.C, k.res);
        const bool is_max = k.pool.kind == OP_MAXPOOL;
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            if (is_max) {
                float best = -INFINITY;
                int32_t bi = (int32_t)((oh[u] * KH) * (uint32_t)k.W + cv[u] * VEC + j * KW);
#pragma unroll
                for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) {
                        const float v = x[dh][j * KW + dw];
                        const bool g = v > best;
                        best = g ? v : best;
                        bi = g ? (int32_t)((oh[u] * KH + dh) * (uint32_t)k.W + cv[u] * VEC + j * KW + dw) : bi;
                    }
                y[u][j] = best;
                yi[u][j] = bi;
            } else {
                float sum = 0.0f;
#pragma unroll
                for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) sum = sum + x[dh][j * KW + dw];
                y[u][j] = round_store<BF16>(sum * k.pool.inv_kk);
                yi[u][j] = 0;
            }
        }
    }
    apply_ew<BF16, NO, U>(y, valid, c, out_off, k.post, k.n_post, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!valid[u]) continue;
        store_elems<BF16, NO>(k.out, out_off[u], y[u]);
        if (k.idx) {
            int32_t *ip = k.idx + out_off[u];
            if constexpr (NO == 4) *reinterpret_cast<int4 *>(ip) = make_int4(yi[u][0], yi[u][1], yi[u][2], yi[u][3]);
            else if constexpr (NO == 2) *reinterpret_cast<int2 *>(ip) = make_int2(yi[u][0], yi[u][1]);
            else {
#pragma unroll
                for (int j = 0; j < NO; ++j) ip[j] = yi[u][j];
            }
        }
    }
}

// =============================================================================
// lds_tile_kernel: depth-first execution of a multi-step (or overlapping-window)
// sequence on one tile per work-group.
//
// Levels: level 0 is the sequence input, pooling operation l (1..L) turns level l-1
// into level l.  A work-group owns PPG planes x the tile [th*TH, +TH) x [tw*TW, +TW)
// of level L.  The region of level l-1 it needs is found by walking the windows of
// pooling operation l backwards and clipping to the plane: cells outside the plane are
// that operation's padding (never a max candidate, nothing added to a sum) and are
// neither loaded nor computed.  Level l (l < L) lives in LDS buffer l & 1.
// =============================================================================
template <bool BF16, int VEC>
__global__ __launch_bounds__(512) void lds_tile_kernel(const LdsSeqK k)
{
    extern __shared__ float lds[];
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const int32_t L = k.n_levels;

    // work-group -> (plane group, tile row, tile column)
    const uint32_t pg = fdiv(blockIdx.x, k.div_tiles_hw);
    const uint32_t trem = blockIdx.x - pg * (uint32_t)(k.tiles_h * k.tiles_w);
    const int32_t ti = (int32_t)fdiv(trem, k.div_tiles_w);
    const int32_t tj = (int32_t)(trem - (uint32_t)ti * (uint32_t)k.tiles_w);
    const int32_t plane0 = (int32_t)pg * k.PPG;
    const int32_t nplanes = min(k.PPG, k.NC - plane0);

    // ---------------- phase 0: load the level-0 region, apply its element-wise ops ----
    {
        const LevelK &lv = k.level[0];
        const Region g = region_at(k, ti, tj, 0);
        const int32_t rh = g.r_hi - g.r_lo, rwv = (g.c_hi - g.c_lo) / VEC;
        const uint32_t pitchv = (uint32_t)lv.pitch / VEC;
        const uint32_t planev = (uint32_t)lv.plane_stride / VEC;
        const uint32_t items = (uint32_t)k.PPG * planev;
        float *dst = lds + lv.buf_off;
        constexpr int U = 4;
        for (uint32_t base = tid; base < items; base += nthr * U) {
            Raw<BF16, VEC> raw[U];
            bool valid[U];
            uint32_t off[U], loff[U];
            int32_t c[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t i = base + u * nthr;
                const uint32_t pl = fdiv(i, lv.div_plane);
                const uint32_t rem = i - pl * planev;
                const uint32_t r = fdiv(rem, lv.div_pitch);
                const uint32_t cvv = rem - r * pitchv;
                valid[u] = i < items && (int32_t)pl < nplanes && (int32_t)r < rh && (int32_t)cvv < rwv;
                const uint32_t plane = (uint32_t)plane0 + pl;
                c[u] = valid[u] ? (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C) : 0;
                off[u] = (plane * (uint32_t)lv.H + (uint32_t)g.r_lo + r) * (uint32_t)lv.W + (uint32_t)g.c_lo + cvv * VEC;
                loff[u] = pl * (uint32_t)lv.plane_stride + r * (uint32_t)lv.pitch + cvv * VEC;
                if (valid[u]) raw[u] = load_raw<BF16, VEC>(k.in, off[u]);
            }
            float x[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (valid[u]) unpack<BF16, VEC>(raw[u], x[u]);
                else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) x[u][i] = 0.0f;
                }
            }
            apply_ew<BF16, VEC, U>(x, valid, c, off, lv.ew, lv.n_ew, k.params, k.C, k.res);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!valid[u]) continue;
                if constexpr (VEC >= 4) {
#pragma unroll
                    for (int h = 0; h < VEC / 4; ++h)
                        *reinterpret_cast<float4 *>(dst + loff[u] + 4 * h) =
                            make_float4(x[u][4 * h], x[u][4 * h + 1], x[u][4 * h + 2], x[u][4 * h + 3]);
                } else {
                    dst[loff[u]] = x[u][0];
                }
            }
        }
    }
    __syncthreads();

    // ---------------- phases 1..L: one pooling operation each -------------------------
    for (int32_t l = 1; l <= L; ++l) {
        const LevelK &lv = k.level[l];
        const LevelK &pv = k.level[l - 1];
        const PoolK &p = k.pool[l];
        const Region g = region_at(k, ti, tj, l);
        const Region pgn = region_at(k, ti, tj, l - 1);
        const int32_t rh = g.r_hi - g.r_lo, rw = g.c_hi - g.c_lo;
        const float *src = lds + pv.buf_off;
        float *dst = lds + lv.buf_off;
        const bool last = (l == L);
        const bool is_max = p.kind == OP_MAXPOOL;
        int32_t *idxp = p.idx_slot >= 0 ? k.idx[p.idx_slot] : nullptr;
        // cells of this level the tile owns for index output: up to where the next tile's
        // region starts (regions overlap by the halo; each cell is written once)
        int32_t own_r_hi = g.r_hi, own_c_hi = g.c_hi;
        if (idxp && !last) {
            own_r_hi = (ti + 1 < k.tiles_h) ? region_at(k, ti + 1, tj, l).r_lo : lv.H;
            own_c_hi = (tj + 1 < k.tiles_w) ? region_at(k, ti, tj + 1, l).c_lo : lv.W;
        }
        const uint32_t items = (uint32_t)k.PPG * (uint32_t)lv.plane_stride;
        for (uint32_t i = tid; i < items; i += nthr) {
            const uint32_t pl = fdiv(i, lv.div_plane);
            const uint32_t rem = i - pl * (uint32_t)lv.plane_stride;
            const uint32_t r = fdiv(rem, lv.div_pitch);
            const uint32_t cc = rem - r * (uint32_t)lv.pitch;
            if ((int32_t)pl >= nplanes || (int32_t)r >= rh || (int32_t)cc >= rw) continue;
            const uint32_t plane = (uint32_t)plane0 + pl;
            const int32_t oh = g.r_lo + (int32_t)r, ow = g.c_lo + (int32_t)cc;
            const int32_t h0 = oh * p.sh - p.ph, w0 = ow * p.sw - p.pw;
            const int32_t hs = max(h0, 0), he = min(h0 + p.kh, pv.H);
            const int32_t ws = max(w0, 0), we = min(w0 + p.kw, pv.W);
            const float *sp = src + pl * (uint32_t)pv.plane_stride + (hs - pgn.r_lo) * pv.pitch + (ws - pgn.c_lo);
            float val;
            if (is_max) {
                float best = -INFINITY;
                int32_t bi = hs * pv.W + ws;
                for (int32_t ih = hs; ih < he; ++ih) {
                    for (int32_t iw = ws; iw < we; ++iw) {
                        const float v = sp[iw - ws];
                        const bool gt = v > best;
                        best = gt ? v : best;
                        bi = gt ? ih * pv.W + iw : bi;
                    }
                    sp += pv.pitch;
                }
                val = best;
                if (idxp && oh < own_r_hi && ow < own_c_hi)
                    idxp[(plane * (uint32_t)lv.H + (uint32_t)oh) * (uint32_t)lv.W + (uint32_t)ow] = bi;
            } else {
                float sum = 0.0f;
                for (int32_t ih = hs; ih < he; ++ih) {
                    for (int32_t iw = ws; iw < we; ++iw) sum = sum + sp[iw - ws];
                    sp += pv.pitch;
                }
                const float inv = p.count_include_pad ? p.inv_kk : 1.0f / (float)((he - hs) * (we - ws));
                val = round_store<BF16>(sum * inv);
            }
            // element-wise operations attached to this level
            float x[1][1] = {{val}};
            const bool v1[1] = {true};
            const int32_t c1[1] = {(int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C)};
            const uint32_t o1[1] = {(plane * (uint32_t)lv.H + (uint32_t)oh) * (uint32_t)lv.W + (uint32_t)ow};
            apply_ew<BF16, 1, 1>(x, v1, c1, o1, lv.ew, lv.n_ew, k.params, k.C, k.res);
            if (last) {
                store_elems<BF16, 1>(k.out, o1[0], x[0]);
            } else {
                dst[pl * (uint32_t)lv.plane_stride + r * (uint32_t)lv.pitch + cc] = x[0][0];
            }
        }
        if (!last) __syncthreads();
    }
}

// =============================================================================
// Host side: device queries, parameter upload, launchers.
// =============================================================================
static bs_status hip_fail(hipError_t e)
{
    set_hip_error((int32_t)e);
    (void)hipGetLastError();
    return BS_ERR_HIP;
}

bs_status device_limits(Limits *lim, int *device)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e);
    int smem = 0;
    e = hipDeviceGetAttribute(&smem, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return hip_fail(e);
    lim->num_cus = cus;
    lim->max_lds_bytes = (uint64_t)smem;
    *device = dev;
    return BS_OK;
}

bs_status upload_params(bs_stack *s)
{
    free_params(s);
    if (s->host_params.empty()) return BS_OK;
    const size_t bytes = s->host_params.size() * sizeof(float);
    float *d = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&d), bytes);
    if (e != hipSuccess) return hip_fail(e);
    // synchronous copy from pageable memory: complete when it returns
    e = hipMemcpy(d, s->host_params.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(d);
        return hip_fail(e);
    }
    s->dev_params = d;
    return BS_OK;
}

void free_params(bs_stack *s)
{
    if (s->dev_params) {
        (void)hipFree(s->dev_params);
        s->dev_params = nullptr;
    }
}

template <bool BF16, int VEC, int KH>
static void launch_direct_kw(const PoolDirectK &k, int kw, dim3 grid, dim3 block, hipStream_t st)
{
    if constexpr (VEC == 8) {
        if (kw == 8) { pool_direct_kernel<BF16, VEC, KH, 8><<<grid, block, 0, st>>>(k); return; }
    }
    if (kw == 1) pool_direct_kernel<BF16, VEC, KH, 1><<<grid, block, 0, st>>>(k);
    else if (kw == 2) pool_direct_kernel<BF16, VEC, KH, 2><<<grid, block, 0, st>>>(k);
    else pool_direct_kernel<BF16, VEC, KH, 4><<<grid, block, 0, st>>>(k);
}

template <bool BF16, int VEC>
static void launch_direct(const PoolDirectK &k, dim3 grid, dim3 block, hipStream_t st)
{
    switch (k.pool.kh) {
    case 1: launch_direct_kw<BF16, VEC, 1>(k, k.pool.kw, grid, block, st); break;
    case 2: launch_direct_kw<BF16, VEC, 2>(k, k.pool.kw, grid, block, st); break;
    case 3: launch_direct_kw<BF16, VEC, 3>(k, k.pool.kw, grid, block, st); break;
    default: launch_direct_kw<BF16, VEC, 4>(k, k.pool.kw, grid, block, st); break;
    }
}

bs_status launch_sequence(const bs_stack *s, const Sequence &q, const void *in, void *out,
                          const void *const *res, int32_t *const *idx, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = s->dtype == BS_BF16;
    if (q.grid < 1 || q.grid > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)q.grid), block((uint32_t)q.threads);
    const void *rp[K_MAX_RES] = {nullptr, nullptr, nullptr, nullptr};
    for (int32_t j = 0; j < q.n_res; ++j) rp[j] = res[q.res_map[j]];
    int32_t *ip[K_MAX_IDX] = {nullptr, nullptr, nullptr, nullptr};
    for (int32_t j = 0; j < q.n_idx; ++j) ip[j] = idx ? idx[q.idx_map[j]] : nullptr;

    switch (q.variant) {
    case BS_VARIANT_STREAM: {
        StreamK k = q.stream;
        k.in = in; k.out = out; k.params = s->dev_params;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        if (bf16) {
            if (q.vec == 8) stream_kernel<true, 8><<<grid, block, 0, st>>>(k);
            else stream_kernel<true, 1><<<grid, block, 0, st>>>(k);
        } else {
            if (q.vec == 4) stream_kernel<false, 4><<<grid, block, 0, st>>>(k);
            else stream_kernel<false, 1><<<grid, block, 0, st>>>(k);
        }
        break;
    }
    case BS_VARIANT_POOL_DIRECT: {
        PoolDirectK k = q.direct;
        k.in = in; k.out = out; k.params = s->dev_params;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        k.idx = ip[0];
        if (bf16) launch_direct<true, 8>(k, grid, block, st);
        else launch_direct<false, 4>(k, grid, block, st);
        break;
    }
    case BS_VARIANT_LDS_TILE: {
        LdsSeqK k = q.lds;
        k.in = in; k.out = out; k.params = s->dev_params;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        for (int j = 0; j < K_MAX_IDX; ++j) k.idx[j] = ip[j];
        const size_t lds = (size_t)q.lds_bytes;
        if (bf16) {
            if (q.vec == 8) lds_tile_kernel<true, 8><<<grid, block, lds, st>>>(k);
            else lds_tile_kernel<true, 1><<<grid, block, lds, st>>>(k);
        } else {
            if (q.vec == 4) lds_tile_kernel<false, 4><<<grid, block, lds, st>>>(k);
            else lds_tile_kernel<false, 1><<<grid, block, lds, st>>>(k);
        }
        break;
    }
    default:
        return BS_ERR_UNSUPPORTED;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return BS_OK;
}

}  // namespace bs
