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
// Apply a list of element-wise operations to U register vectors at once.  The list is
// wave-uniform, so interpreting it costs scalar instructions only.  Lanes that have no
// work carry c = 0 / off = 0 (safe addresses) and simply compute values nobody stores:
// no load here is predicated.
//   c[u]    channel of vector u (BatchNorm parameters)
//   off[u]  element offset of vector u in this level's tensors (residual loads)
template <bool BF16, int VEC, int U>
BS_DEV void apply_ew(float (&x)[U][VEC], const int32_t (&c)[U], const uint32_t (&off)[U],
                     const EwOp *ew, int32_t n_ew, const float *__restrict__ params, int32_t C,
                     const void *const *res)
{
#pragma clang loop unroll(disable)
    for (int32_t j = 0; j < n_ew; ++j) {
        const int32_t kind = ew[j].kind, arg = ew[j].arg;
        if (kind == OP_BN) {
            float sc[U], sh[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                sc[u] = params[arg + c[u]];
                sh[u] = params[arg + C + c[u]];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<BF16>(__builtin_fmaf(x[u][i], sc[u], sh[u]));
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = __builtin_fmaxf(x[u][i], 0.0f);  // NaN, -0 -> +0
        } else {  // OP_ADD
            const void *rp = res[arg];
            Raw<BF16, VEC> rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) rr[u] = load_raw<BF16, VEC>(rp, off[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float r[VEC];
                unpack<BF16, VEC>(rr[u], r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<BF16>(x[u][i] + r[i]);
            }
        }
    }
}

// =============================================================================
// stream_kernel: element-wise only sequence.  A work-group takes nthr * U
// consecutive 128-bit vectors; lane t handles vectors t, t + nthr, ...
// =============================================================================
template <bool BF16, int VEC, int U>
__global__ __launch_bounds__(512) void stream_kernel(const StreamK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    Raw<BF16, VEC> raw[U];
    bool valid[U];
    uint32_t off[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        i = valid[u] ? i : 0u;
        off[u] = i * VEC;
        raw[u] = load_raw<BF16, VEC>(k.in, off[u]);
        const uint32_t plane = fdiv(i, k.div_plane);
        c[u] = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);
    }
    float x[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) unpack<BF16, VEC>(raw[u], x[u]);
    apply_ew<BF16, VEC, U>(x, c, off, k.ew, k.n_ew, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (valid[u]) store_elems<BF16, VEC>(k.out, off[u], x[u]);
}

// =============================================================================
// pool_direct_kernel: [element-wise]* pool(k == s, p == 0) [element-wise]*,
// windows disjoint, one 128-bit column block (VEC input columns) per unit.
// unit = (plane, output row oh, column block cv); it reads KH rows x VEC columns and
// produces VEC / KW outputs.  Consecutive lanes take consecutive column blocks, so each
// row load of a wave is one contiguous run.
// =============================================================================
template <bool BF16, int VEC, int KH, int KW, int U>
__global__ __launch_bounds__(512) void pool_direct_kernel(const PoolDirectK k)
{
    constexpr int NO = VEC / KW;  // outputs per unit
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t wv = k.div_wv.d;

    Raw<BF16, VEC> raw[U][KH];
    bool valid[U];
    uint32_t in_off[U], out_off[U], idx0[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        i = valid[u] ? i : 0u;
        const uint32_t t = fdiv(i, k.div_wv);
        const uint32_t cv = i - t * wv;
        const uint32_t plane = fdiv(t, k.div_ho);
        const uint32_t oh = t - plane * (uint32_t)k.Ho;
        c[u] = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);
        idx0[u] = (oh * KH) * (uint32_t)k.W + cv * VEC;  // first cell of the unit in its plane
        in_off[u] = plane * (uint32_t)(k.H * k.W) + idx0[u];
        out_off[u] = (plane * (uint32_t)k.Ho + oh) * (uint32_t)k.Wo + cv * NO;
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) raw[u][dh] = load_raw<BF16, VEC>(k.in, in_off[u] + dh * (uint32_t)k.W);
    }

    float y[U][NO];
    int32_t yi[U][NO];
    const bool is_max = k.pool.kind == OP_MAXPOOL;
    const bool want_idx = k.idx != nullptr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float x[KH][VEC];
        int32_t c1[KH];
        uint32_t o1[KH];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) {
            c1[dh] = c[u];
            o1[dh] = in_off[u] + dh * (uint32_t)k.W;
            unpack<BF16, VEC>(raw[u][dh], x[dh]);
        }
        apply_ew<BF16, VEC, KH>(x, c1, o1, k.pre, k.n_pre, k.params, k.C, k.res);
        if (is_max) {
            if (want_idx) {
#pragma unroll
                for (int j = 0; j < NO; ++j) {
                    float best = -INFINITY;
                    int32_t bi = (int32_t)idx0[u] + j * KW;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            const float v = x[dh][j * KW + dw];
                            const bool g = v > best;
                            best = g ? v : best;
                            bi = g ? (int32_t)(idx0[u] + dh * (uint32_t)k.W) + j * KW + dw : bi;
                        }
                    y[u][j] = best;
                    yi[u][j] = bi;
                }
            } else {
#pragma unroll
                for (int j = 0; j < NO; ++j) {
                    float best = -INFINITY;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            best = __builtin_fmaxf(best, x[dh][j * KW + dw]);
                        }
                    y[u][j] = best;
                    yi[u][j] = 0;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NO; ++j) {
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
    apply_ew<BF16, NO, U>(y, c, out_off, k.post, k.n_post, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!valid[u]) continue;
        store_elems<BF16, NO>(k.out, out_off[u], y[u]);
        if (want_idx && is_max) {
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
// sequence, one tile per work-group.
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
// LDS buffer l & 1; a barrier separates the phases (Section 4.4's two-buffer scheme).
//
// Lane grid.  In every phase the work-group's lanes form a ct x rt grid (one division per
// lane per phase): ct lanes along a row, rt rows in flight; a lane keeps its column and
// walks down the rows, so all column arithmetic and predicates are loop-invariant and the
// plane (hence the BatchNorm channel) is uniform per iteration: folded parameters are read
// with scalar loads.
//
// Phase 0 loads 128-bit global vectors and stores them with one 128-bit LDS write each,
// after the level-0 element-wise operations: the level-0 LDS row starts at the global
// vector that contains the rectangle's first column (D = delta0 columns earlier).
// Phase l gives each lane a strip of four horizontally adjacent outputs: it reads the
// kh rows x (D + 3*sw + kw) columns it needs with aligned 128/64/32-bit LDS reads and keeps
// the windows in registers.
// =============================================================================
BS_DEV float pad_value(const PoolK &p) { return p.kind == OP_MAXPOOL ? -INFINITY : 0.0f; }

typedef const __attribute__((address_space(4))) float *const_f32_ptr;

// Folded BatchNorm parameters of one level for one (uniform) channel, fetched with scalar loads.
struct EwRegs {
    float sc[K_MAX_EW], sh[K_MAX_EW];
};

BS_DEV void load_ew_regs(const LevelK &lv, const float *params, int32_t C, int32_t c, EwRegs &e)
{
    const_f32_ptr cp = (const_f32_ptr)params;
#pragma unroll
    for (int j = 0; j < K_MAX_EW; ++j) {
        e.sc[j] = 1.0f;
        e.sh[j] = 0.0f;
        if (j < lv.n_ew && lv.ew[j].kind == OP_BN) {
            e.sc[j] = cp[lv.ew[j].arg + c];
            e.sh[j] = cp[lv.ew[j].arg + C + c];
        }
    }
}

// Element-wise operations of a level on N values of one plane.  contiguous: the N values are
// consecutive elements starting at off[0] (one vector residual load); else off[i] each.
template <bool BF16, int N, bool CONTIG>
BS_DEV void apply_level_ew(float (&x)[N], const LevelK &lv, const EwRegs &er, const void *const *res,
                           const uint32_t (&off)[CONTIG ? 1 : N])
{
#pragma unroll
    for (int j = 0; j < K_MAX_EW; ++j) {
        if (j >= lv.n_ew) break;
        const int32_t kind = lv.ew[j].kind;
        if (kind == OP_BN) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<BF16>(__builtin_fmaf(x[i], er.sc[j], er.sh[j]));
        } else if (kind == OP_RELU) {
            // v_max_f32: NaN -> 0, and max(-0, +0) = +0 in either operand order
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = __builtin_fmaxf(x[i], 0.0f);
        } else {
            const void *rp = res[lv.ew[j].arg];
            float r[N];
            if constexpr (CONTIG) {
                const Raw<BF16, N> rr = load_raw<BF16, N>(rp, off[0]);
                unpack<BF16, N>(rr, r);
            } else {
#pragma unroll
                for (int i = 0; i < N; ++i) {
                    const Raw<BF16, 1> rr = load_raw<BF16, 1>(rp, off[i]);
                    float one[1];
                    unpack<BF16, 1>(rr, one);
                    r[i] = one[0];
                }
            }
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = round_store<BF16>(x[i] + r[i]);
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

// One strip of four outputs of pooling operation p from the cached level below.
//   src      16-byte aligned LDS address; the strip's first window starts D floats after it
//   h0, w0   global row / column of the first window's first cell in the input plane (may be
//            negative: padding)
// KH/KW/SW > 0: compile-time window and stride (D < 4); KH == 0: run-time shape, scalar reads.
template <int KH, int KW, int SW, int D, bool WANT_IDX>
BS_DEV void pool_strip(const PoolK &p, const float *src, int32_t d_rt, int32_t pitch, int32_t h0, int32_t w0,
                       int32_t Hp, int32_t Wp, float (&val)[4], int32_t (&bidx)[4])
{
    const bool is_max = p.kind == OP_MAXPOOL;
    const int32_t kh = KH > 0 ? KH : p.kh, kw = KH > 0 ? KW : p.kw, sw = KH > 0 ? SW : p.sw;
    constexpr int NC = 3 * SW + KW;                           // columns four windows span
    constexpr int NR = KH > 0 ? (D == 0 ? NC : (D + NC + 3) / 4 * 4) : 1;  // floats read per row
    float acc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        acc[e] = is_max ? -INFINITY : 0.0f;
        if constexpr (WANT_IDX) bidx[e] = max(h0, 0) * Wp + max(w0 + e * sw, 0);  // first in-range cell
    }
    if constexpr (KH > 0) {
        float r[KH][NR];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) lds_read_row<NR>(src + dh * pitch, r[dh]);
        if (is_max) {
#pragma unroll
            for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                for (int e = 0; e < 4; ++e)
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
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) acc[e] = acc[e] + r[dh][D + e * SW + dw];
        }
    } else {
        for (int32_t dh = 0; dh < kh; ++dh) {
            const float *rowp = src + dh * pitch + d_rt;
            const int32_t rbase = (h0 + dh) * Wp + w0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
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
    if (is_max) {
#pragma unroll
        for (int e = 0; e < 4; ++e) val[e] = acc[e];
    } else if (p.count_include_pad) {
#pragma unroll
        for (int e = 0; e < 4; ++e) val[e] = acc[e] * p.inv_kk;
    } else {
        const int32_t nr = min(h0 + kh, Hp) - max(h0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t we = w0 + e * sw;
            const int32_t nc = min(we + kw, Wp) - max(we, 0);
            // windows wholly outside the plane can make nr * nc <= 0; such outputs are never stored
            val[e] = acc[e] * (1.0f / (float)max(nr * nc, 1));
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
    int32_t nplanes, plane0;
    bool last, vec_store_ok;
    float padv;
    int32_t *idxp;
};

template <bool BF16, int KH, int KW, int SW, int D, bool WANT_IDX>
BS_DEV void pool_phase(const LdsSeqK &k, const LevelK &lv, const LevelK &pv, const PoolK &p, const PhaseCtx &cx)
{
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t ty = fdiv(tid, lv.div_ct), tx = tid - ty * (uint32_t)lv.ct;
    if ((int32_t)ty >= lv.rt) return;
    const int32_t spr = lv.items_per_row;
    for (int32_t pl = 0; pl < cx.nplanes; ++pl) {
        const uint32_t plane = (uint32_t)(cx.plane0 + pl);
        const int32_t ch = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);
        EwRegs er;
        load_ew_regs(lv, k.params, k.C, ch, er);
        const float *splane = cx.src + pl * pv.plane_stride;
        float *dplane = cx.dst + pl * lv.plane_stride;
        const uint32_t gplane = plane * (uint32_t)(lv.H * lv.W);
        for (int32_t j = (int32_t)tx; j < spr; j += lv.ct) {
            const int32_t gc = cx.c0 + 4 * j;
            const int32_t w0 = gc * p.sw - p.pw;
            // aligned LDS column where this strip's reads start; the first window starts D (or,
            // for run-time shapes, d_rt) floats later
            const int32_t scol = 4 * j * p.sw + (KH > 0 ? (cx.d_lo - D) : 0);
            const int32_t d_rt = KH > 0 ? 0 : cx.d_lo;
            bool cin[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) cin[e] = gc + e >= 0 && gc + e < lv.W;
            const bool strip_vec = cx.vec_store_ok && gc >= 0 && gc + 3 < cx.end_c;
            for (int32_t r = (int32_t)ty; r < lv.rows; r += lv.rt) {
                const int32_t gr = cx.r0 + r;
                const int32_t h0 = gr * p.sh - p.ph;
                float val[4];
                int32_t bi[4] = {0, 0, 0, 0};
                pool_strip<KH, KW, SW, D, WANT_IDX>(p, splane + (r * p.sh) * pv.pitch + scol, d_rt, pv.pitch, h0, w0,
                                                    pv.H, pv.W, val, bi);
                if (p.kind != OP_MAXPOOL) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) val[e] = round_store<BF16>(val[e]);
                }
                const bool row_in = gr >= 0 && gr < lv.H;
                const uint32_t goff = gplane + (uint32_t)(row_in ? gr : 0) * (uint32_t)lv.W;
                if constexpr (WANT_IDX) {
                    if (row_in && gr < cx.end_r) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (gc + e >= 0 && gc + e < cx.end_c) cx.idxp[goff + (uint32_t)(gc + e)] = bi[e];
                    }
                }
                if (lv.n_ew > 0) {
                    uint32_t o4[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (row_in && cin[e]) ? goff + (uint32_t)(gc + e) : 0u;
                    apply_level_ew<BF16, 4, false>(val, lv, er, k.res, o4);
                }
                if (cx.last) {
                    if (row_in && gr < cx.end_r) {
                        if (strip_vec) {
                            store_elems<BF16, 4>(k.out, goff + (uint32_t)gc, val);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (gc + e >= 0 && gc + e < cx.end_c) {
                                    const float one[1] = {val[e]};
                                    store_elems<BF16, 1>(k.out, goff + (uint32_t)(gc + e), one);
                                }
                        }
                    }
                } else {
                    float4 w;
                    w.x = (row_in && cin[0]) ? val[0] : cx.padv;
                    w.y = (row_in && cin[1]) ? val[1] : cx.padv;
                    w.z = (row_in && cin[2]) ? val[2] : cx.padv;
                    w.w = (row_in && cin[3]) ? val[3] : cx.padv;
                    *reinterpret_cast<float4 *>(dplane + r * lv.pitch + 4 * j) = w;
                }
            }
        }
    }
    (void)nthr;
}

template <bool BF16, int D, bool WANT_IDX>
BS_DEV void pool_phase_dispatch(const LdsSeqK &k, const LevelK &lv, const LevelK &pv, const PoolK &p,
                                const PhaseCtx &cx)
{
    if (p.kh == 3 && p.kw == 3 && p.sw == 2) pool_phase<BF16, 3, 3, 2, D, WANT_IDX>(k, lv, pv, p, cx);
    else if (p.kh == 3 && p.kw == 3 && p.sw == 1) pool_phase<BF16, 3, 3, 1, D, WANT_IDX>(k, lv, pv, p, cx);
    else if (p.kh == 2 && p.kw == 2 && p.sw == 2) pool_phase<BF16, 2, 2, 2, D, WANT_IDX>(k, lv, pv, p, cx);
    else pool_phase<BF16, 0, 0, 0, 0, WANT_IDX>(k, lv, pv, p, cx);
}

template <bool BF16, int VEC>
__global__ __launch_bounds__(512) void lds_tile_kernel(const LdsSeqK k)
{
    extern __shared__ __align__(16) float lds[];
    const uint32_t tid = threadIdx.x;
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
        int32_t r0 = ti * k.TH, c0 = tj * k.TW;
        for (int32_t l = L; l >= 1; --l) origin_step(k.pool[l], r0, c0);
        const float padv = pad_value(k.pool[1]);
        const int32_t g0 = c0 - k.delta0;  // global column of LDS column 0: a multiple of VEC
        const uint32_t ty = fdiv(tid, lv.div_ct), tx = tid - ty * (uint32_t)lv.ct;
        const bool active = (int32_t)ty < lv.rt;
        constexpr int U = (VEC == 8) ? 2 : 4;
        float *dst = lds + lv.buf_off;
        for (int32_t pl = 0; pl < nplanes && active; ++pl) {
            const uint32_t plane = (uint32_t)(plane0 + pl);
            const int32_t ch = (int32_t)(plane - fdiv(plane, k.div_c) * (uint32_t)k.C);
            EwRegs er;
            load_ew_regs(lv, k.params, k.C, ch, er);
            const uint32_t gplane = plane * (uint32_t)(lv.H * lv.W);
            float *dplane = dst + pl * lv.plane_stride;
            for (int32_t v = (int32_t)tx; v < lv.items_per_row; v += lv.ct) {
                const int32_t gc = g0 + v * VEC;
                const bool col_in = gc >= 0 && gc < lv.W;  // W % VEC == 0: a vector is all in or all out
                for (int32_t rb = (int32_t)ty; rb < lv.rows; rb += lv.rt * U) {
                    Raw<BF16, VEC> raw[U];
                    bool inimg[U];
                    uint32_t off[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int32_t r = rb + u * lv.rt;
                        const int32_t gr = r0 + r;
                        inimg[u] = col_in && r < lv.rows && gr >= 0 && gr < lv.H;
                        off[u] = inimg[u] ? gplane + (uint32_t)gr * (uint32_t)lv.W + (uint32_t)gc : 0u;
                        raw[u] = load_raw<BF16, VEC>(k.in, off[u]);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int32_t r = rb + u * lv.rt;
                        float x[VEC];
                        unpack<BF16, VEC>(raw[u], x);
                        const uint32_t o1[1] = {off[u]};
                        apply_level_ew<BF16, VEC, true>(x, lv, er, k.res, o1);
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
    __syncthreads();

    // ---------------- phases 1..L: one pooling operation each -------------------------
    for (int32_t l = 1; l <= L; ++l) {
        const LevelK &lv = k.level[l];
        const LevelK &pv = k.level[l - 1];
        const PoolK &p = k.pool[l];
        PhaseCtx cx;
        cx.r0 = ti * k.TH;
        cx.c0 = tj * k.TW;
        int32_t step_r = k.TH, step_c = k.TW;  // distance between neighbouring tiles' origins
        for (int32_t m = L; m > l; --m) {
            origin_step(k.pool[m], cx.r0, cx.c0);
            step_r *= k.pool[m].sh;
            step_c *= k.pool[m].sw;
        }
        cx.src = lds + pv.buf_off;
        cx.dst = lds + lv.buf_off;
        cx.last = (l == L);
        cx.padv = cx.last ? 0.0f : pad_value(k.pool[l + 1]);
        cx.idxp = p.idx_slot >= 0 ? k.idx[p.idx_slot] : nullptr;
        // rows / columns of this level the tile may write to memory: its own tile at the last
        // level; elsewhere (index output in the middle of a sequence) up to where the next
        // tile's rectangle starts, so every cell is written exactly once
        const int32_t own_r = (ti + 1 < k.tiles_h) ? cx.r0 + step_r : lv.H;
        const int32_t own_c = (tj + 1 < k.tiles_w) ? cx.c0 + step_c : lv.W;
        cx.end_r = min(own_r, lv.H);
        cx.end_c = min(own_c, lv.W);
        cx.d_lo = (l == 1) ? k.delta0 : 0;
        cx.nplanes = nplanes;
        cx.plane0 = plane0;
        cx.vec_store_ok = cx.last && (lv.W & 3) == 0 && ((k.TW & 3) == 0 || k.tiles_w == 1);
        const int32_t d = cx.d_lo & 3;
        if (cx.idxp) {
            if (d == 0) pool_phase_dispatch<BF16, 0, true>(k, lv, pv, p, cx);
            else if (d == 1) pool_phase_dispatch<BF16, 1, true>(k, lv, pv, p, cx);
            else if (d == 2) pool_phase_dispatch<BF16, 2, true>(k, lv, pv, p, cx);
            else pool_phase_dispatch<BF16, 3, true>(k, lv, pv, p, cx);
        } else {
            if (d == 0) pool_phase_dispatch<BF16, 0, false>(k, lv, pv, p, cx);
            else if (d == 1) pool_phase_dispatch<BF16, 1, false>(k, lv, pv, p, cx);
            else if (d == 2) pool_phase_dispatch<BF16, 2, false>(k, lv, pv, p, cx);
            else pool_phase_dispatch<BF16, 3, false>(k, lv, pv, p, cx);
        }
        if (!cx.last) __syncthreads();
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
        if (kw == 8) { pool_direct_kernel<BF16, VEC, KH, 8, K_DIRECT_U><<<grid, block, 0, st>>>(k); return; }
    }
    if (kw == 1) pool_direct_kernel<BF16, VEC, KH, 1, K_DIRECT_U><<<grid, block, 0, st>>>(k);
    else if (kw == 2) pool_direct_kernel<BF16, VEC, KH, 2, K_DIRECT_U><<<grid, block, 0, st>>>(k);
    else pool_direct_kernel<BF16, VEC, KH, 4, K_DIRECT_U><<<grid, block, 0, st>>>(k);
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
            if (q.vec == 8) stream_kernel<true, 8, K_STREAM_U><<<grid, block, 0, st>>>(k);
            else stream_kernel<true, 1, K_STREAM_U><<<grid, block, 0, st>>>(k);
        } else {
            if (q.vec == 4) stream_kernel<false, 4, K_STREAM_U><<<grid, block, 0, st>>>(k);
            else stream_kernel<false, 1, K_STREAM_U><<<grid, block, 0, st>>>(k);
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
