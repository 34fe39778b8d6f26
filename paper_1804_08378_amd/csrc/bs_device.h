// Device-side helpers shared by the HIP kernels: fast division, bfloat16 conversion,
// 128-bit register blocks and their loads / stores.
#pragma once

#if !defined(__HIPCC_RTC__)
#include <hip/hip_runtime.h>

#include <cmath>
#endif
#if !defined(INFINITY)
#define INFINITY __builtin_inff()
#endif

#include "bs_kargs.h"

namespace bs {


#define BS_DEV __device__ __forceinline__

BS_DEV uint32_t fdiv(uint32_t n, const FastDiv &f)
{
    return f.d == 1 ? n : (__umulhi(n, f.mul) >> f.shift);
}

// ------------------------------------------------------------ work-group order
// Work-groups are handed to the chip's 8 XCDs round-robin, and each XCD has its own L2.
// Overlapping windows and tile halos make neighbouring work-groups read the same input rows
// and columns; with this remapping XCD x gets one contiguous eighth of the work and finds the
// shared cells in its own L2.  A bijection of [0, n): the last n % 8 groups keep their index.
// Measured on MI355X: 8 % faster for the channels-last 3x3/2 pool in float32, 4 % slower for
// disjoint 2x2/2 windows, no difference for the LDS tile kernels (bound by instruction issue):
// used by the channels-last pooling kernel for overlapping windows only.
BS_DEV uint32_t xcd_contiguous(uint32_t bid, uint32_t n)
{
    constexpr uint32_t X = 8;
    const uint32_t per = n / X;
    return bid >= per * X ? bid : (bid % X) * per + bid / X;
}

// ------------------------------------------------------- 16-bit storage types
// DT: 0 = float32, 1 = bfloat16, 2 = IEEE binary16 storage (the values of bs_dtype).  Arithmetic
// is float32 for all three; a layer's output is rounded to the storage type (nearest-even)
// by the compiler's conversions (v_cvt_pk_bf16_f32 / v_cvt_f16_f32).
constexpr int DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2;

// Two float32 values rounded to the 16-bit storage type, in one 32-bit word (a in the low half).  bfloat16: one
// v_cvt_pk_bf16_f32.
template <int DT>
BS_DEV uint32_t pack2(float a, float b)
{
    typedef float f2 __attribute__((ext_vector_type(2)));
    const f2 v = {a, b};
    if constexpr (DT == DT_BF16) {
        typedef __bf16 h2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, h2));
    } else {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, h2));
    }
}

template <int DT>
BS_DEV uint16_t half_bits(float f)
{
    if constexpr (DT == DT_BF16) {
        const __bf16 h = (__bf16)f;
        return __builtin_bit_cast(uint16_t, h);
    } else {
        const _Float16 h = (_Float16)f;
        return __builtin_bit_cast(uint16_t, h);
    }
}

template <int DT>
BS_DEV float half_up(uint32_t bits16)
{
    if constexpr (DT == DT_BF16) return __uint_as_float(bits16 << 16);
    else return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

template <int DT>
BS_DEV float round_store(float v)
{
    if constexpr (DT == DT_BF16) {
        return (float)(__bf16)v;
    } else if constexpr (DT == DT_F16) {
        // A layer's float32 result is rounded to float32 first and to binary16 second.  Without
        // this barrier the compiler merges a preceding fused multiply-add with the conversion into
        // one v_fma_mixlo_f16, which rounds once, straight to binary16: a different (if closer)
        // value in rare double-rounding cases than the layer definition gives.
        asm("" : "+v"(v));
        return (float)(_Float16)v;
    } else {
        return v;
    }
}

// round_store on N values at once.  bfloat16: pairs share one v_cvt_pk_bf16_f32 (three instructions per two values
// instead of four, and no conversion with an unused second operand, which the compiler fills with whatever register is
// at hand -- the target of a load in flight makes the conversion wait for that load).
template <int DT, int N>
BS_DEV void round_store_all(float (&x)[N])
{
    if constexpr (DT == DT_BF16 && N % 2 == 0) {
#pragma unroll
        for (int i = 0; i < N; i += 2) {
            const uint32_t w = pack2<DT_BF16>(x[i], x[i + 1]);
            x[i] = __uint_as_float(w << 16);
            x[i + 1] = __uint_as_float(w & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) x[i] = round_store<DT>(x[i]);
    }
}

// ------------------------------------------------------------ strided images
// The input and the output of a sequence may be channel slices of larger NCHW tensors: image n
// then starts `extra` elements later than in a dense tensor for every image before it
// (extra = batch stride - C*H*W).  All element offsets in the kernels stay those of a dense
// tensor (they also address residuals and index outputs, which are dense); only the base
// pointer moves per image.
template <int DT>
BS_DEV const void *image_base(const void *p, uint32_t n, uint32_t extra)
{
    return static_cast<const char *>(p) + (size_t)n * extra * (DT != DT_F32 ? 2 : 4);
}
template <int DT>
BS_DEV void *image_base(void *p, uint32_t n, uint32_t extra)
{
    return static_cast<char *>(p) + (size_t)n * extra * (DT != DT_F32 ? 2 : 4);
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

template <int DT, int N>
struct Raw {
    using type = typename RawT<N * (DT != DT_F32 ? 2 : 4)>::type;
    type q;
};

// NT: non-temporal (streaming) load for data that is read exactly once; leave it off where
// neighbouring lanes or tiles re-read the same cache lines.
template <int DT, int N, bool NT = false>
BS_DEV Raw<DT, N> load_raw(const void *base, uint32_t elem)
{
    using T = typename Raw<DT, N>::type;
    Raw<DT, N> r;
    const char *ptr = static_cast<const char *>(base) + (size_t)elem * (DT != DT_F32 ? 2 : 4);
    constexpr int BYTES = N * (DT != DT_F32 ? 2 : 4);
    if constexpr (!NT) {
        r.q = *reinterpret_cast<const T *>(ptr);
    } else if constexpr (BYTES == 16) {
        typedef unsigned u4 __attribute__((ext_vector_type(4)));
        const u4 t = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(ptr));
        r.q = make_uint4(t.x, t.y, t.z, t.w);
    } else if constexpr (BYTES == 8) {
        typedef unsigned u2 __attribute__((ext_vector_type(2)));
        const u2 t = __builtin_nontemporal_load(reinterpret_cast<const u2 *>(ptr));
        r.q = make_uint2(t.x, t.y);
    } else {
        r.q = __builtin_nontemporal_load(reinterpret_cast<const T *>(ptr));
    }
    return r;
}

template <int DT, int N>
BS_DEV void unpack(const Raw<DT, N> &r, float (&v)[N])
{
    constexpr int BYTES = N * (DT != DT_F32 ? 2 : 4);
    if constexpr (BYTES == 2) {
        v[0] = half_up<DT>(r.q);
    } else {
        constexpr int WORDS = BYTES / 4;
        uint32_t w[WORDS];
        if constexpr (BYTES == 16) { w[0] = r.q.x; w[1] = r.q.y; w[2] = r.q.z; w[3] = r.q.w; }
        else if constexpr (BYTES == 8) { w[0] = r.q.x; w[1] = r.q.y; }
        else w[0] = r.q;
        if constexpr (DT == DT_F32) {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) v[i] = __uint_as_float(w[i]);
        } else {
#pragma unroll
            for (int i = 0; i < WORDS; ++i) {
                if constexpr (DT == DT_BF16) {
                    v[2 * i] = __uint_as_float(w[i] << 16);
                    v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
                } else {
                    v[2 * i] = half_up<DT>(w[i] & 0xffffu);
                    v[2 * i + 1] = half_up<DT>(w[i] >> 16);
                }
            }
        }
    }
}

// Store N consecutive int32 indices at an address aligned to N * 4 bytes (N = 1, 2, 4; 8 as two
// halves).  Plain stores: non-temporal ones measured 3..8 % slower here in every kernel.
template <int N>
BS_DEV void store_indices(int32_t *p, const int32_t (&v)[N])
{
    typedef int i4 __attribute__((ext_vector_type(4)));
    typedef int i2 __attribute__((ext_vector_type(2)));
    if constexpr (N == 8) {
        const i4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
        *reinterpret_cast<i4 *>(p) = a;
        *reinterpret_cast<i4 *>(p + 4) = b;
    } else if constexpr (N == 4) {
        const i4 t = {v[0], v[1], v[2], v[3]};
        *reinterpret_cast<i4 *>(p) = t;
    } else if constexpr (N == 2) {
        const i2 t = {v[0], v[1]};
        *reinterpret_cast<i2 *>(p) = t;
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) p[i] = v[i];
    }
}

// Store N consecutive elements (N * element size is 2, 4, 8 or 16 bytes, naturally aligned).
// Outputs are written once and not read again by the kernel.  NT: non-temporal vector stores,
// measured 2..7 % faster in every kernel except the two-level sliding-window kernel (7 % slower
// there), which uses plain stores.
template <int DT, int N, bool NT = true>
BS_DEV void store_elems(void *base, uint32_t elem, const float (&v)[N])
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    if constexpr (DT == DT_F32) {
        float *p = static_cast<float *>(base) + elem;
        if constexpr (N == 4) {
            const u4 t = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
            if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<u4 *>(p));
            else *reinterpret_cast<u4 *>(p) = t;
        } else if constexpr (N == 2) {
            const u2 t = {__float_as_uint(v[0]), __float_as_uint(v[1])};
            if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<u2 *>(p));
            else *reinterpret_cast<u2 *>(p) = t;
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) p[i] = v[i];
        }
    } else {
        uint16_t *p = static_cast<uint16_t *>(base) + elem;
        if constexpr (N == 8 || N == 4 || N == 2) {
            uint32_t w[N / 2];
#pragma unroll
            for (int i = 0; i < N / 2; ++i)
                w[i] = pack2<DT>(v[2 * i], v[2 * i + 1]);
            if constexpr (N == 8) {
                const u4 t = {w[0], w[1], w[2], w[3]};
                if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<u4 *>(p));
            else *reinterpret_cast<u4 *>(p) = t;
            } else if constexpr (N == 4) {
                const u2 t = {w[0], w[1]};
                if constexpr (NT) __builtin_nontemporal_store(t, reinterpret_cast<u2 *>(p));
            else *reinterpret_cast<u2 *>(p) = t;
            } else {
                *reinterpret_cast<uint32_t *>(p) = w[0];
            }
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) p[i] = half_bits<DT>(v[i]);
        }
    }
}

}  // namespace bs
