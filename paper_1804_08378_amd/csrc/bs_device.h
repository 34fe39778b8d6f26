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

// NT: non-temporal (streaming) load for data that is read exactly once; leave it off where
// neighbouring lanes or tiles re-read the same cache lines.
template <bool BF16, int N, bool NT = false>
BS_DEV Raw<BF16, N> load_raw(const void *base, uint32_t elem)
{
    using T = typename Raw<BF16, N>::type;
    Raw<BF16, N> r;
    const char *ptr = static_cast<const char *>(base) + (size_t)elem * (BF16 ? 2 : 4);
    constexpr int BYTES = N * (BF16 ? 2 : 4);
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
template <bool BF16, int N, bool NT = true>
BS_DEV void store_elems(void *base, uint32_t elem, const float (&v)[N])
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    if constexpr (!BF16) {
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
                w[i] = (uint32_t)bf16_bits(v[2 * i]) | ((uint32_t)bf16_bits(v[2 * i + 1]) << 16);
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
            for (int i = 0; i < N; ++i) p[i] = bf16_bits(v[i]);
        }
    }
}

}  // namespace bs
