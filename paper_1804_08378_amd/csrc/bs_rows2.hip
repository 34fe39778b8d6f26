// Host side of pool_rows2_kernel: signature table, applicability test and launcher.
#include <cstdio>
#include <string>
#include <type_traits>

#include "bs_rows_tables.h"
#include "bs_internal.h"

namespace bs {

// =============================================================================
// Signature table, applicability test and launcher.
// =============================================================================
bool rows2_supported(const PoolRows2K &k)
{
    const int c0 = rows_ew_code(k.pre, k.n_pre), c1 = rows_ew_code(k.mid, k.n_mid), c2 = rows_ew_code(k.post, k.n_post);
    if (c0 < 0 || c1 < 0 || c2 < 0) return false;
    return rows2_for_each_signature([&](auto s1, auto s2, auto e0, auto e1, auto e2) {
        return rows_pool_is<decltype(s1)>(k.pool1) && rows_pool_is<decltype(s2)>(k.pool2) && c0 == decltype(e0)::value &&
               c1 == decltype(e1)::value && c2 == decltype(e2)::value;
    });
}

// Can pool_rows2_kernel be instantiated for these shapes (see its static_assert), with
// register windows of a reasonable size?
bool rows2_buildable(const PoolRows2K &k, int32_t vec)
{
    if (rows_ew_code(k.pre, k.n_pre) < 0 || rows_ew_code(k.mid, k.n_mid) < 0 || rows_ew_code(k.post, k.n_post) < 0)
        return false;
    const PoolK &a = k.pool1, &b = k.pool2;
    if (a.sw < 1 || b.sw < 1 || vec % (a.sw * b.sw) != 0 || a.kh < a.sh || b.kh < b.sh) return false;
    const int32_t vo = vec / (a.sw * b.sw);
    const int32_t nc1 = (vo - 1) * b.sw + b.kw, nl = b.pw * a.sw + a.pw, nc0 = (nc1 - 1) * a.sw + a.kw;
    if (nc0 - nl - vec < 0) return false;
    const int32_t r0 = (b.kh - 1) * a.sh + a.kh;
    return r0 * nc0 + b.kh * nc1 <= 160;
}

std::string rows2_expr(const PoolRows2K &k, int32_t dtype, bool want_idx)
{
    char b[400];
    const PoolK &p = k.pool1, &q = k.pool2;
    std::snprintf(b, sizeof b,
                  "bs::pool_rows2_kernel<%d, %d, bs::RowsSpec<%d, %d, %d, %d, %d, %d, %d>, "
                  "bs::RowsSpec<%d, %d, %d, %d, %d, %d, %d>, %d, %d, %d, %s>",
                  dtype, rows2_vec(dtype), p.kind, p.kh, p.kw, p.sh, p.sw, p.ph, p.pw, q.kind, q.kh, q.kw, q.sh,
                  q.sw, q.ph, q.pw, rows_ew_code(k.pre, k.n_pre), rows_ew_code(k.mid, k.n_mid),
                  rows_ew_code(k.post, k.n_post), want_idx ? "true" : "false");
    return b;
}

template <int DT, int VEC>
static bool rows2_launch_t(const PoolRows2K &k, bool want_idx, dim3 grid, dim3 block, hipStream_t st)
{
    // the argument block must have been planned for this instance's column-block width
    if ((int64_t)k.cbs * VEC != k.W) return false;
    const int c0 = rows_ew_code(k.pre, k.n_pre), c1 = rows_ew_code(k.mid, k.n_mid), c2 = rows_ew_code(k.post, k.n_post);
    return rows2_for_each_signature([&](auto s1, auto s2, auto e0, auto e1, auto e2) {
        using P1 = decltype(s1);
        using P2 = decltype(s2);
        constexpr int C0 = decltype(e0)::value, C1 = decltype(e1)::value, C2 = decltype(e2)::value;
        if (!rows_pool_is<P1>(k.pool1) || !rows_pool_is<P2>(k.pool2) || c0 != C0 || c1 != C1 || c2 != C2) return false;
        if (want_idx) pool_rows2_kernel<DT, VEC, P1, P2, C0, C1, C2, true><<<grid, block, 0, st>>>(k);
        else pool_rows2_kernel<DT, VEC, P1, P2, C0, C1, C2, false><<<grid, block, 0, st>>>(k);
        return true;
    });
}

bs_status launch_rows2(const PoolRows2K &k, int32_t dtype, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const bool want_idx = k.idx != nullptr && k.pool2.kind == OP_MAXPOOL;
    if (!dtype_has_tables(dtype)) return BS_ERR_UNSUPPORTED;
    const bool ok = dtype == BS_BF16 ? rows2_launch_t<DT_BF16, K_ROWS2_VEC16>(k, want_idx, grid, block, st)
                                     : rows2_launch_t<DT_F32, K_ROWS2_VEC32>(k, want_idx, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
