// Host side of pool_rows_kernel: signature table, applicability test and launcher.
#include <cstdio>
#include <string>
#include <type_traits>

#include "bs_rows_tables.h"
#include "bs_internal.h"

namespace bs {

// =============================================================================
// Signature table, applicability test and launcher.
// =============================================================================
bool rows_supported(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post)
{
    const int cp = rows_ew_code(pre, n_pre), cq = rows_ew_code(post, n_post);
    if (cp < 0 || cq < 0) return false;
    return rows_for_each_signature([&](auto spec, auto pc, auto qc) {
        using P = decltype(spec);
        return rows_pool_is<P>(pool) && cp == decltype(pc)::value && cq == decltype(qc)::value;
    });
}

// Can pool_rows_kernel be instantiated for this shape?  The lane's column block must hold whole
// windows strides (vec % sw), the windows may reach past the block on the right only
// (kw - sw - pw >= 0), and the register window must stay small.
bool rows_buildable(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post, int32_t vec)
{
    if (rows_ew_code(pre, n_pre) < 0 || rows_ew_code(post, n_post) < 0) return false;
    if (pool.sw < 1 || vec % pool.sw != 0 || pool.kw - pool.sw - pool.pw < 0 || pool.kh < pool.sh || pool.kw < pool.sw)
        return false;
    const int32_t wr = pool.kh + (K_ROWS_OR - 1) * pool.sh, nc = pool.pw + vec + (pool.kw - pool.sw - pool.pw);
    return wr * nc <= 128;
}

static std::string spec_expr(const PoolK &p)
{
    char b[160];
    std::snprintf(b, sizeof b, "bs::RowsSpec<%d, %d, %d, %d, %d, %d, %d>", p.kind, p.kh, p.kw, p.sh, p.sw, p.ph, p.pw);
    return b;
}

std::string rows_expr(const PoolRowsK &k, int32_t dtype, bool want_idx)
{
    char b[96];
    std::snprintf(b, sizeof b, ", %d, %d, %s, %d>", rows_ew_code(k.pre, k.n_pre), rows_ew_code(k.post, k.n_post),
                  want_idx ? "true" : "false", K_ROWS_OR);
    return std::string("bs::pool_rows_kernel<") + std::to_string(dtype) + ", " + std::to_string(rows_vec(dtype)) + ", " +
           spec_expr(k.pool) + b;
}

template <int DT, int VEC>
static bool rows_launch_t(const PoolRowsK &k, bool want_idx, dim3 grid, dim3 block, hipStream_t st)
{
    // the argument block must have been planned for this instance's column-block width
    if ((int64_t)k.cbs * VEC != k.W) return false;
    const int cp = rows_ew_code(k.pre, k.n_pre), cq = rows_ew_code(k.post, k.n_post);
    return rows_for_each_signature([&](auto spec, auto pc, auto qc) {
        using P = decltype(spec);
        constexpr int PC = decltype(pc)::value, QC = decltype(qc)::value;
        if (!rows_pool_is<P>(k.pool) || cp != PC || cq != QC) return false;
        if (want_idx) pool_rows_kernel<DT, VEC, P, PC, QC, true, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        else pool_rows_kernel<DT, VEC, P, PC, QC, false, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        return true;
    });
}

bs_status launch_rows(const PoolRowsK &k, int32_t dtype, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const bool want_idx = k.idx != nullptr && k.pool.kind == OP_MAXPOOL;
    if (!dtype_has_tables(dtype)) return BS_ERR_UNSUPPORTED;
    const bool ok = dtype == BS_BF16 ? rows_launch_t<DT_BF16, K_ROWS_VEC16>(k, want_idx, grid, block, st)
                                     : rows_launch_t<DT_F32, 4>(k, want_idx, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
