// Host side of pool_xrows_kernel and pool_xrows2_kernel (the sliding-window kernels whose
// lanes exchange edge columns): applicability tests, run-time build names and launchers.
// The pre-compiled signatures are those of the kernels that load their edge columns.
#include <cstdio>
#include <string>
#include <type_traits>

#include "bs_xrows_device.h"
#include "bs_rows_tables.h"
#include "bs_internal.h"

namespace bs {

// Can pool_xrows_kernel be instantiated for this shape?  The lane's column block must hold
// whole window strides, the edge columns must come from the adjacent lanes only, and the
// register window must stay small.
bool xrows_buildable(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post, int32_t vec)
{
    if (rows_ew_code(pre, n_pre) < 0 || rows_ew_code(post, n_post) < 0) return false;
    const int32_t nx = pool.kw - pool.sw - pool.pw;
    if (pool.sw < 1 || vec % pool.sw != 0 || nx < 0 || nx > vec || pool.pw > vec || pool.kh < pool.sh || pool.kw < pool.sw)
        return false;
    const int32_t wr = pool.kh + (K_ROWS_OR - 1) * pool.sh, nc = pool.pw + vec + nx;
    return wr * nc <= 160;
}

// The same for pool_xrows2_kernel (see its static_assert).
bool xrows2_buildable(const PoolRows2K &k, int32_t vec)
{
    if (rows_ew_code(k.pre, k.n_pre) < 0 || rows_ew_code(k.mid, k.n_mid) < 0 || rows_ew_code(k.post, k.n_post) < 0)
        return false;
    const PoolK &a = k.pool1, &b = k.pool2;
    if (a.sw < 1 || b.sw < 1 || vec % (a.sw * b.sw) != 0 || a.kh < a.sh || b.kh < b.sh || a.kw < a.sw || b.kw < b.sw)
        return false;
    const int32_t vb = vec / a.sw;
    const int32_t nx0 = a.kw - a.sw - a.pw, nx1 = b.kw - b.sw - b.pw;
    if (nx0 < 0 || nx0 > vec || a.pw > vec || nx1 < 0 || nx1 > vb || b.pw > vb) return false;
    const int32_t r0 = (b.kh - 1) * a.sh + a.kh;
    return r0 * (a.pw + vec + nx0) + b.kh * (b.pw + vb + nx1) <= 200;
}

static std::string spec_expr(const PoolK &p)
{
    char b[160];
    std::snprintf(b, sizeof b, "bs::RowsSpec<%d, %d, %d, %d, %d, %d, %d>", p.kind, p.kh, p.kw, p.sh, p.sw, p.ph, p.pw);
    return b;
}

std::string xrows_expr(const PoolRowsK &k, int32_t dtype, bool want_idx)
{
    char b[96];
    std::snprintf(b, sizeof b, ", %d, %d, %s, %d>", rows_ew_code(k.pre, k.n_pre), rows_ew_code(k.post, k.n_post),
                  want_idx ? "true" : "false", K_ROWS_OR);
    return std::string("bs::pool_xrows_kernel<") + std::to_string(dtype) + ", " + std::to_string(xrows_vec(dtype)) + ", " +
           spec_expr(k.pool) + b;
}

// The conditions pool_xrows2_kernel's PLAIN instances take for granted.
bool xrows2_is_plain(const PoolRows2K &k, int32_t dtype)
{
    const int32_t vec = xrows2_vec(dtype);
    if (k.pool1.sw < 1 || k.pool2.sw < 1 || vec % (k.pool1.sw * k.pool2.sw) != 0) return false;
    const int32_t vb = vec / k.pool1.sw, vo = vb / k.pool2.sw;
    const bool divisors = (k.pool1.kind == OP_MAXPOOL || k.pool1.count_include_pad == 1) &&
                          (k.pool2.kind == OP_MAXPOOL || k.pool2.count_include_pad == 1);
    return divisors && k.W1 >= k.cbs * vb && k.Wo % vo == 0 && k.cbs * vo <= k.Wo;
}

std::string xrows2_expr(const PoolRows2K &k, int32_t dtype, bool want_idx)
{
    char b[96];
    std::snprintf(b, sizeof b, ", %d, %d, %d, %s, %s>", rows_ew_code(k.pre, k.n_pre), rows_ew_code(k.mid, k.n_mid),
                  rows_ew_code(k.post, k.n_post), want_idx ? "true" : "false", xrows2_is_plain(k, dtype) ? "true" : "false");
    return std::string("bs::pool_xrows2_kernel<") + std::to_string(dtype) + ", " + std::to_string(xrows2_vec(dtype)) + ", " +
           spec_expr(k.pool1) + ", " + spec_expr(k.pool2) + b;
}

// What the kernels assume about their argument block: rows fit a wave, whole column blocks,
// whole 4-wave work-groups, a grid that covers every segment.
template <class K>
static bool xrows_args_ok(const K &k, int32_t vec, int64_t grid_n, int32_t threads)
{
    if (k.cbs < 1 || k.cbs > 64 || (int64_t)k.cbs * vec != k.W || k.spw != 64 / k.cbs) return false;
    if (k.div_cbs.d != (uint32_t)k.cbs || k.div_chunks.d != (uint32_t)k.chunks || k.div_c.d != (uint32_t)k.C) return false;
    if (threads < 64 || threads % 64 != 0 || k.rc < 1 || (int64_t)k.chunks * k.rc < k.Ho) return false;
    const int64_t waves = grid_n * (threads / 64);
    return waves * k.spw >= (int64_t)k.units;
}

bool xrows_launchable(const PoolRowsK &k, int32_t dtype, int64_t grid_n, int32_t threads)
{
    return xrows_args_ok(k, xrows_vec(dtype), grid_n, threads) && k.rc % K_ROWS_OR == 0;
}

bool xrows2_launchable(const PoolRows2K &k, int32_t dtype, int64_t grid_n, int32_t threads)
{
    // every column of the plane between the pools must belong to some lane
    return xrows_args_ok(k, xrows2_vec(dtype), grid_n, threads) &&
           (int64_t)k.cbs * (xrows2_vec(dtype) / k.pool1.sw) >= k.W1;
}

template <int DT, int VEC>
static bool xrows_launch_t(const PoolRowsK &k, bool want_idx, dim3 grid, dim3 block, hipStream_t st)
{
    const int cp = rows_ew_code(k.pre, k.n_pre), cq = rows_ew_code(k.post, k.n_post);
    return rows_for_each_signature([&](auto spec, auto pc, auto qc) {
        using P = decltype(spec);
        constexpr int PC = decltype(pc)::value, QC = decltype(qc)::value;
        if (!rows_pool_is<P>(k.pool) || cp != PC || cq != QC) return false;
        if (want_idx) pool_xrows_kernel<DT, VEC, P, PC, QC, true, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        else pool_xrows_kernel<DT, VEC, P, PC, QC, false, K_ROWS_OR><<<grid, block, 0, st>>>(k);
        return true;
    });
}

bs_status launch_xrows(const PoolRowsK &k, int32_t dtype, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const bool want_idx = k.idx != nullptr && k.pool.kind == OP_MAXPOOL;
    if (!dtype_has_tables(dtype) || !xrows_launchable(k, dtype, grid_n, threads)) return BS_ERR_UNSUPPORTED;
    const bool ok = dtype == BS_BF16 ? xrows_launch_t<DT_BF16, K_XROWS_VEC16>(k, want_idx, grid, block, st)
                                     : xrows_launch_t<DT_F32, K_XROWS_VEC32>(k, want_idx, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

template <int DT, int VEC>
static bool xrows2_launch_t(const PoolRows2K &k, bool want_idx, dim3 grid, dim3 block, hipStream_t st)
{
    const int c0 = rows_ew_code(k.pre, k.n_pre), c1 = rows_ew_code(k.mid, k.n_mid), c2 = rows_ew_code(k.post, k.n_post);
    return rows2_for_each_signature([&](auto s1, auto s2, auto e0, auto e1, auto e2) {
        using P1 = decltype(s1);
        using P2 = decltype(s2);
        constexpr int C0 = decltype(e0)::value, C1 = decltype(e1)::value, C2 = decltype(e2)::value;
        if (!rows_pool_is<P1>(k.pool1) || !rows_pool_is<P2>(k.pool2) || c0 != C0 || c1 != C1 || c2 != C2) return false;
        const bool plain = xrows2_is_plain(k, DT == DT_BF16 ? BS_BF16 : BS_F32);
        if (want_idx && plain) pool_xrows2_kernel<DT, VEC, P1, P2, C0, C1, C2, true, true><<<grid, block, 0, st>>>(k);
        else if (want_idx) pool_xrows2_kernel<DT, VEC, P1, P2, C0, C1, C2, true, false><<<grid, block, 0, st>>>(k);
        else if (plain) pool_xrows2_kernel<DT, VEC, P1, P2, C0, C1, C2, false, true><<<grid, block, 0, st>>>(k);
        else pool_xrows2_kernel<DT, VEC, P1, P2, C0, C1, C2, false, false><<<grid, block, 0, st>>>(k);
        return true;
    });
}

bs_status launch_xrows2(const PoolRows2K &k, int32_t dtype, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const bool want_idx = k.idx != nullptr && k.pool2.kind == OP_MAXPOOL;
    if (!dtype_has_tables(dtype) || !xrows2_launchable(k, dtype, grid_n, threads)) return BS_ERR_UNSUPPORTED;
    const bool ok = dtype == BS_BF16 ? xrows2_launch_t<DT_BF16, K_XROWS2_VEC16>(k, want_idx, grid, block, st)
                                     : xrows2_launch_t<DT_F32, K_XROWS2_VEC32>(k, want_idx, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

// Instances of the chain kernel compiled into the library: 3 x 3 max pooling (stride 1, padding 1) followed by
// BatchNorm, ReLU (the blocks of Section 5.1), three to eight levels, float32 and bfloat16.
bool xrows_chain_supported(const RowsChainK &k, int32_t dtype)
{
    if (!dtype_has_tables(dtype) || k.n_levels < 1 || k.n_levels > K_CHAIN_MAX || !rows_pool_is<RMax3s1p1>(k.pool)) return false;
    for (int32_t l = 0; l < k.n_levels; ++l)
        if (rows_ew_code(k.ew[l], k.n_ew) != RW_BN_RELU) return false;
    return true;
}

// Can the chain kernel be instantiated for this chain (a run-time build)?  Max pooling with an odd window, stride 1,
// padding (k - 1) / 2, edge columns from the adjacent lanes only, every level the same list without Add, and rings
// (levels x window rows x columns) that stay in registers.
bool xrows_chain_buildable(const RowsChainK &k, int32_t vec)
{
    const PoolK &p = k.pool;
    if (k.n_levels < 1 || k.n_levels > K_CHAIN_MAX || p.kind != OP_MAXPOOL || p.sh != 1 || p.sw != 1 || p.kh != 2 * p.ph + 1 ||
        p.kw != 2 * p.pw + 1 || p.pw > vec || p.kh > 7)
        return false;
    const int code = rows_ew_code(k.ew[0], k.n_ew);
    if (code < 0) return false;
    for (int32_t l = 1; l < k.n_levels; ++l)
        if (rows_ew_code(k.ew[l], k.n_ew) != code) return false;
    return k.n_levels * p.kh * vec <= 200;
}

std::string xrows_chain_expr(const RowsChainK &k, int32_t dtype)
{
    char b[64];
    std::snprintf(b, sizeof b, ", %d, %d>", rows_ew_code(k.ew[0], k.n_ew), k.n_levels);
    return std::string("bs::pool_xrows_chain_kernel<") + std::to_string(dtype) + ", " + std::to_string(xrows_vec(dtype)) + ", " +
           spec_expr(k.pool) + b;
}

// What the chain kernel assumes about its argument block and launch.
bool xrows_chain_launchable(const RowsChainK &k, int32_t dtype, int64_t grid_n, int32_t threads)
{
    const int32_t vec = xrows_vec(dtype);
    return k.cbs >= 1 && k.cbs <= 64 && (int64_t)k.cbs * vec == k.W && k.spw == 64 / k.cbs && k.div_cbs.d == (uint32_t)k.cbs &&
           k.div_chunks.d == (uint32_t)k.chunks && k.div_c.d == (uint32_t)k.C && threads >= 64 && threads % 64 == 0 && k.rc >= 1 &&
           (int64_t)k.chunks * k.rc >= k.H && grid_n * (threads / 64) * k.spw >= (int64_t)k.units;
}

template <int DT, int VEC>
static bool xrows_chain_launch_t(const RowsChainK &k, dim3 grid, dim3 block, hipStream_t st)
{
    switch (k.n_levels) {
    case 1: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 1><<<grid, block, 0, st>>>(k); return true;
    case 2: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 2><<<grid, block, 0, st>>>(k); return true;
    case 3: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 3><<<grid, block, 0, st>>>(k); return true;
    case 4: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 4><<<grid, block, 0, st>>>(k); return true;
    case 5: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 5><<<grid, block, 0, st>>>(k); return true;
    case 6: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 6><<<grid, block, 0, st>>>(k); return true;
    case 7: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 7><<<grid, block, 0, st>>>(k); return true;
    case 8: pool_xrows_chain_kernel<DT, VEC, RMax3s1p1, RW_BN_RELU, 8><<<grid, block, 0, st>>>(k); return true;
    default: return false;
    }
}

bs_status launch_xrows_chain(const RowsChainK &k, int32_t dtype, int64_t grid_n, int32_t threads, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    // what the kernel assumes: rows of whole column blocks in one wave, chunks that cover the plane, whole work-groups
    if (!xrows_chain_supported(k, dtype) || !xrows_chain_launchable(k, dtype, grid_n, threads)) return BS_ERR_UNSUPPORTED;
    const bool ok = dtype == BS_BF16 ? xrows_chain_launch_t<DT_BF16, K_XROWS_VEC16>(k, grid, block, st)
                                     : xrows_chain_launch_t<DT_F32, K_XROWS_VEC32>(k, grid, block, st);
    return ok ? BS_OK : BS_ERR_UNSUPPORTED;
}

}  // namespace bs
