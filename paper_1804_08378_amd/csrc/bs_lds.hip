// Host side of the lds_tile kernels: the table of stack signatures with a pre-compiled
// build, and the launcher.
#include <cstdio>
#include <string>

#include "bs_lds_device.h"
#include "bs_internal.h"

namespace bs {

// =============================================================================
// Signature table and launcher.
// =============================================================================
using Max3s2p1 = PoolSpec<OP_MAXPOOL, 3, 3, 2, 2, 1, 1, 1>;
using Max3s1p1 = PoolSpec<OP_MAXPOOL, 3, 3, 1, 1, 1, 1, 1>;
using Avg3s1p1 = PoolSpec<OP_AVGSUM, 3, 3, 1, 1, 1, 1, 1>;
using Max2s2p0 = PoolSpec<OP_MAXPOOL, 2, 2, 2, 2, 0, 0, 1>;
using Avg2s2p0 = PoolSpec<OP_AVGSUM, 2, 2, 2, 2, 0, 0, 1>;

constexpr int EW_NONE = 0;
constexpr int EW_BN_RELU = OP_BN + K_EW_BASE * OP_RELU;

static int ew_code(const LevelK &lv)
{
    int code = 0, mul = 1;
    for (int j = 0; j < lv.n_ew; ++j) {
        code += lv.ew[j].kind * mul;
        mul *= K_EW_BASE;
    }
    return code;
}

template <class P>
static bool pool_is(const PoolK &q)
{
    return q.kind == P::kind() && q.kh == P::kh() && q.kw == P::kw() && q.sh == P::sh() && q.sw == P::sw() &&
           q.ph == P::ph() && q.pw == P::pw() && (q.kind == OP_MAXPOOL || q.count_include_pad == P::cip());
}

enum { LAUNCH = 0, DRY_SIGNATURE = 1, DRY_FULL = 2 };  // what the table walk does on a match

template <int DT, int VEC, int EW0, class... Ls>
static bool try_sig(const LdsSeqK &k, bool want_idx, dim3 grid, dim3 block, size_t lds, hipStream_t st, int dry)
{
    constexpr int NL = (int)sizeof...(Ls);
    if (k.n_levels != NL || (dry != DRY_SIGNATURE && k.vec != VEC)) return false;
    if (ew_code(k.level[0]) != EW0) return false;
    int l = 0;
    const bool same = ((++l, pool_is<typename Ls::P>(k.pool[l]) && ew_code(k.level[l]) == Ls::EW::code) && ...);
    if (!same) return false;
    if (dry == DRY_SIGNATURE) return true;
    if (k.delta0 != sig_delta0<VEC, Ls...>()) return false;
    if (dry == DRY_FULL) return true;
    if (want_idx) lds_sig_kernel<DT, VEC, true, EW0, Ls...><<<grid, block, lds, st>>>(k);
    else lds_sig_kernel<DT, VEC, false, EW0, Ls...><<<grid, block, lds, st>>>(k);
    return true;
}

template <int DT, int VEC, int EW0, class LV>
static bool try_rep(const LdsSeqK &k, bool want_idx, dim3 grid, dim3 block, size_t lds, hipStream_t st, int dry)
{
    if (k.n_levels < 3 || (dry != DRY_SIGNATURE && k.vec != VEC) || ew_code(k.level[0]) != EW0) return false;
    for (int l = 1; l <= k.n_levels; ++l)
        if (!pool_is<typename LV::P>(k.pool[l]) || ew_code(k.level[l]) != LV::EW::code) return false;
    if (dry != LAUNCH) return true;
    if (want_idx) lds_rep_kernel<DT, VEC, true, EW0, LV><<<grid, block, lds, st>>>(k);
    else lds_rep_kernel<DT, VEC, false, EW0, LV><<<grid, block, lds, st>>>(k);
    return true;
}

// Stack signatures with a dedicated build.  First match wins; anything else runs the
// run-time build.
template <int DT, int VEC>
static bool launch_sig(const LdsSeqK &k, bool want_idx, dim3 grid, dim3 block, size_t lds, hipStream_t st, int dry)
{
    // BN -> ReLU -> MaxPool 3/2/1 (ResNet stem), and the pool on its own (layer by layer)
    if (try_sig<DT, VEC, EW_BN_RELU, Lvl<Max3s2p1, EW_NONE>>(k, want_idx, grid, block, lds, st, dry)) return true;
    if (try_sig<DT, VEC, EW_NONE, Lvl<Max3s2p1, EW_NONE>>(k, want_idx, grid, block, lds, st, dry)) return true;
    // BN -> ReLU -> AvgPool 3/1/1 -> MaxPool 3/2/1 -> BN -> ReLU (halo stress), and its average alone
    if (try_sig<DT, VEC, EW_BN_RELU, Lvl<Avg3s1p1, EW_NONE>, Lvl<Max3s2p1, EW_BN_RELU>>(k, want_idx, grid, block, lds, st, dry)) return true;
    if (try_sig<DT, VEC, EW_NONE, Lvl<Avg3s1p1, EW_NONE>>(k, want_idx, grid, block, lds, st, dry)) return true;
    // <MaxPool 3/1/1, BN, ReLU> blocks of Section 5.1: one and two per sequence, and the pool alone
    if (try_sig<DT, VEC, EW_NONE, Lvl<Max3s1p1, EW_BN_RELU>>(k, want_idx, grid, block, lds, st, dry)) return true;
    if (try_sig<DT, VEC, EW_NONE, Lvl<Max3s1p1, EW_BN_RELU>, Lvl<Max3s1p1, EW_BN_RELU>>(k, want_idx, grid, block, lds, st, dry)) return true;
    if (try_sig<DT, VEC, EW_NONE, Lvl<Max3s1p1, EW_NONE>>(k, want_idx, grid, block, lds, st, dry)) return true;
    // three or more of those blocks in one sequence
    if (try_rep<DT, VEC, EW_NONE, Lvl<Max3s1p1, EW_BN_RELU>>(k, want_idx, grid, block, lds, st, dry)) return true;
    return false;
}

// Is there a signature / repeated build for this sequence shape (pooling operations and
// element-wise lists only; tile geometry is not looked at)?  The planner uses it to avoid
// merging steps into a sequence that would fall back to the much slower run-time build.
bool lds_fast_path(const LdsSeqK &k)
{
    return launch_sig<DT_F32, 4>(k, false, dim3(1), dim3(64), 0, nullptr, DRY_SIGNATURE);
}

// Will launch_lds run a pre-compiled signature / repeated build for this planned sequence
// (signature, vector width and row alignment all match)?
bool lds_precompiled(const LdsSeqK &k, int32_t dtype)
{
    if (!dtype_has_tables(dtype)) return false;
    return dtype == BS_BF16 ? launch_sig<DT_BF16, 8>(k, false, dim3(1), dim3(64), 0, nullptr, DRY_FULL)
                            : launch_sig<DT_F32, 4>(k, false, dim3(1), dim3(64), 0, nullptr, DRY_FULL);
}

// Can lds_sig_kernel be instantiated for this planned sequence?  Its level-1 phase takes the
// row alignment from the pooling shapes; the planner's geometry must agree.
bool lds_buildable(const LdsSeqK &k)
{
    int32_t c = 0;
    for (int l = k.n_levels; l >= 1; --l) c = c * k.pool[l].sw - k.pool[l].pw;
    const int32_t d0 = ((c % k.vec) + k.vec) % k.vec;
    return k.n_levels >= 1 && k.delta0 == d0;
}

// Name of the lds_sig_kernel instance for this sequence (run-time build).
std::string lds_expr(const LdsSeqK &k, int32_t dtype, bool want_idx)
{
    char b[200];
    std::snprintf(b, sizeof b, "bs::lds_sig_kernel<%d, %d, %s, %d", dtype, k.vec,
                  want_idx ? "true" : "false", ew_code(k.level[0]));
    std::string e = b;
    for (int l = 1; l <= k.n_levels; ++l) {
        const PoolK &p = k.pool[l];
        std::snprintf(b, sizeof b, ", bs::Lvl<bs::PoolSpec<%d, %d, %d, %d, %d, %d, %d, %d>, %d>", p.kind, p.kh, p.kw, p.sh,
                      p.sw, p.ph, p.pw, p.kind == OP_MAXPOOL ? 1 : p.count_include_pad, ew_code(k.level[l]));
        e += b;
    }
    return e + ">";
}

bs_status launch_lds(const LdsSeqK &k, int32_t dtype, int64_t grid_n, int32_t threads, uint64_t lds_bytes, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)grid_n), block((uint32_t)threads);
    const size_t lds = (size_t)lds_bytes;
    bool want_idx = false;
    for (int l = 1; l <= k.n_levels; ++l)
        if (k.pool[l].idx_slot >= 0 && k.idx[k.pool[l].idx_slot]) want_idx = true;
    // vector widths the compiled instances exist for (guards against a plan / kernel mismatch)
    if (k.vec != 1 && k.vec != (dtype == BS_F32 ? 4 : 8)) return BS_ERR_UNSUPPORTED;
    if (dtype == BS_F16) {  // no signature table for binary16: the run-time-shape kernel
        if (k.vec == 8) lds_tile_kernel<DT_F16, 8><<<grid, block, lds, st>>>(k);
        else lds_tile_kernel<DT_F16, 1><<<grid, block, lds, st>>>(k);
    } else if (dtype == BS_BF16) {
        if (k.vec == 8) {
            if (!launch_sig<DT_BF16, 8>(k, want_idx, grid, block, lds, st, LAUNCH))
                lds_tile_kernel<DT_BF16, 8><<<grid, block, lds, st>>>(k);
        } else {
            lds_tile_kernel<DT_BF16, 1><<<grid, block, lds, st>>>(k);
        }
    } else {
        if (k.vec == 4) {
            if (!launch_sig<DT_F32, 4>(k, want_idx, grid, block, lds, st, LAUNCH))
                lds_tile_kernel<DT_F32, 4><<<grid, block, lds, st>>>(k);
        } else {
            lds_tile_kernel<DT_F32, 1><<<grid, block, lds, st>>>(k);
        }
    }
    return BS_OK;
}

}  // namespace bs
