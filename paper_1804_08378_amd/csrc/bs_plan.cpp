// Planner: the "collapse process" of Section 4.1.
//   layers -> basic operations -> steps -> sequences -> kernel variant + tile geometry
// Host code only; the device is touched solely through device_limits() /
// upload_params() (bs_kernels.hip) when the options do not forbid it.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "bs_internal.h"

namespace bs {

// ---------------------------------------------------------------------------
// Layers -> operations (Section 4.1: "map those layers onto basic computational
// operations").  Average pooling becomes a window sum followed by an
// element-wise normalisation, as in Listing 2.
// ---------------------------------------------------------------------------
bs_status build_operations(bs_stack *s)
{
    s->ops.clear();
    s->host_params.clear();
    const int64_t C = s->in_shape[1];
    int32_t res = 0, idx = 0;
    for (size_t i = 0; i < s->layers.size(); ++i) {
        const Layer &L = s->layers[i];
        Op op;
        op.layer = (int32_t)i;
        op.in_h = (int32_t)L.in_shape[2];
        op.in_w = (int32_t)L.in_shape[3];
        op.out_h = (int32_t)L.out_shape[2];
        op.out_w = (int32_t)L.out_shape[3];
        switch (L.desc.kind) {
        case BS_BATCHNORM:
            op.kind = OP_BN;
            op.param_off = (int32_t)s->host_params.size();
            s->host_params.insert(s->host_params.end(), L.scale.begin(), L.scale.end());
            s->host_params.insert(s->host_params.end(), L.shift.begin(), L.shift.end());
            (void)C;
            s->ops.push_back(op);
            break;
        case BS_RELU:
            op.kind = OP_RELU;
            s->ops.push_back(op);
            break;
        case BS_ADD:
            op.kind = OP_ADD;
            op.res_slot = res++;
            s->ops.push_back(op);
            break;
        case BS_MAXPOOL:
        case BS_AVGPOOL: {
            const bs_layer_desc &d = L.desc;
            op.kh = d.kh; op.kw = d.kw; op.sh = d.sh; op.sw = d.sw; op.ph = d.ph; op.pw = d.pw;
            if (d.kind == BS_MAXPOOL) {
                op.kind = OP_MAXPOOL;
                if (d.return_indices) op.idx_slot = idx++;
                s->ops.push_back(op);
            } else {
                op.kind = OP_AVGSUM;
                op.count_include_pad = d.count_include_pad ? 1 : 0;
                s->ops.push_back(op);
                Op norm;
                norm.kind = OP_AVGNORM;
                norm.layer = (int32_t)i;
                norm.in_h = norm.out_h = op.out_h;
                norm.in_w = norm.out_w = op.out_w;
                s->ops.push_back(norm);
            }
            break;
        }
        default:
            return BS_ERR_UNSUPPORTED;
        }
    }
    return BS_OK;
}

// ---------------------------------------------------------------------------
// Operations -> steps (Section 4.1): an element-wise operation always joins the
// current step; a non-element-wise one joins unless the step already holds one,
// in which case the step is closed and a new one starts with this operation.
// The trailing step is kept.  (Listing 1's loop as printed contradicts this
// prose and its own example, Listing 2; the prose and the example are followed.)
// With `per_layer` every layer boundary also closes the step: that is the
// breadth-first execution of Figure 2.
// ---------------------------------------------------------------------------
static void group_steps_impl(bs_stack *s, bool per_layer)
{
    s->steps.clear();
    Step cur;
    cur.first_op = 0;
    // Kernel argument blocks hold a bounded number of element-wise operations per level and
    // of residual tensors; a step that would exceed them is closed early (capacity only --
    // the results do not depend on where steps end).
    int32_t ew_run = 0, adds = 0;
    for (int32_t i = 0; i < (int32_t)s->ops.size(); ++i) {
        const Op &op = s->ops[i];
        bool close = false;
        if (cur.n_ops > 0) {
            if (per_layer && s->ops[i - 1].layer != op.layer) close = true;
            if (!op_is_elementwise(op.kind) && cur.pool_op >= 0) close = true;
            if (op_is_elementwise(op.kind) && op.kind != OP_AVGNORM && ew_run >= K_MAX_EW) close = true;
            if (op.kind == OP_ADD && adds >= K_MAX_RES) close = true;
        }
        if (close) {
            s->steps.push_back(cur);
            cur = Step();
            cur.first_op = i;
            ew_run = adds = 0;
        }
        if (!op_is_elementwise(op.kind)) {
            cur.pool_op = i;
            ew_run = 0;
        } else if (op.kind != OP_AVGNORM) {
            ++ew_run;
            if (op.kind == OP_ADD) ++adds;
        }
        cur.n_ops++;
    }
    if (cur.n_ops > 0) s->steps.push_back(cur);
}

bs_status group_steps(bs_stack *s)
{
    group_steps_impl(s, s->opts.breadth_first != 0);
    return BS_OK;
}

// ---------------------------------------------------------------------------
// Tile geometry.  For a tile [lo, hi) of a pooling operation's output, the input
// cells its windows touch are [lo*s - p, (hi-1)*s - p + k) clipped to the plane
// (cells outside the plane are padding and are never loaded or computed).
// Rows and columns are independent.
// ---------------------------------------------------------------------------
struct Dim {
    int32_t k, s, p;
};

static inline void back_one(const Dim &d, int32_t size_in, int32_t &lo, int32_t &hi)
{
    int32_t nlo = lo * d.s - d.p, nhi = (hi - 1) * d.s - d.p + d.k;
    lo = std::max(0, nlo);
    hi = std::min(size_in, nhi);
}

// Largest region extent per level over all tiles of size `tile` along one dimension.
// dims[l] (l = 1..L) is the pool producing level l; size[l] the plane extent at level l.
static void max_extents(const std::vector<Dim> &dims, const std::vector<int32_t> &size, int32_t tile,
                        int32_t vec0, std::vector<int32_t> &ext)
{
    const int L = (int)dims.size() - 1;
    ext.assign(L + 1, 0);
    const int32_t n_tiles = (size[L] + tile - 1) / tile;
    for (int32_t t = 0; t < n_tiles; ++t) {
        int32_t lo = t * tile, hi = std::min(size[L], lo + tile);
        ext[L] = std::max(ext[L], hi - lo);
        for (int l = L; l >= 1; --l) {
            back_one(dims[l], size[l - 1], lo, hi);
            int32_t a = lo, b = hi;
            if (l - 1 == 0 && vec0 > 1) {
                a = a / vec0 * vec0;
                b = (b + vec0 - 1) / vec0 * vec0;
            }
            ext[l - 1] = std::max(ext[l - 1], b - a);
        }
    }
}

struct LdsGeom {
    int32_t L = 0;
    std::vector<Dim> dh, dw;        // index 1..L
    std::vector<int32_t> H, W;      // index 0..L
    std::vector<int32_t> rows, cols;  // max region extents per level
    uint64_t lds_bytes = 0;
    uint64_t buf_floats[2] = {0, 0};
    double redundancy = 1.0;
};

static void lds_geometry(const bs_stack *s, int32_t first_op, int32_t n_ops, int32_t th, int32_t tw,
                         int32_t ppg, int32_t vec0, LdsGeom &g)
{
    g.dh.assign(1, Dim{1, 1, 0});
    g.dw.assign(1, Dim{1, 1, 0});
    g.H.assign(1, s->ops[first_op].in_h);
    g.W.assign(1, s->ops[first_op].in_w);
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (op_is_elementwise(op.kind)) continue;
        g.dh.push_back(Dim{op.kh, op.sh, op.ph});
        g.dw.push_back(Dim{op.kw, op.sw, op.pw});
        g.H.push_back(op.out_h);
        g.W.push_back(op.out_w);
    }
    g.L = (int32_t)g.dh.size() - 1;
    max_extents(g.dh, g.H, th, 1, g.rows);
    max_extents(g.dw, g.W, tw, vec0, g.cols);
    if (vec0 > 1) g.cols[0] = (g.cols[0] + vec0 - 1) / vec0 * vec0;
    g.buf_floats[0] = g.buf_floats[1] = 0;
    for (int l = 0; l < g.L; ++l) {  // level L goes to memory, not to LDS
        uint64_t need = (uint64_t)ppg * g.rows[l] * g.cols[l];
        need = (need + 3) / 4 * 4;
        g.buf_floats[l & 1] = std::max(g.buf_floats[l & 1], need);
    }
    g.lds_bytes = (g.buf_floats[0] + g.buf_floats[1]) * sizeof(float);
    // elements loaded per plane (sum over tiles of the level-0 region) / plane size
    const int32_t nth = (g.H[g.L] + th - 1) / th, ntw = (g.W[g.L] + tw - 1) / tw;
    uint64_t rsum = 0, csum = 0;
    for (int32_t t = 0; t < nth; ++t) {
        int32_t lo = t * th, hi = std::min(g.H[g.L], lo + th);
        for (int l = g.L; l >= 1; --l) back_one(g.dh[l], g.H[l - 1], lo, hi);
        rsum += (uint64_t)(hi - lo);
    }
    for (int32_t t = 0; t < ntw; ++t) {
        int32_t lo = t * tw, hi = std::min(g.W[g.L], lo + tw);
        for (int l = g.L; l >= 1; --l) back_one(g.dw[l], g.W[l - 1], lo, hi);
        if (vec0 > 1) {
            lo = lo / vec0 * vec0;
            hi = (hi + vec0 - 1) / vec0 * vec0;
        }
        csum += (uint64_t)(hi - lo);
    }
    g.redundancy = (double)rsum * (double)csum / ((double)g.H[0] * (double)g.W[0]);
}

// Does every cell of a pooling operation's input lie in some window?  (k >= s and the
// floor-mode remainder is absorbed by the padding.)  Needed to keep an index-producing
// max pool in the middle of a sequence: its whole output must then be computed by tiles.
static bool covers_input(const Op &op)
{
    auto ok = [](int32_t size, int32_t k, int32_t st, int32_t p) {
        return k >= st && ((size + 2 * p - k) % st) <= p;
    };
    return ok(op.in_h, op.kh, op.sh, op.ph) && ok(op.in_w, op.kw, op.sw, op.pw);
}

static int32_t vec_of(const bs_stack *s) { return s->dtype == BS_BF16 ? 8 : 4; }

struct SeqDraft {
    int32_t first_step, n_steps;
};

// Smallest tile that keeps one work-group busy: one output per thread (Section 4.1's
// resource example counts the data of as many outputs as there are SIMD units).
static void min_tile(int32_t hl, int32_t wl, int32_t threads, int32_t &th, int32_t &tw)
{
    tw = std::min(wl, 64);
    th = std::min(hl, std::max(1, threads / tw));
}

static bool seq_capacity_ok(const bs_stack *s, int32_t first_op, int32_t n_ops, bool allow_stream)
{
    int32_t pools = 0, ew_level = 0, ew_total = 0, res = 0, idx = 0;
    bool has_mid_idx = false;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (op_is_elementwise(op.kind)) {
            if (op.kind == OP_AVGNORM) continue;  // folded into the pooling operation
            ++ew_level;
            ++ew_total;
            if (op.kind == OP_ADD) ++res;
        } else {
            if (has_mid_idx && !covers_input(op)) return false;
            ++pools;
            ew_level = 0;
            if (op.idx_slot >= 0) {
                ++idx;
                has_mid_idx = true;
            }
        }
        if (pools > 0 && ew_level > K_MAX_EW) return false;
    }
    if (pools > K_MAX_LEVELS || res > K_MAX_RES || idx > K_MAX_IDX) return false;
    if (pools == 0) return allow_stream && ew_total <= K_MAX_STREAM_EW;
    // level-0 element-wise operations
    int32_t ew0 = 0;
    for (int32_t i = first_op; i < first_op + n_ops && op_is_elementwise(s->ops[i].kind); ++i) ++ew0;
    return ew0 <= K_MAX_EW;
}

static int32_t count_pools(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    int32_t n = 0;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) n += !op_is_elementwise(s->ops[i].kind);
    return n;
}

static bool direct_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    if (count_pools(s, first_op, n_ops) != 1) return false;
    const int32_t vec = vec_of(s);
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (op_is_elementwise(op.kind)) continue;
        if (op.kh != op.sh || op.kw != op.sw || op.ph != 0 || op.pw != 0) return false;
        if (op.in_w % vec != 0 || vec % op.kw != 0) return false;
        if (op.kh > 4 || (op.kw != 1 && op.kw != 2 && op.kw != 4 && op.kw != 8)) return false;
    }
    int32_t pre = 0, post = 0;
    bool seen = false;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) { seen = true; continue; }
        if (op.kind == OP_AVGNORM) continue;
        (seen ? post : pre)++;
    }
    return pre <= K_MAX_EW && post <= K_MAX_EW;
}

// Resource consumption of a candidate sequence (Section 4.1): the on-chip bytes of the
// smallest useful tile, including the overlap that padding / k > s adds at every level.
static uint64_t seq_min_lds(const bs_stack *s, int32_t first_op, int32_t n_ops, int32_t threads)
{
    if (count_pools(s, first_op, n_ops) == 0) return 0;
    if (direct_applicable(s, first_op, n_ops) && s->opts.force_variant != BS_VARIANT_LDS_TILE) return 0;
    const Op &last = s->ops[first_op + n_ops - 1];
    int32_t th, tw;
    min_tile(last.out_h, last.out_w, threads, th, tw);
    LdsGeom g;
    const int32_t vec0 = (s->ops[first_op].in_w % vec_of(s) == 0) ? vec_of(s) : 1;
    lds_geometry(s, first_op, n_ops, th, tw, 1, vec0, g);
    return g.lds_bytes;
}

static uint64_t seq_smallest_lds(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    LdsGeom g;
    lds_geometry(s, first_op, n_ops, 1, 1, 1, 1, g);
    return g.lds_bytes;
}

// ---------------------------------------------------------------------------
// Fill the kernel argument blocks.
// ---------------------------------------------------------------------------
static void fill_ew(const bs_stack *s, const Op &op, Sequence &q, EwOp &e)
{
    e.kind = op.kind;
    e.arg = 0;
    if (op.kind == OP_BN) e.arg = op.param_off;
    if (op.kind == OP_ADD) {
        int32_t slot = -1;
        for (int32_t j = 0; j < q.n_res; ++j)
            if (q.res_map[j] == op.res_slot) slot = j;
        if (slot < 0) {
            slot = q.n_res++;
            q.res_map[slot] = op.res_slot;
        }
        e.arg = slot;
    }
    (void)s;
}

static PoolK make_pool(const Op &op, const Op *norm, Sequence &q)
{
    PoolK p{};
    p.kind = op.kind;
    p.kh = op.kh; p.kw = op.kw; p.sh = op.sh; p.sw = op.sw; p.ph = op.ph; p.pw = op.pw;
    p.count_include_pad = op.count_include_pad;
    p.inv_kk = 1.0f / (float)(op.kh * op.kw);
    p.idx_slot = -1;
    if (op.idx_slot >= 0) {
        p.idx_slot = q.n_idx++;
        q.idx_map[p.idx_slot] = op.idx_slot;
    }
    (void)norm;
    return p;
}

static void plan_stream(const bs_stack *s, Sequence &q)
{
    q.variant = BS_VARIANT_STREAM;
    const int64_t hw = q.in_shape[2] * q.in_shape[3];
    const int64_t total = q.in_shape[0] * q.in_shape[1] * hw;
    const int32_t vec = (hw % vec_of(s) == 0) ? vec_of(s) : 1;
    q.vec = vec;
    StreamK &k = q.stream;
    k = StreamK{};
    k.n_ew = 0;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) fill_ew(s, s->ops[i], q, k.ew[k.n_ew++]);
    k.total = (uint32_t)(total / vec);
    k.C = (int32_t)q.in_shape[1];
    k.div_plane = make_fastdiv((uint32_t)(hw / vec));
    k.div_c = make_fastdiv((uint32_t)k.C);
    const int64_t per_group = (int64_t)q.threads * 4;  // four 128-bit accesses per thread
    q.grid = (k.total + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.redundancy = 1.0;
    q.tile_rows = q.tile_cols = 0;
    q.planes_per_group = 0;
}

static void plan_direct(const bs_stack *s, Sequence &q)
{
    q.variant = BS_VARIANT_POOL_DIRECT;
    PoolDirectK &k = q.direct;
    k = PoolDirectK{};
    const int32_t vec = vec_of(s);
    q.vec = vec;
    bool seen = false;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            k.pool = make_pool(op, nullptr, q);
            k.H = op.in_h; k.W = op.in_w; k.Ho = op.out_h; k.Wo = op.out_w;
            seen = true;
        } else if (op.kind != OP_AVGNORM) {
            if (seen) fill_ew(s, op, q, k.post[k.n_post++]);
            else fill_ew(s, op, q, k.pre[k.n_pre++]);
        }
    }
    k.C = (int32_t)q.in_shape[1];
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    const int32_t wv = k.W / vec;
    k.total = (uint32_t)(planes * k.Ho * wv);
    k.div_wv = make_fastdiv((uint32_t)wv);
    k.div_ho = make_fastdiv((uint32_t)k.Ho);
    k.div_c = make_fastdiv((uint32_t)k.C);
    const int64_t per_group = (int64_t)q.threads * 2;  // two units (kh rows each) per thread
    q.grid = ((int64_t)k.total + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.redundancy = (double)(k.Ho * k.pool.kh) / (double)k.H;
    q.tile_rows = q.tile_cols = 0;
    q.planes_per_group = 0;
    q.n_levels = 1;
}

static bool audit_lds(const Sequence &q);

static bs_status plan_lds(const bs_stack *s, Sequence &q, const bs_plan_options &o, const Limits &lim)
{
    q.variant = BS_VARIANT_LDS_TILE;
    const Op &last = s->ops[q.first_op + q.n_ops - 1];
    const int32_t HL = last.out_h, WL = last.out_w;
    const int32_t vec0 = (s->ops[q.first_op].in_w % vec_of(s) == 0) ? vec_of(s) : 1;
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    const uint64_t budget = lim.max_lds_bytes;

    int32_t best_th = 0, best_tw = 0, best_ppg = 0;
    double best_score = 1e300;
    LdsGeom g;
    auto consider = [&](int32_t th, int32_t tw, int32_t ppg) {
        if (th < 1 || tw < 1 || ppg < 1 || th > HL || tw > WL || ppg > planes) return;
        lds_geometry(s, q.first_op, q.n_ops, th, tw, ppg, vec0, g);
        if (g.lds_bytes > budget) return;
        const int64_t nth = (HL + th - 1) / th, ntw = (WL + tw - 1) / tw;
        const int64_t grid = nth * ntw * ((planes + ppg - 1) / ppg);
        // cost model: redundant loads, ragged last tile, idle lanes in tiny tiles, too few
        // work-groups to fill the chip, and a mild preference for smaller LDS (occupancy).
        double score = g.redundancy;
        score *= (double)(nth * th) / HL * (double)(ntw * tw) / WL;
        const double outs = (double)th * tw * ppg;
        if (outs < q.threads) score *= 1.0 + 0.5 * (q.threads - outs) / q.threads;
        const double want = 4.0 * std::max(1, lim.num_cus);
        if ((double)grid < want) score *= 1.0 + 0.25 * (want - grid) / want;
        score *= 1.0 + 0.15 * (double)g.lds_bytes / (double)std::max<uint64_t>(budget, 1);
        if (tw != WL) score *= 1.05;
        if (score < best_score) {
            best_score = score;
            best_th = th; best_tw = tw; best_ppg = ppg;
        }
    };
    if (o.tile_rows > 0 || o.tile_cols > 0 || o.planes_per_group > 0) {
        consider(o.tile_rows > 0 ? std::min(o.tile_rows, HL) : HL,
                 o.tile_cols > 0 ? std::min(o.tile_cols, WL) : WL,
                 o.planes_per_group > 0 ? (int32_t)std::min<int64_t>(o.planes_per_group, planes) : 1);
    } else {
        std::vector<int32_t> tws, ths;
        for (int32_t d = 1; d <= 16; d *= 2) tws.push_back((WL + d - 1) / d);
        for (int32_t t : {1, 2, 4, 8, 16, 32}) if (t < WL) tws.push_back(t);
        for (int32_t d = 1; d <= HL; ++d) {
            int32_t t = (HL + d - 1) / d;
            if (ths.empty() || ths.back() != t) ths.push_back(t);
        }
        for (int32_t tw : tws)
            for (int32_t th : ths) {
                consider(th, tw, 1);
                if (th == HL && tw == WL)
                    for (int32_t ppg : {2, 4, 8, 16}) consider(th, tw, ppg);
            }
    }
    if (best_th == 0) return BS_ERR_NO_FIT;

    lds_geometry(s, q.first_op, q.n_ops, best_th, best_tw, best_ppg, vec0, g);
    q.tile_rows = best_th;
    q.tile_cols = best_tw;
    q.planes_per_group = best_ppg;
    q.vec = vec0;
    q.lds_bytes = g.lds_bytes;
    q.redundancy = g.redundancy;
    q.n_levels = g.L;
    int32_t sprod_h = 1, sprod_w = 1;
    for (int l = 1; l <= g.L; ++l) { sprod_h *= g.dh[l].s; sprod_w *= g.dw[l].s; }
    q.halo_rows = std::max(0, g.rows[0] - best_th * sprod_h);
    q.halo_cols = std::max(0, g.cols[0] - best_tw * sprod_w);

    LdsSeqK &k = q.lds;
    k = LdsSeqK{};
    k.n_levels = g.L;
    k.NC = (int32_t)planes;
    k.C = (int32_t)q.in_shape[1];
    k.TH = best_th; k.TW = best_tw;
    k.tiles_h = (HL + best_th - 1) / best_th;
    k.tiles_w = (WL + best_tw - 1) / best_tw;
    k.PPG = best_ppg;
    k.vec = vec0;
    k.div_tiles_w = make_fastdiv((uint32_t)k.tiles_w);
    k.div_tiles_hw = make_fastdiv((uint32_t)(k.tiles_w * k.tiles_h));
    k.div_c = make_fastdiv((uint32_t)k.C);
    q.grid = (int64_t)k.tiles_h * k.tiles_w * ((planes + best_ppg - 1) / best_ppg);
    int level = 0;
    for (int l = 0; l <= g.L; ++l) {
        LevelK &lv = k.level[l];
        lv.H = g.H[l]; lv.W = g.W[l];
        lv.rows_max = g.rows[l];
        lv.pitch = g.cols[l];
        lv.plane_stride = lv.rows_max * lv.pitch;
        lv.buf_off = (l & 1) ? (int32_t)g.buf_floats[0] : 0;
        lv.n_ew = 0;
        const uint32_t v = (l == 0) ? (uint32_t)vec0 : 1u;
        lv.div_pitch = make_fastdiv((uint32_t)lv.pitch / v);
        lv.div_plane = make_fastdiv((uint32_t)lv.plane_stride / v);
    }
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            ++level;
            k.pool[level] = make_pool(op, nullptr, q);
        } else if (op.kind != OP_AVGNORM) {
            LevelK &lv = k.level[level];
            fill_ew(s, op, q, lv.ew[lv.n_ew++]);
        }
    }
    if (!audit_lds(q)) return BS_ERR_NO_FIT;
    return BS_OK;
}

// Bounds audit of an LDS sequence, run on the host at plan time with the very function the
// kernel uses for its geometry: every region lies inside its plane and inside the LDS buffer
// reserved for its level, every pooling window's in-range cells lie inside the region cached
// from the level below, and index outputs in the middle of a sequence are covered without gaps.
// A plan that fails it is never launched.
static bool audit_lds(const Sequence &q)
{
    const LdsSeqK &k = q.lds;
    const int32_t L = k.n_levels;
    const uint64_t lds_floats = q.lds_bytes / sizeof(float);
    if (L < 1 || L > K_MAX_LEVELS || k.PPG < 1 || k.TH < 1 || k.TW < 1) return false;
    for (int l = 0; l < L; ++l) {
        const LevelK &lv = k.level[l];
        if (lv.plane_stride != lv.rows_max * lv.pitch) return false;
        if ((uint64_t)lv.buf_off + (uint64_t)k.PPG * lv.plane_stride > lds_floats) return false;
        if (l == 0 && k.vec > 1 && (lv.pitch % k.vec != 0 || lv.W % k.vec != 0 || lv.buf_off % 4 != 0)) return false;
    }
    for (int pass = 0; pass < 2; ++pass) {  // rows with tj = 0, then columns with ti = 0
        const int32_t n_tiles = pass == 0 ? k.tiles_h : k.tiles_w;
        for (int32_t t = 0; t < n_tiles; ++t) {
            const int32_t ti = pass == 0 ? t : 0, tj = pass == 0 ? 0 : t;
            for (int l = 0; l <= L; ++l) {
                const Region g = region_at(k, ti, tj, l);
                const int32_t lo = pass == 0 ? g.r_lo : g.c_lo, hi = pass == 0 ? g.r_hi : g.c_hi;
                const int32_t size = pass == 0 ? k.level[l].H : k.level[l].W;
                const int32_t cap = pass == 0 ? k.level[l].rows_max : k.level[l].pitch;
                if (lo < 0 || hi <= lo || hi > size || hi - lo > cap) return false;
                if (l == 0 && pass == 1 && k.vec > 1 && (lo % k.vec || hi % k.vec)) return false;
                if (l == 0) continue;
                const Region pg = region_at(k, ti, tj, l - 1);
                const PoolK &p = k.pool[l];
                const int32_t plo = pass == 0 ? pg.r_lo : pg.c_lo, phi = pass == 0 ? pg.r_hi : pg.c_hi;
                const int32_t psize = pass == 0 ? k.level[l - 1].H : k.level[l - 1].W;
                const int32_t kk = pass == 0 ? p.kh : p.kw, ss = pass == 0 ? p.sh : p.sw, pp = pass == 0 ? p.ph : p.pw;
                for (int32_t o = lo; o < hi; ++o) {
                    const int32_t s0 = std::max(o * ss - pp, 0), s1 = std::min(o * ss - pp + kk, psize);
                    if (s0 >= s1 || s0 < plo || s1 > phi) return false;
                }
                if (p.idx_slot >= 0 && l < L && t + 1 < n_tiles) {
                    const Region nx = pass == 0 ? region_at(k, ti + 1, tj, l) : region_at(k, ti, tj + 1, l);
                    const int32_t nlo = pass == 0 ? nx.r_lo : nx.c_lo;
                    if (nlo > hi || nlo < lo) return false;
                }
                if (p.idx_slot >= 0 && l < L && t + 1 == n_tiles && hi != size) return false;
            }
        }
    }
    return true;
}

// ---------------------------------------------------------------------------
// Steps -> sequences (Section 4.1): steps are appended to the current sequence
// while its resource consumption stays within the device limit; otherwise the
// sequence is closed and a new one starts with that step.  The trailing sequence
// is kept.  A step-count cap implements the strategies of Section 5.1.
// ---------------------------------------------------------------------------
bs_status group_sequences(bs_stack *s, const bs_plan_options &o, const Limits &lim)
{
    s->seqs.clear();
    const int32_t threads = o.threads_per_group > 0 ? o.threads_per_group : 256;
    const bool per_layer = o.breadth_first != 0;
    std::vector<SeqDraft> drafts;
    SeqDraft cur{0, 0};
    auto range_ops = [&](const SeqDraft &d, int32_t &first_op, int32_t &n_ops) {
        first_op = s->steps[d.first_step].first_op;
        const Step &lst = s->steps[d.first_step + d.n_steps - 1];
        n_ops = lst.first_op + lst.n_ops - first_op;
    };
    for (int32_t i = 0; i < (int32_t)s->steps.size(); ++i) {
        if (cur.n_steps == 0) {
            cur = SeqDraft{i, 1};
        } else {
            SeqDraft trial{cur.first_step, cur.n_steps + 1};
            int32_t fo, no;
            range_ops(trial, fo, no);
            bool fits = !per_layer;
            if (fits && o.max_steps_per_sequence > 0 && trial.n_steps > o.max_steps_per_sequence) fits = false;
            if (fits && !seq_capacity_ok(s, fo, no, true)) fits = false;
            if (fits && seq_min_lds(s, fo, no, threads) > lim.max_lds_bytes) fits = false;
            if (fits) {
                cur = trial;
            } else {
                drafts.push_back(cur);
                cur = SeqDraft{i, 1};
            }
        }
        // a single step must be executable on its own
        if (cur.n_steps == 1) {
            int32_t fo, no;
            range_ops(cur, fo, no);
            if (!seq_capacity_ok(s, fo, no, true)) return BS_ERR_UNSUPPORTED;
            if (seq_min_lds(s, fo, no, threads) > lim.max_lds_bytes &&
                seq_smallest_lds(s, fo, no) > lim.max_lds_bytes)
                return BS_ERR_NO_FIT;
        }
    }
    if (cur.n_steps > 0) drafts.push_back(cur);

    const size_t es = dtype_size(s->dtype);
    uint64_t max_inter = 0;
    for (size_t di = 0; di < drafts.size(); ++di) {
        Sequence q;
        q.first_step = drafts[di].first_step;
        q.n_steps = drafts[di].n_steps;
        range_ops(drafts[di], q.first_op, q.n_ops);
        q.first_layer = s->ops[q.first_op].layer;
        q.n_layers = s->ops[q.first_op + q.n_ops - 1].layer - q.first_layer + 1;
        q.threads = threads;
        for (int32_t st = q.first_step; st < q.first_step + q.n_steps; ++st) s->steps[st].sequence = (int32_t)di;
        const Op &fo = s->ops[q.first_op], &lo = s->ops[q.first_op + q.n_ops - 1];
        q.in_shape[0] = q.out_shape[0] = s->in_shape[0];
        q.in_shape[1] = q.out_shape[1] = s->in_shape[1];
        q.in_shape[2] = fo.in_h; q.in_shape[3] = fo.in_w;
        q.out_shape[2] = lo.out_h; q.out_shape[3] = lo.out_w;
        const int32_t pools = count_pools(s, q.first_op, q.n_ops);
        q.n_levels = pools;
        bs_status st = BS_OK;
        if (pools == 0) {
            plan_stream(s, q);
        } else if (direct_applicable(s, q.first_op, q.n_ops) && o.force_variant != BS_VARIANT_LDS_TILE) {
            plan_direct(s, q);
        } else {
            st = plan_lds(s, q, o, lim);
        }
        if (st != BS_OK) return st;
        if (di + 1 < drafts.size()) {
            uint64_t bytes = (uint64_t)q.out_shape[0] * q.out_shape[1] * q.out_shape[2] * q.out_shape[3] * es;
            max_inter = std::max(max_inter, bytes);
        }
        s->seqs.push_back(q);
    }
    s->ws_half_bytes = (max_inter + 255) / 256 * 256;
    const size_t n = s->seqs.size();
    s->workspace_bytes = n <= 1 ? 0 : (n == 2 ? s->ws_half_bytes : 2 * s->ws_half_bytes);
    return BS_OK;
}

}  // namespace bs

using namespace bs;

extern "C" {

bs_status bs_stack_plan(bs_stack *stack, const bs_plan_options *opts)
{
    if (!stack) return BS_ERR_NULL;
    bs_plan_options o{};
    if (opts) o = *opts;
    if (o.max_steps_per_sequence < 0 || o.num_cus < 0 || o.tile_rows < 0 || o.tile_cols < 0 ||
        o.planes_per_group < 0)
        return BS_ERR_PARAM;
    if (o.threads_per_group != 0 &&
        (o.threads_per_group < 64 || o.threads_per_group > 512 || o.threads_per_group % 64 != 0))
        return BS_ERR_PARAM;
    if (o.force_variant < 0 || o.force_variant > BS_VARIANT_LDS_TILE) return BS_ERR_PARAM;
    if (o.max_lds_bytes > 64 * 1024) return BS_ERR_PARAM;

    stack->planned = stack->device_planned = false;
    free_params(stack);

    Limits lim;
    lim.max_lds_bytes = o.max_lds_bytes;
    lim.num_cus = o.num_cus;
    int device = -1;
    if (!o.host_only) {
        Limits dev;
        bs_status st = device_limits(&dev, &device);
        if (st != BS_OK) return st;
        if (lim.num_cus == 0) lim.num_cus = dev.num_cus;
    }
    if (lim.num_cus == 0) lim.num_cus = 256;
    // Default on-chip budget per work-group: a quarter of the 64 KiB a group may address
    // keeps several groups resident per compute unit (the paper caps shared memory well
    // below what the device offers for the same reason, Section 4.4).
    if (lim.max_lds_bytes == 0) lim.max_lds_bytes = 32 * 1024;

    stack->opts = o;
    bs_status st;
    try {
        st = build_operations(stack);
        if (st == BS_OK) st = group_steps(stack);
        if (st == BS_OK) st = group_sequences(stack, o, lim);
    } catch (const std::bad_alloc &) {
        st = BS_ERR_ALLOC;
    }
    if (st != BS_OK) return st;

    const size_t es = dtype_size(stack->dtype);
    auto numel = [](const int64_t *sh) { return (uint64_t)sh[0] * sh[1] * sh[2] * sh[3]; };
    uint64_t bytes = numel(stack->in_shape) * es + numel(stack->out_shape) * es;
    for (int32_t i = 0; i < stack->n_res; ++i) bytes += numel(stack->res_shape[i]) * es;
    for (int32_t i = 0; i < stack->n_idx; ++i) bytes += numel(stack->idx_shape[i]) * 4;
    stack->algorithmic_bytes = bytes;
    stack->planned = true;

    if (!o.host_only) {
        st = upload_params(stack);
        if (st != BS_OK) return st;
        stack->device = device;
        stack->device_planned = true;
    }
    return BS_OK;
}

bs_status bs_stack_plan_info(const bs_stack *stack, bs_plan_info *info)
{
    if (!stack || !info) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    bs_plan_info r{};
    r.n_operations = (int32_t)stack->ops.size();
    r.n_steps = (int32_t)stack->steps.size();
    r.n_sequences = (int32_t)stack->seqs.size();
    r.device_planned = stack->device_planned ? 1 : 0;
    r.workspace_bytes = stack->workspace_bytes;
    r.algorithmic_bytes = stack->algorithmic_bytes;
    *info = r;
    return BS_OK;
}

bs_status bs_stack_step_info(const bs_stack *stack, int32_t step, bs_step_info *info)
{
    if (!stack || !info) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    if (step < 0 || step >= (int32_t)stack->steps.size()) return BS_ERR_RANGE;
    const Step &st = stack->steps[step];
    info->first_operation = st.first_op;
    info->n_operations = st.n_ops;
    info->pool_operation = st.pool_op;
    info->sequence = st.sequence;
    return BS_OK;
}

bs_status bs_stack_sequence_info(const bs_stack *stack, int32_t sequence, bs_sequence_info *info)
{
    if (!stack || !info) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    if (sequence < 0 || sequence >= (int32_t)stack->seqs.size()) return BS_ERR_RANGE;
    const Sequence &q = stack->seqs[sequence];
    bs_sequence_info r{};
    r.first_step = q.first_step; r.n_steps = q.n_steps;
    r.first_layer = q.first_layer; r.n_layers = q.n_layers;
    r.variant = q.variant;
    r.n_levels = q.n_levels;
    r.tile_rows = q.tile_rows; r.tile_cols = q.tile_cols;
    r.planes_per_group = q.planes_per_group;
    r.halo_rows = q.halo_rows; r.halo_cols = q.halo_cols;
    r.threads_per_group = q.threads;
    r.grid = q.grid;
    r.lds_bytes = q.lds_bytes;
    std::memcpy(r.in_shape, q.in_shape, sizeof(r.in_shape));
    std::memcpy(r.out_shape, q.out_shape, sizeof(r.out_shape));
    r.redundancy = q.redundancy;
    *info = r;
    return BS_OK;
}

const char *bs_stack_operation_name(const bs_stack *stack, int32_t op)
{
    if (!stack || !stack->planned || op < 0 || op >= (int32_t)stack->ops.size()) return nullptr;
    switch (stack->ops[op].kind) {
    case OP_BN: return "BatchNorm";
    case OP_RELU: return "ReLU";
    case OP_ADD: return "Add";
    case OP_MAXPOOL: return "MaxPooling";
    case OP_AVGSUM: return "AvgPooling";
    case OP_AVGNORM: return "AvgNormalization";
    }
    return nullptr;
}

uint64_t bs_stack_workspace_bytes(const bs_stack *stack)
{
    return (stack && stack->planned) ? stack->workspace_bytes : 0;
}

}  // extern "C"
