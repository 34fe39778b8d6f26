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
            // tables start at a multiple of 8 floats: the channels-last kernels read them with
            // 128-bit loads
            while (s->host_params.size() % 8 != 0) s->host_params.push_back(0.0f);
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
        case BS_LEAKY_RELU:
            op.kind = OP_LEAKY;
            op.param_off = (int32_t)s->host_params.size();
            s->host_params.push_back(L.desc.negative_slope);
            s->host_params.push_back(0.0f);
            s->ops.push_back(op);
            break;
        case BS_CLAMP:
            op.kind = OP_CLAMP;
            op.param_off = (int32_t)s->host_params.size();
            s->host_params.push_back(L.desc.clamp_min);
            s->host_params.push_back(L.desc.clamp_max);
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
            op.ceil = d.ceil_mode ? 1 : 0;
            if (d.kind == BS_MAXPOOL) {
                op.kind = OP_MAXPOOL;
                if (d.return_indices) op.idx_slot = idx++;
                s->ops.push_back(op);
            } else {
                op.kind = OP_AVGSUM;
                // 0: in-range cells; 1: kh * kw; 2: the window cells inside the padded plane (ceil
                // mode with count_include_pad: a last window may overhang the padding)
                op.count_include_pad = d.count_include_pad ? (L.desc.ceil_mode ? 2 : 1) : 0;
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
// Tile geometry of an LDS sequence.  A work-group owns a TH x TW tile of the last
// level.  The rectangle it keeps of level l-1 holds exactly the windows of its
// rectangle of level l:  extent[l-1] = (extent[l] - 1) * stride + kernel, and its
// origin is origin[l] * stride - pad (possibly outside the plane: those cells are the
// pooling operation's padding).  Column extents of levels >= 1 are rounded up to 4,
// the strip of outputs one lane produces.  Rows and columns are independent.
// ---------------------------------------------------------------------------
struct Dim {
    int32_t k, s, p;
};

struct LdsGeom {
    int32_t L = 0;
    std::vector<Dim> dh, dw;          // index 1..L
    std::vector<int32_t> H, W;        // index 0..L
    std::vector<int32_t> rows, cols;  // region extents per level
    std::vector<int32_t> pitch;
    int32_t delta0 = 0, nvr = 0;      // level-0 LDS row: starts delta0 columns before the rectangle, nvr vectors
    uint64_t lds_bytes = 0;
    uint64_t buf_floats[2] = {0, 0};
    double redundancy = 1.0;
};

static inline int32_t round4(int32_t v) { return (v + 3) / 4 * 4; }

// in-plane cells of [origin - before, origin - before + extent) summed over all tiles, along
// one dimension
static uint64_t loaded_extent(const std::vector<Dim> &d, const std::vector<int32_t> &size, int32_t tile,
                              int32_t before, int32_t extent)
{
    const int L = (int)d.size() - 1;
    const int32_t n_tiles = (size[L] + tile - 1) / tile;
    uint64_t sum = 0;
    for (int32_t t = 0; t < n_tiles; ++t) {
        int64_t o = (int64_t)t * tile;
        for (int l = L; l >= 1; --l) o = o * d[l].s - d[l].p;
        o -= before;
        const int64_t lo = std::max<int64_t>(o, 0), hi = std::min<int64_t>(o + extent, size[0]);
        if (hi > lo) sum += (uint64_t)(hi - lo);
    }
    return sum;
}

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
    const int L = g.L = (int32_t)g.dh.size() - 1;
    g.rows.assign(L + 1, 0);
    g.cols.assign(L + 1, 0);
    g.pitch.assign(L + 1, 0);
    g.rows[L] = th;
    g.cols[L] = round4(tw);
    for (int l = L; l >= 1; --l) {
        g.rows[l - 1] = (g.rows[l] - 1) * g.dh[l].s + g.dh[l].k;
        g.cols[l - 1] = (g.cols[l] - 1) * g.dw[l].s + g.dw[l].k;
        if (l - 1 >= 1) g.cols[l - 1] = round4(g.cols[l - 1]);
    }
    // level-0 LDS rows start at the 128-bit global vector holding the rectangle's first column
    int64_t c00 = 0;
    for (int l = L; l >= 1; --l) c00 = c00 * g.dw[l].s - g.dw[l].p;
    g.delta0 = vec0 > 1 ? (int32_t)(((c00 % vec0) + vec0) % vec0) : 0;
    g.nvr = vec0 > 1 ? (g.delta0 + g.cols[0] + vec0 - 1) / vec0 : g.cols[0];
    g.buf_floats[0] = g.buf_floats[1] = 0;
    for (int l = 0; l <= L; ++l) {
        g.pitch[l] = round4(g.cols[l]);
        if (l == 0 && vec0 > 1) g.pitch[0] = g.nvr * vec0 + 4;  // + slack for aligned over-reads
        if (l == L) continue;  // level L goes to memory, not to LDS
        const uint64_t need = (uint64_t)ppg * g.rows[l] * g.pitch[l];
        g.buf_floats[l & 1] = std::max(g.buf_floats[l & 1], need);
    }
    g.lds_bytes = (g.buf_floats[0] + g.buf_floats[1]) * sizeof(float);
    const uint64_t rsum = loaded_extent(g.dh, g.H, th, 0, g.rows[0]);
    const uint64_t csum = loaded_extent(g.dw, g.W, tw, g.delta0, vec0 > 1 ? g.nvr * vec0 : g.cols[0]);
    g.redundancy = (double)rsum * (double)csum / ((double)g.H[0] * (double)g.W[0]);
}

// Does every cell of a pooling operation's input lie in some window?  (k >= s and the
// floor-mode remainder is absorbed by the padding.)  Needed to keep an index-producing
// max pool in the middle of a sequence: its whole output must then be computed by tiles.
static bool covers_input(const Op &op)
{
    if (op.ceil) return op.kh >= op.sh && op.kw >= op.sw;  // the extra last window reaches the plane's end
    auto ok = [](int32_t size, int32_t k, int32_t st, int32_t p) {
        return k >= st && ((size + 2 * p - k) % st) <= p;
    };
    return ok(op.in_h, op.kh, op.sh, op.ph) && ok(op.in_w, op.kw, op.sw, op.pw);
}

static int32_t vec_of(const bs_stack *s) { return s->dtype == BS_F32 ? 4 : 8; }

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

// Column block (elements per lane and row) of the disjoint-window kernel for a pooling operation: one
// 128-bit vector, or -- 16-bit storage and rows that are a multiple of 4 but not of 8 elements, the
// 28 x 28 planes of VGG and DenseNet -- one 64-bit vector; 0: rows that are neither.
static int32_t direct_vec(const bs_stack *s, const Op &op)
{
    const int32_t full = s->dtype == BS_F32 ? 4 : 8;
    if (op.in_w % full == 0) return full;
    return s->dtype != BS_F32 && op.in_w % 4 == 0 ? 4 : 0;
}

static bool direct_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    if (count_pools(s, first_op, n_ops) != 1) return false;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (op_is_elementwise(op.kind)) continue;
        if (op.kh != op.sh || op.kw != op.sw || op.ph != 0 || op.pw != 0) return false;
        if (op.ceil) return false;  // its last windows overhang the plane: the kernel reads whole windows
        const int32_t vec = direct_vec(s, op);
        if (vec == 0 || vec % op.kw != 0) return false;
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
static bool rows_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops, Sequence *fill);
static bool plane_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops);
static bool chain_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops, Sequence *fill);
// Fewest identical pooling blocks the chain kernel is used for.  Measured on 64 x 64 x 56 x 56, float32: one block 25 us
// (one-level sliding-window kernel: 22 us), two blocks 25 us (two-level kernel: 34 us), three 26 us, four 27 us.
#if !defined(BS_CHAIN_MIN)
#define BS_CHAIN_MIN 2
#endif

static uint64_t seq_min_lds(const bs_stack *s, int32_t first_op, int32_t n_ops, int32_t threads)
{
    if (count_pools(s, first_op, n_ops) == 0) return 0;
    if (direct_applicable(s, first_op, n_ops) && s->opts.force_variant != BS_VARIANT_LDS_TILE) return 0;
    if (rows_applicable(s, first_op, n_ops, nullptr) && s->opts.force_variant != BS_VARIANT_LDS_TILE) return 0;
    if (plane_applicable(s, first_op, n_ops) && s->opts.force_variant != BS_VARIANT_LDS_TILE) return 0;
    if (chain_applicable(s, first_op, n_ops, nullptr)) return 0;
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
    if (op.kind == OP_BN || op.kind == OP_LEAKY || op.kind == OP_CLAMP) e.arg = op.param_off;
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
    // planes that are no multiple of the vector width: vectors over the whole tensor (they may
    // straddle two planes) when the tensor is a whole number of vectors and a plane holds at
    // least one; the scalar kernel otherwise
    const bool flat = hw % vec_of(s) != 0 && total % vec_of(s) == 0 && hw >= vec_of(s);
    const int32_t vec = (hw % vec_of(s) == 0 || flat) ? vec_of(s) : 1;
    q.vec = vec;
    StreamK &k = q.stream;
    k = StreamK{};
    k.n_ew = 0;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) fill_ew(s, s->ops[i], q, k.ew[k.n_ew++]);
    k.total = (uint32_t)(total / vec);
    k.C = (int32_t)q.in_shape[1];
    k.flat = flat ? 1 : 0;
    k.div_plane = make_fastdiv((uint32_t)(flat ? hw : hw / vec));
    k.div_c = make_fastdiv((uint32_t)k.C);
    const int64_t per_group = (int64_t)q.threads * K_STREAM_U;
    q.grid = (k.total + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.redundancy = 1.0;
    q.tile_rows = q.tile_cols = 0;
    q.planes_per_group = 0;
}

// Does an element-wise list give the same value applied to a maximum as the maximum of the list
// applied to every cell?  True when no operation decreases as its input increases (BatchNorm
// with scales >= 0, ReLU, leaky ReLU with a slope >= 0, clamp; rounding to the storage type is
// of that kind too) -- then max_i f(x_i) = f(max_i x_i), the same float32 value, up to the sign
// of a zero -- and the list holds a ReLU, which makes every zero +0.
static bool commutes_with_max(const bs_stack *s, const EwOp *ew, int32_t n, int32_t C)
{
    bool monotone = true, relu = false;
    for (int32_t j = 0; j < n && monotone; ++j) {
        const EwOp &e = ew[j];
        if (e.kind == OP_BN) {
            for (int32_t c = 0; c < C; ++c) monotone = monotone && s->host_params[(size_t)e.arg + c] >= 0.0f;
        } else if (e.kind == OP_LEAKY) {
            monotone = s->host_params[(size_t)e.arg] >= 0.0f;
        } else if (e.kind == OP_RELU) {
            relu = true;
        } else if (e.kind != OP_CLAMP) {
            monotone = false;  // a residual Add differs from cell to cell
        }
    }
    return monotone && relu;
}

// Channels-last sequence: element-wise only, or one pooling step.
static bs_status plan_nhwc(const bs_stack *s, Sequence &q)
{
    NhwcK &k = q.nhwc;
    k = NhwcK{};
    const int32_t C = (int32_t)q.in_shape[1];
    const int32_t vec = (C % vec_of(s) == 0) ? vec_of(s) : 1;
    q.vec = vec;
    bool seen = false;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            if (seen) return BS_ERR_UNSUPPORTED;  // one pooling operation per channels-last sequence
            k.pool = make_pool(op, nullptr, q);
            k.H = op.in_h; k.W = op.in_w; k.Ho = op.out_h; k.Wo = op.out_w;
            seen = true;
        } else if (op.kind != OP_AVGNORM) {
            if (seen) {
                if (k.n_post >= K_MAX_EW) return BS_ERR_UNSUPPORTED;
                fill_ew(s, op, q, k.post[k.n_post++]);
            } else {
                if (k.n_pre >= (count_pools(s, q.first_op, q.n_ops) ? K_MAX_EW : K_MAX_STREAM_EW))
                    return BS_ERR_UNSUPPORTED;
                fill_ew(s, op, q, k.pre[k.n_pre++]);
            }
        }
    }
    k.C = C;
    // Maximum first.  Element-wise operations that never decrease when their input increases
    // (BatchNorm with scales >= 0, ReLU, leaky ReLU with a slope >= 0, clamp; rounding to the
    // storage type is of that kind too) commute with the maximum: max_i f(x_i) = f(max_i x_i),
    // the same float32 value.  Only the sign of a zero could differ, and not once a ReLU has
    // made every zero +0.  So when no argmax is wanted and the list before a max pool is of
    // that kind and holds a ReLU, the pool runs on the raw input and the list on its output:
    // once per output instead of once per window cell.
    if (seen && k.pool.kind == OP_MAXPOOL && k.pool.idx_slot < 0 && k.n_pre > 0 && k.n_pre + k.n_post <= K_MAX_EW &&
        commutes_with_max(s, k.pre, k.n_pre, C)) {
        EwOp moved[K_MAX_EW];
        int32_t m = 0;
        for (int32_t j = 0; j < k.n_pre; ++j) moved[m++] = k.pre[j];
        for (int32_t j = 0; j < k.n_post; ++j) moved[m++] = k.post[j];
        for (int32_t j = 0; j < m; ++j) k.post[j] = moved[j];
        k.n_post = m;
        k.n_pre = 0;
    }
    if (!seen) {
        k.H = k.Ho = (int32_t)q.in_shape[2];
        k.W = k.Wo = (int32_t)q.in_shape[3];
    }
    q.variant = seen ? BS_VARIANT_NHWC_POOL : BS_VARIANT_NHWC_STREAM;
    if (seen) {
        // pooling over the whole plane, the plane not tiny: staged through LDS, one work-group per
        // image and group of channel vectors
        const int64_t hw = (int64_t)k.H * k.W;
        const int32_t cv = nhwc_plane_group(hw, vec, k.pool, k.H, k.W, k.Ho, k.Wo);
        if (cv > 0) {
            const int32_t groups = (C / vec + cv - 1) / cv;
            k.cv_group = cv;
            k.total = (uint32_t)(q.in_shape[0] * groups);
            k.div_cv = make_fastdiv((uint32_t)(C / vec));
            k.div_wo = make_fastdiv((uint32_t)groups);
            k.div_ho = make_fastdiv(1u);
            q.variant = BS_VARIANT_NHWC_POOL;
            q.threads = 256;
            q.grid = (int64_t)k.total;
            q.lds_bytes = (uint64_t)hw * cv * vec * 4;
            q.redundancy = 1.0;
            q.tile_rows = q.tile_cols = 1;
            q.planes_per_group = cv * vec;
            q.n_levels = 1;
            return BS_OK;
        }
    }
    // a lane takes one channel vector of a block of ohb x owb output pixels (1 x 1: one pixel)
    int32_t ohb = 1, owb = 1;
    if (seen) nhwc_block(k.pool, vec, s->dtype, ohb, owb);
    const int32_t bh = (k.Ho + ohb - 1) / ohb, bw = (k.Wo + owb - 1) / owb;
    k.total = (uint32_t)(q.in_shape[0] * (int64_t)bh * bw * (C / vec));
    k.div_cv = make_fastdiv((uint32_t)(C / vec));
    k.div_wo = make_fastdiv((uint32_t)bw);
    k.div_ho = make_fastdiv((uint32_t)bh);
    q.tile_rows = ohb;
    q.tile_cols = owb;
    q.threads = std::min(q.threads, 256);
    const int64_t per_group = (int64_t)q.threads * (seen ? 1 : K_STREAM_U);
    q.grid = ((int64_t)k.total + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.redundancy = !seen ? 1.0 : (double)bh * ((ohb - 1) * k.pool.sh + k.pool.kh) * bw * ((owb - 1) * k.pool.sw + k.pool.kw) /
                                      ((double)k.H * k.W);
    q.planes_per_group = 0;
    q.n_levels = seen ? 1 : 0;
    return BS_OK;
}

// Channels-last sequence of two pooling steps: one kernel, tiles of both planes in LDS.
// BS_ERR_UNSUPPORTED when the pair is not one the kernel exists for (the steps then run one by one).
static bs_status plan_nhwc_tile2(const bs_stack *s, Sequence &q, const bs_plan_options &o, const Limits &lim)
{
    NhwcTile2K &k = q.nhwc2;
    k = NhwcTile2K{};
    const int32_t C = (int32_t)q.in_shape[1], vec = vec_of(s);
    if (C % vec != 0 || count_pools(s, q.first_op, q.n_ops) != 2) return BS_ERR_UNSUPPORTED;
    q.vec = vec;
    int32_t pools = 0;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            if (pools == 0) {
                if (op.idx_slot >= 0) return BS_ERR_UNSUPPORTED;  // picks inside the plane between the pools: tiles overlap there
                k.pool1 = make_pool(op, nullptr, q);
                k.H = op.in_h; k.W = op.in_w; k.H1 = op.out_h; k.W1 = op.out_w;
            } else {
                k.pool2 = make_pool(op, nullptr, q);
                if (op.in_h != k.H1 || op.in_w != k.W1) return BS_ERR_UNSUPPORTED;
                k.Ho = op.out_h; k.Wo = op.out_w;
            }
            ++pools;
        } else if (op.kind != OP_AVGNORM) {
            EwOp *list = pools == 0 ? k.pre : pools == 1 ? k.mid : k.post;
            int32_t &n = pools == 0 ? k.n_pre : pools == 1 ? k.n_mid : k.n_post;
            if (n >= K_MAX_EW) return BS_ERR_UNSUPPORTED;
            fill_ew(s, op, q, list[n++]);
        }
    }
    if (!nhwc_tile2_supported(k.pool1, k.pool2)) return BS_ERR_UNSUPPORTED;
    if (!nhwc_tile2_sizes_ok(k.H, k.W, C, 0, s->dtype) || !nhwc_tile2_sizes_ok(k.H1, k.W1, C, 0, s->dtype) ||
        !nhwc_tile2_sizes_ok(k.Ho, k.Wo, C, 0, s->dtype))
        return BS_ERR_UNSUPPORTED;
    k.C = C;
    // maximum first (see plan_nhwc): a list in front of a max pool that commutes with the maximum
    // runs once per pooled value, behind the pool
    auto move_behind = [&](EwOp *from, int32_t &n_from, EwOp *to, int32_t &n_to) {
        EwOp moved[K_MAX_EW];
        int32_t m = 0;
        for (int32_t j = 0; j < n_from; ++j) moved[m++] = from[j];
        for (int32_t j = 0; j < n_to; ++j) moved[m++] = to[j];
        for (int32_t j = 0; j < m; ++j) to[j] = moved[j];
        n_to = m;
        n_from = 0;
    };
    if (k.pool1.kind == OP_MAXPOOL && k.n_pre > 0 && k.n_pre + k.n_mid <= K_MAX_EW && commutes_with_max(s, k.pre, k.n_pre, C))
        move_behind(k.pre, k.n_pre, k.mid, k.n_mid);
    if (k.pool2.kind == OP_MAXPOOL && k.pool2.idx_slot < 0 && k.n_mid > 0 && k.n_mid + k.n_post <= K_MAX_EW &&
        commutes_with_max(s, k.mid, k.n_mid, C))
        move_behind(k.mid, k.n_mid, k.post, k.n_post);

    // The register kernel where it exists for this pair (plan option lane_exchange = -1: not used).
    // A work-group is the channel vectors that share a cache line and a chunk of output rows (tile_rows overrides its length).
    if (o.lane_exchange >= 0 && nhwc_rows2_supported(k, s->dtype)) {
        const int32_t cvn = C / vec;
        int32_t cvb = std::min(cvn, K_NHWC_ROWS_WAVES);
        while (cvn % cvb != 0) --cvb;
        k.cvb = cvb;
        k.cvgs = cvn / cvb;
        k.rc = std::min(o.tile_rows > 0 ? o.tile_rows : K_NHWC_ROWS_RC, k.Ho);
        k.chunks = (k.Ho + k.rc - 1) / k.rc;
        const int64_t total = q.in_shape[0] * (int64_t)k.chunks * k.cvgs;
        if (total <= 0x7fffffffll) {
            k.div_cvgs = make_fastdiv((uint32_t)k.cvgs);
            k.div_chunks = make_fastdiv((uint32_t)k.chunks);
            k.div_n = make_fastdiv((uint32_t)q.in_shape[0]);
            q.variant = BS_VARIANT_NHWC_ROWS;
            q.threads = 64 * cvb;
            q.grid = total;
            q.lds_bytes = 0;
            q.tile_rows = k.rc;
            q.tile_cols = k.Wo;
            q.planes_per_group = cvb * vec;
            // input rows a chunk settles against the rows it owns (k1 = 3, s1 = 1: two rows above, two below the chunk's)
            q.redundancy = (double)k.chunks * (k.rc * k.pool2.sh + 3) / (double)k.H;
            q.n_levels = 2;
            return BS_OK;
        }
    }
    // BatchNorm operations of the three lists, in order: the kernel stages their parameters in LDS
    {
        const EwOp *lists[3] = {k.pre, k.mid, k.post};
        const int32_t counts[3] = {k.n_pre, k.n_mid, k.n_post};
        for (int l = 0; l < 3; ++l) {
            k.bn_base[l] = k.n_bn;
            for (int32_t j = 0; j < counts[l]; ++j)
                if (lists[l][j].kind == OP_BN) k.bn_arg[k.n_bn++] = lists[l][j].arg;
        }
    }
    // Tile and channel group.  A lane has a fixed share of a tile (a few input cells, one block
    // per pooling level), so every tile takes about the same time whatever its size: the best
    // tile is the one that covers the output plane with the fewest work-group passes.
    // Candidates: channel groups that divide the pixel's vectors (at most 16 per work-group)
    // and tiles that leave no lane more than its share and fit the LDS budget; tile options
    // are upper bounds.  Small penalties for channel runs shorter than a 128-byte line and
    // for tiles that leave many lanes idle break ties.
    const int32_t cvn = C / vec;
    const uint64_t lds_cap = std::min<uint64_t>(64 * 1024, o.max_lds_bytes ? o.max_lds_bytes : 64 * 1024);
    double best = 0.0;
    int32_t bth = 0, btw = 0, bcvb = 0;
    for (int32_t cvb = std::min(cvn, 16); cvb >= 1; --cvb) {
        if (cvn % cvb != 0) continue;
        if (o.planes_per_group > 0 && cvb * vec != o.planes_per_group) continue;
        const int32_t pl = 256 / cvb;
        for (int32_t th = 1; th <= std::min(o.tile_rows > 0 ? o.tile_rows : 32, k.Ho); ++th)
            for (int32_t tw = 1; tw <= std::min(o.tile_cols > 0 ? o.tile_cols : 32, k.Wo); ++tw) {
                if (!nhwc_tile2_fits(k.pool1, k.pool2, th, tw, pl)) continue;
                if (nhwc_tile2_lds(k.pool1, k.pool2, th, tw, cvb, k.n_bn, vec) > lds_cap) continue;
                const int64_t tiles = (int64_t)((k.Ho + th - 1) / th) * ((k.Wo + tw - 1) / tw);
                double cost = (double)tiles * (cvn / cvb);
                if ((uint64_t)cvb * 16 < 128) cost *= 1.0 + 0.05 * (128.0 / (cvb * 16.0) - 1.0);
                cost *= 1.0 + 0.02 * (1.0 - (double)th * tw / pl);
                if (bth == 0 || cost < best) { best = cost; bth = th; btw = tw; bcvb = cvb; }
            }
    }
    if (bth == 0) return BS_ERR_UNSUPPORTED;
    int32_t r0[2], r1[2], cells[2], bw[2];
    nhwc_tile2_shape(k.pool1, k.pool2, bth, btw, r0, r1, cells, bw);
    q.lds_bytes = nhwc_tile2_lds(k.pool1, k.pool2, bth, btw, bcvb, k.n_bn, vec);
    k.TH = bth; k.TW = btw; k.cvb = bcvb; k.pl = 256 / bcvb;
    k.r0h = r0[0]; k.r0w = r0[1]; k.r1h = r1[0]; k.r1w = r1[1];
    k.lds1_off = (uint32_t)(cells[0] * bcvb);
    k.par_off = (uint32_t)((cells[0] + cells[1]) * bcvb);
    k.cvgs = cvn / bcvb;
    k.tiles_h = (k.Ho + bth - 1) / bth;
    k.tiles_w = (k.Wo + btw - 1) / btw;
    const int64_t total = q.in_shape[0] * (int64_t)k.tiles_h * k.tiles_w * k.cvgs;
    if (total > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    k.total_tiles = (uint32_t)total;
    k.div_cvb = make_fastdiv((uint32_t)k.cvb);
    k.div_r0w = make_fastdiv((uint32_t)k.r0w);
    k.div_bw1 = make_fastdiv((uint32_t)bw[0]);
    k.div_bw2 = make_fastdiv((uint32_t)bw[1]);
    k.div_n = make_fastdiv((uint32_t)q.in_shape[0]);
    k.div_tiles_w = make_fastdiv((uint32_t)k.tiles_w);
    k.div_tiles_h = make_fastdiv((uint32_t)k.tiles_h);
    q.variant = BS_VARIANT_NHWC_TILE;
    q.threads = 256;
    // work-groups: at most as many as the chip could hold at once by LDS, each with a run of
    // consecutive tiles (the launcher lowers the count to what the kernel's registers allow)
    {
        const int32_t resident = (int32_t)std::min<uint64_t>(8, (160 * 1024) / std::max<uint64_t>(q.lds_bytes, 1));
        q.grid = std::min<int64_t>(total, (int64_t)std::max(1, lim.num_cus) * std::max(1, resident));
    }
    q.tile_rows = bth;
    q.tile_cols = btw;
    q.planes_per_group = bcvb * vec;
    q.redundancy = (double)k.tiles_h * k.tiles_w * r0[0] * r0[1] / ((double)k.H * k.W);
    q.n_levels = 2;
    return BS_OK;
}

// One pooling operation whose window is the whole plane (global pooling), the plane small
// enough for one lane to walk it.
static bool plane_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    if (count_pools(s, first_op, n_ops) != 1) return false;
    int32_t pre = 0, post = 0;
    bool seen = false;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            if (op.kh != op.in_h || op.kw != op.in_w || op.ph != 0 || op.pw != 0) return false;
            if (op.out_h != 1 || op.out_w != 1 || (int64_t)op.in_h * op.in_w > 1024) return false;
            seen = true;
        } else if (op.kind != OP_AVGNORM) {
            (seen ? post : pre)++;
        }
    }
    return pre <= K_MAX_EW && post <= K_MAX_EW;
}

static void plan_direct(const bs_stack *s, Sequence &q, bool whole_plane = false)
{
    q.variant = whole_plane ? BS_VARIANT_PLANE_POOL : BS_VARIANT_POOL_DIRECT;
    PoolDirectK &k = q.direct;
    k = PoolDirectK{};
    int32_t vec = vec_of(s);
    bool seen = false;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            k.pool = make_pool(op, nullptr, q);
            k.H = op.in_h; k.W = op.in_w; k.Ho = op.out_h; k.Wo = op.out_w;
            if (!whole_plane) vec = direct_vec(s, op);  // non-zero: direct_applicable said so
            seen = true;
        } else if (op.kind != OP_AVGNORM) {
            if (seen) fill_ew(s, op, q, k.post[k.n_post++]);
            else fill_ew(s, op, q, k.pre[k.n_pre++]);
        }
    }
    q.vec = vec;
    k.C = (int32_t)q.in_shape[1];
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    if (whole_plane) {
        q.vec = 1;
        k.total = (uint32_t)planes;
        k.div_c = make_fastdiv((uint32_t)k.C);
        q.threads = std::min(q.threads, 256);
        q.redundancy = 1.0;
        q.tile_rows = q.tile_cols = 1;
        q.n_levels = 1;
        const int64_t hw = (int64_t)k.H * k.W;
        if (hw > K_PLANE_WALK_CELLS) {
            // staged through LDS: so many planes per work-group that a lane fetches at most eight
            // cells (one memory round trip), at most one plane per lane of a wave
            q.threads = 256;
            k.ppg = (int32_t)std::max<int64_t>(1, std::min<int64_t>(64, (int64_t)q.threads * 8 / hw));
            k.pitch = (int32_t)(hw | 1);
            k.div_wv = make_fastdiv((uint32_t)hw);
            q.grid = (planes + k.ppg - 1) / k.ppg;
            q.lds_bytes = (uint64_t)k.ppg * k.pitch * 4;
            q.planes_per_group = k.ppg;
            return;
        }
        q.grid = (planes + q.threads - 1) / q.threads;
        q.lds_bytes = 0;
        q.planes_per_group = q.threads;
        return;
    }
    const int32_t wv = k.W / vec;
    k.total = (uint32_t)(planes * k.Ho * wv);
    k.div_wv = make_fastdiv((uint32_t)wv);
    k.div_ho = make_fastdiv((uint32_t)k.Ho);
    k.div_c = make_fastdiv((uint32_t)k.C);
    const int64_t per_group = (int64_t)q.threads * K_DIRECT_U;
    q.grid = ((int64_t)k.total + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.redundancy = (double)(k.Ho * k.pool.kh) / (double)k.H;
    q.tile_rows = q.tile_cols = 0;
    q.planes_per_group = 0;
    q.n_levels = 1;
}

constexpr int32_t K_AUTO_STEPS = 5;                  // steps per sequence of an unrestricted automatic plan
constexpr uint64_t K_DEFAULT_LDS_BYTES = 64 * 1024;  // on-chip budget per work-group when the caller gives none

// May this plan rely on run-time kernel builds for signatures without a pre-compiled instance?
static bool jit_allowed(const bs_stack *s)
{
    return s->opts.jit >= 0 && !s->jit_failed && jit_enabled();
}

// A lane of the register sliding-window kernels computes (and, beyond its own 128-bit block,
// loads with scalar loads) every input column its windows touch: nc0 columns for vec owned.
// Measured on MI355X, once that ratio passes 1.75 (5x5 windows, or a 3x3 stride-1 pool behind
// another pool) the LDS kernels, which share those columns between lanes, are faster --
// provided the sequence gets a specialised LDS build rather than the run-time-shape kernel.
static bool rows_columns_pay(const bs_stack *s, int32_t nc0, int32_t vec)
{
    return nc0 * 4 <= vec * 7 || !jit_allowed(s) || s->opts.force_variant == BS_VARIANT_POOL_ROWS;
}

// May the sliding-window kernels whose lanes exchange edge columns serve a plane of width W?  All
// column blocks of a row must sit in one wave.
static bool exchange_fits(const bs_stack *s, int32_t W, int32_t vec)
{
    return s->opts.lane_exchange >= 0 && W % vec == 0 && W / vec <= 64;
}

// Two consecutive pooling operations, BatchNorm and ReLU only around them, no index output on
// the first, in shapes one of the two-level rows kernels is instantiated for (or can be built
// for).  Preferred: the kernel whose lanes exchange edge columns (k.spw > 0 says so).
static bool rows2_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops, Sequence *fill)
{
    Sequence tmp;
    Sequence &q = fill ? *fill : tmp;
    PoolRows2K k{};
    int seen = 0;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            if (seen == 0) {
                if (op.idx_slot >= 0) return false;
                k.pool1 = make_pool(op, nullptr, q);
                k.H = op.in_h; k.W = op.in_w; k.H1 = op.out_h; k.W1 = op.out_w;
            } else {
                k.pool2 = make_pool(op, nullptr, q);
                k.Ho = op.out_h; k.Wo = op.out_w;
            }
            ++seen;
        } else if (op.kind != OP_AVGNORM) {
            if (op.kind == OP_ADD) return false;
            int32_t &n = seen == 0 ? k.n_pre : (seen == 1 ? k.n_mid : k.n_post);
            EwOp *list = seen == 0 ? k.pre : (seen == 1 ? k.mid : k.post);
            if (n >= K_MAX_EW) return false;
            fill_ew(s, op, q, list[n++]);
        }
    }
    if (seen != 2) return false;
    const int32_t sws = k.pool1.sw * k.pool2.sw;
    const bool in_table = dtype_has_tables(s->dtype) && rows2_supported(k);
    // lanes exchange edge columns: every column of the plane between the pools and every output
    // column must belong to some lane
    {
        const int32_t vec = xrows2_vec(s->dtype);
        if (exchange_fits(s, k.W, vec) && sws >= 1 && vec % sws == 0 && (in_table || (jit_allowed(s) && xrows2_buildable(k, vec))) &&
            (int64_t)(k.W / vec) * (vec / k.pool1.sw) >= k.W1 && (int64_t)(k.W / vec) * (vec / sws) >= k.Wo) {
            k.cbs = k.W / vec;
            k.spw = 64 / k.cbs;
            if (fill) fill->rows2 = k;
            return true;
        }
    }
    const int32_t vec = rows2_vec(s->dtype);
    if (k.W % vec != 0) return false;
    if (!in_table && !(jit_allowed(s) && rows2_buildable(k, vec))) return false;
    // every output column must fall under some lane's column block
    if (vec % sws != 0 || (int64_t)(k.W / vec) * (vec / sws) < k.Wo) return false;
    {
        const int32_t nc1 = (vec / sws - 1) * k.pool2.sw + k.pool2.kw;
        if (!rows_columns_pay(s, (nc1 - 1) * k.pool1.sw + k.pool1.kw, vec)) return false;
    }
    if (fill) fill->rows2 = k;
    return true;
}

// One pooling operation with overlapping / padded windows, BatchNorm and ReLU only around it,
// in a shape one of the rows kernels is instantiated for -- or two such operations
// (rows2_applicable).  Preferred: the kernel whose lanes exchange edge columns (k.spw > 0).
static bool rows_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops, Sequence *fill)
{
    if (count_pools(s, first_op, n_ops) == 2) return rows2_applicable(s, first_op, n_ops, fill);
    if (count_pools(s, first_op, n_ops) != 1) return false;
    Sequence tmp;
    Sequence &q = fill ? *fill : tmp;
    PoolRowsK k{};
    bool seen = false;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            k.pool = make_pool(op, nullptr, q);
            k.H = op.in_h; k.W = op.in_w; k.Ho = op.out_h; k.Wo = op.out_w;
            seen = true;
        } else if (op.kind != OP_AVGNORM) {
            if (op.kind == OP_ADD) return false;
            if ((seen ? k.n_post : k.n_pre) >= K_MAX_EW) return false;
            if (seen) fill_ew(s, op, q, k.post[k.n_post++]);
            else fill_ew(s, op, q, k.pre[k.n_pre++]);
        }
    }
    if (!seen) return false;
    if (k.pool.sw < 1 || k.pool.kw - k.pool.sw - k.pool.pw < 0) return false;
    const bool in_table = dtype_has_tables(s->dtype) && rows_supported(k.pool, k.pre, k.n_pre, k.post, k.n_post);
    {
        const int32_t vec = xrows_vec(s->dtype);
        if (exchange_fits(s, k.W, vec) && vec % k.pool.sw == 0 &&
            (in_table || (jit_allowed(s) && xrows_buildable(k.pool, k.pre, k.n_pre, k.post, k.n_post, vec))) &&
            (int64_t)(k.W / vec) * (vec / k.pool.sw) >= k.Wo) {
            k.cbs = k.W / vec;
            k.spw = 64 / k.cbs;
            if (fill) fill->rows = k;
            return true;
        }
    }
    const int32_t vec = rows_vec(s->dtype);
    if (k.W % vec != 0 || vec % k.pool.sw != 0) return false;
    if (!in_table && !(jit_allowed(s) && rows_buildable(k.pool, k.pre, k.n_pre, k.post, k.n_post, vec))) return false;
    // every output column must fall under some lane's column block
    if ((int64_t)(k.W / vec) * (vec / k.pool.sw) < k.Wo) return false;
    if (!rows_columns_pay(s, vec + k.pool.kw - k.pool.sw, vec)) return false;
    if (fill) fill->rows = k;
    return true;
}

// Argument block and launch shape of a lane-exchange kernel: spw segments of cbs lanes per wave,
// whole waves, chunks of rc output rows evened out over the plane.
template <class K>
static void plan_exchange(Sequence &q, K &k, int64_t planes, int32_t rc, int32_t multiple)
{
    rc = std::max(1, std::min(rc, k.Ho));
    k.chunks = (k.Ho + rc - 1) / rc;
    rc = (k.Ho + k.chunks - 1) / k.chunks;
    k.rc = (rc + multiple - 1) / multiple * multiple;
    k.chunks = (k.Ho + k.rc - 1) / k.rc;
    k.units = (uint32_t)(planes * k.chunks);
    k.total = (uint32_t)(planes * k.chunks * k.cbs);
    k.div_cbs = make_fastdiv((uint32_t)k.cbs);
    k.div_chunks = make_fastdiv((uint32_t)k.chunks);
    k.div_c = make_fastdiv((uint32_t)k.C);
    q.threads = std::max(64, std::min(q.threads, 256));  // whole waves; the kernels have no barrier, any number of waves works
    const int64_t per_group = (int64_t)k.spw * (q.threads / 64);
    q.grid = ((int64_t)k.units + per_group - 1) / per_group;
}

// Two and more identical max-pooling steps that keep the plane's size (odd window, stride 1, padding (k - 1) / 2,
// no index output), each followed by element-wise operations of the same kinds (no Add), nothing in front of the
// first: the blocks of Section 5.1.  The chain kernel exists for the shapes and lists compiled into the library, on
// planes whose rows fit one wave; anything else takes the LDS tiles.
static bool chain_applicable(const bs_stack *s, int32_t first_op, int32_t n_ops, Sequence *fill)
{
    if (s->opts.layout == BS_LAYOUT_NHWC || s->opts.force_variant == BS_VARIANT_LDS_TILE) return false;
    Sequence tmp;
    Sequence &q = fill ? *fill : tmp;
    RowsChainK k{};
    int32_t level = -1, n_here = 0;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            if (op.kind != OP_MAXPOOL || op.idx_slot >= 0 || op.sh != 1 || op.sw != 1 || op.kh != 2 * op.ph + 1 ||
                op.kw != 2 * op.pw + 1 || op.out_h != op.in_h || op.out_w != op.in_w)
                return false;
            if (level >= 0 && n_here != k.n_ew) return false;  // every level has the same list length
            if (++level >= K_CHAIN_MAX) return false;
            const PoolK p = make_pool(op, nullptr, q);
            if (level == 0) {
                k.pool = p;
                k.H = op.in_h;
                k.W = op.in_w;
            } else if (p.kh != k.pool.kh || p.kw != k.pool.kw || p.ph != k.pool.ph || p.pw != k.pool.pw) {
                return false;
            }
            n_here = 0;
        } else if (op.kind != OP_AVGNORM) {
            if (level < 0 || op.kind == OP_ADD || n_here >= K_MAX_EW) return false;
            fill_ew(s, op, q, k.ew[level][n_here]);
            if (level > 0 && k.ew[level][n_here].kind != k.ew[0][n_here].kind) return false;
            ++n_here;
            if (level == 0) k.n_ew = n_here;
        }
    }
    if (level < BS_CHAIN_MIN - 1 || n_here != k.n_ew) return false;
    k.n_levels = level + 1;
    const int32_t vec = xrows_vec(s->dtype);
    if (!exchange_fits(s, k.W, vec)) return false;
    if (!xrows_chain_supported(k, s->dtype) && !(jit_allowed(s) && xrows_chain_buildable(k, vec))) return false;
    k.cbs = k.W / vec;
    k.spw = 64 / k.cbs;
    if (fill) fill->chain = k;
    return true;
}

static void plan_chain(const bs_stack *s, Sequence &q, const bs_plan_options &o)
{
    q.variant = BS_VARIANT_ROWS_CHAIN;
    q.n_idx = 0;
    chain_applicable(s, q.first_op, q.n_ops, &q);
    RowsChainK &k = q.chain;
    q.vec = xrows_vec(s->dtype);
    k.C = (int32_t)q.in_shape[1];
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    // Output rows per lane.  A chunk also computes the n_levels * ph rows above and below it at the first level (one
    // fewer per level after that): longer chunks recompute less, shorter ones give more waves.  Half the plane
    // (measured on 56 x 56 planes, 5 levels, float32: 7 / 14 / 19 / 28 / 56 rows -> 8.1 / 6.5 / 6.4 / 6.3 / 6.7 us per
    // block), and at least as many rows as the chunk recomputes.
    const int32_t halo = 2 * k.n_levels * k.pool.ph;
    int32_t rc = std::max(halo, (k.H + 1) / 2);
    if (o.tile_rows > 0) rc = o.tile_rows;
    rc = std::max(1, std::min(rc, k.H));
    k.chunks = (k.H + rc - 1) / rc;
    k.rc = (k.H + k.chunks - 1) / k.chunks;
    k.chunks = (k.H + k.rc - 1) / k.rc;
    k.units = (uint32_t)(planes * k.chunks);
    k.div_cbs = make_fastdiv((uint32_t)k.cbs);
    k.div_chunks = make_fastdiv((uint32_t)k.chunks);
    k.div_c = make_fastdiv((uint32_t)k.C);
    q.threads = 256;
    const int64_t per_group = (int64_t)k.spw * (q.threads / 64);
    q.grid = ((int64_t)k.units + per_group - 1) / per_group;
    q.lds_bytes = 0;
    q.tile_rows = k.rc;
    q.tile_cols = k.W;
    q.planes_per_group = 0;
    q.n_levels = k.n_levels;
    q.halo_rows = halo;
    q.halo_cols = 0;
    double rows_loaded = 0;
    for (int32_t ch = 0; ch < k.chunks; ++ch) {
        const int32_t a = ch * k.rc, b = std::min(k.H, a + k.rc);
        rows_loaded += std::min(k.H, b + halo / 2) - std::max(0, a - halo / 2);
    }
    q.redundancy = rows_loaded / (double)k.H;
}

static void plan_rows2(const bs_stack *s, Sequence &q, const bs_plan_options &o)
{
    PoolRows2K &k = q.rows2;
    const int32_t vec = k.spw > 0 ? xrows2_vec(s->dtype) : rows2_vec(s->dtype);
    q.vec = vec;
    q.threads = std::min(q.threads, 256);
    k.C = (int32_t)q.in_shape[1];
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    k.cbs = k.W / vec;
    if (k.spw > 0) {
        // Output rows per lane: a chunk recomputes the level-1 rows and re-reads the input rows
        // it shares with the chunk above.
        plan_exchange(q, k, planes, o.tile_rows > 0 ? o.tile_rows : (s->dtype == BS_F32 ? K_XROWS2_RC32 : K_XROWS2_RC16), 1);
    } else {
        // Output rows per lane: a chunk recomputes the level-1 rows and re-reads the input rows it
        // shares with the chunk above, so chunks are longer than in the one-level kernel.
        int32_t rc = std::min(K_ROWS2_RC, k.Ho);
        if (o.tile_rows > 0) rc = std::min(o.tile_rows, k.Ho);
        k.rc = std::max(1, rc);
        k.chunks = (k.Ho + k.rc - 1) / k.rc;
        k.total = (uint32_t)(planes * k.chunks * k.cbs);
        k.div_cbs = make_fastdiv((uint32_t)k.cbs);
        k.div_chunks = make_fastdiv((uint32_t)k.chunks);
        k.div_c = make_fastdiv((uint32_t)k.C);
        q.grid = ((int64_t)k.total + q.threads - 1) / q.threads;
    }
    q.lds_bytes = 0;
    q.tile_rows = k.rc;
    q.tile_cols = k.Wo;
    q.planes_per_group = 0;
    q.n_levels = 2;
    const int32_t r0 = (k.pool2.kh - 1) * k.pool1.sh + k.pool1.kh;  // input rows under one output row
    q.halo_rows = std::max(0, r0 - k.pool1.sh * k.pool2.sh);
    q.halo_cols = k.pool2.pw * k.pool1.sw + k.pool1.pw;
    double rows_loaded = 0;
    for (int32_t ch = 0; ch < k.chunks; ++ch) {
        const int32_t a = ch * k.rc, b = std::min(k.Ho, a + k.rc);
        const int32_t lo1 = a * k.pool2.sh - k.pool2.ph, hi1 = (b - 1) * k.pool2.sh - k.pool2.ph + k.pool2.kh;
        const int32_t lo = std::max(0, lo1 * k.pool1.sh - k.pool1.ph);
        const int32_t hi = std::min(k.H, (hi1 - 1) * k.pool1.sh - k.pool1.ph + k.pool1.kh);
        rows_loaded += std::max(0, hi - lo);
    }
    q.redundancy = rows_loaded / (double)k.H;
}

static void plan_rows(const bs_stack *s, Sequence &q, const bs_plan_options &o, const Limits &lim)
{
    q.variant = BS_VARIANT_POOL_ROWS;
    q.n_idx = 0;
    rows_applicable(s, q.first_op, q.n_ops, &q);
    if (count_pools(s, q.first_op, q.n_ops) == 2) {
        plan_rows2(s, q, o);
        return;
    }
    PoolRowsK &k = q.rows;
    const int32_t vec = k.spw > 0 ? xrows_vec(s->dtype) : rows_vec(s->dtype);
    q.vec = vec;
    q.threads = std::min(q.threads, 256);
    k.C = (int32_t)q.in_shape[1];
    const int64_t planes = q.in_shape[0] * q.in_shape[1];
    k.cbs = k.W / vec;
    // Output rows per lane.  Measured on MI355X, short chunks win: the kh - sh rows two vertically
    // adjacent chunks share are requested by lanes of the same wave within a few instructions and
    // are served by the L1/L2 caches, while long chunks leave each lane a chain of dependent
    // memory round trips.  With two rows per lane (and the kernel producing two output rows per
    // iteration) a lane requests all its input rows at once: one round trip per wave.
    int32_t rc = std::min(K_ROWS_OR, k.Ho);
    (void)lim;
    if (o.tile_rows > 0) rc = std::min(o.tile_rows, k.Ho);
    if (k.spw > 0) {
        plan_exchange(q, k, planes, rc, K_ROWS_OR);  // the kernel produces K_ROWS_OR output rows per iteration
    } else {
        k.rc = std::max(1, rc);
        k.chunks = (k.Ho + k.rc - 1) / k.rc;
        k.total = (uint32_t)(planes * k.chunks * k.cbs);
        k.div_cbs = make_fastdiv((uint32_t)k.cbs);
        k.div_chunks = make_fastdiv((uint32_t)k.chunks);
        k.div_c = make_fastdiv((uint32_t)k.C);
        q.grid = ((int64_t)k.total + q.threads - 1) / q.threads;
    }
    q.lds_bytes = 0;
    q.tile_rows = k.rc;
    q.tile_cols = k.Wo;
    q.planes_per_group = 0;
    q.n_levels = 1;
    q.halo_rows = std::max(0, k.pool.kh - k.pool.sh);
    q.halo_cols = 0;
    // rows loaded per plane / rows of the plane
    double rows_loaded = 0;
    for (int32_t ch = 0; ch < k.chunks; ++ch) {
        const int32_t a = ch * k.rc, b = std::min(k.Ho, a + k.rc);
        const int32_t lo = std::max(0, a * k.pool.sh - k.pool.ph);
        const int32_t hi = std::min(k.H, (b - 1) * k.pool.sh - k.pool.ph + k.pool.kh);
        rows_loaded += std::max(0, hi - lo);
    }
    q.redundancy = rows_loaded / (double)k.H;
}

// Does a pre-compiled fast kernel exist for this op range?  Streaming, disjoint-window and
// rows sequences always have one; an LDS sequence only if its signature is instantiated.
static bool seq_is_fast(const bs_stack *s, int32_t first_op, int32_t n_ops)
{
    if (count_pools(s, first_op, n_ops) == 0) return true;
    if (direct_applicable(s, first_op, n_ops) || rows_applicable(s, first_op, n_ops, nullptr) ||
        plane_applicable(s, first_op, n_ops) || chain_applicable(s, first_op, n_ops, nullptr))
        return true;
    if (!seq_capacity_ok(s, first_op, n_ops, false)) return false;
    if (jit_allowed(s)) return true;  // any signature gets its own build
    if (!dtype_has_tables(s->dtype)) return false;
    Sequence tmp;
    LdsSeqK k{};
    int level = 0;
    for (int32_t i = first_op; i < first_op + n_ops; ++i) {
        const Op &op = s->ops[i];
        if (!op_is_elementwise(op.kind)) {
            k.pool[++level] = make_pool(op, nullptr, tmp);
            tmp.n_idx = 0;
        } else if (op.kind != OP_AVGNORM) {
            LevelK &lv = k.level[level];
            fill_ew(s, op, tmp, lv.ew[lv.n_ew++]);
        }
    }
    k.n_levels = level;
    return lds_fast_path(k);
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
    int32_t sprod_w0 = 1;
    for (int32_t i = q.first_op; i < q.first_op + q.n_ops; ++i)
        if (!op_is_elementwise(s->ops[i].kind)) sprod_w0 *= s->ops[i].sw;
    // the level-0 LDS rows of all tiles must start at the same offset inside a 128-bit vector
    auto vec_for = [&](int32_t tw) {
        const int64_t ntw = (WL + tw - 1) / tw;
        return (ntw == 1 || ((int64_t)tw * sprod_w0) % vec0 == 0) ? vec0 : 1;
    };
    auto consider = [&](int32_t th, int32_t tw, int32_t ppg) {
        if (th < 1 || tw < 1 || ppg < 1 || th > HL || tw > WL || ppg > planes) return;
        lds_geometry(s, q.first_op, q.n_ops, th, tw, ppg, vec_for(tw), g);
        if (g.lds_bytes > budget) return;
        const int64_t nth = (HL + th - 1) / th, ntw = (WL + tw - 1) / tw;
        const int64_t grid = nth * ntw * ((planes + ppg - 1) / ppg);
        // cost model: redundant loads, ragged last tile, lanes idle in the widest pooling
        // phase, too few work-groups to fill the chip, and a mild preference for smaller
        // LDS (occupancy).
        double score = g.redundancy;
        score *= (double)(nth * th) / HL * (double)(ntw * tw) / WL;
        double worst_fill = 1.0;
        for (int l = 1; l <= g.L; ++l) {
            const int32_t vo = strip_outputs(g.dw[l].s);
            const double strips = (double)g.rows[l] * (g.cols[l] / vo);
            const double passes = std::ceil(strips / q.threads);
            worst_fill = std::min(worst_fill, strips / (passes * q.threads));
        }
        score *= 1.0 + 0.35 * (1.0 - worst_fill);
        const double want = 8.0 * std::max(1, lim.num_cus);
        if ((double)grid < want) score *= 1.0 + 0.25 * (want - grid) / want;
        score *= 1.0 + 0.25 * (double)g.lds_bytes / (double)std::max<uint64_t>(budget, 1);
        if (tw != WL) score *= 1.05;
        if (vec_for(tw) != vec0) score *= 1.5;
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
        tws.push_back(WL);
        for (int32_t t = 4; t < WL; t += 4) tws.push_back(t);
        for (int32_t t : {1, 2}) if (t < WL) tws.push_back(t);
        for (int32_t t = 1; t <= HL; ++t) ths.push_back(t);
        for (int32_t tw : tws)
            for (int32_t th : ths) {
                consider(th, tw, 1);
                if (th == HL && tw == WL)
                    for (int32_t ppg : {2, 3, 4, 6, 8, 12, 16}) consider(th, tw, ppg);
            }
    }
    if (best_th == 0) return BS_ERR_NO_FIT;

    const int32_t vec_eff = vec_for(best_tw);
    lds_geometry(s, q.first_op, q.n_ops, best_th, best_tw, best_ppg, vec_eff, g);
    q.tile_rows = best_th;
    q.tile_cols = best_tw;
    q.planes_per_group = best_ppg;
    q.vec = vec_eff;
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
    k.vec = vec_eff;
    k.delta0 = g.delta0;
    k.div_tiles_w = make_fastdiv((uint32_t)k.tiles_w);
    k.div_tiles_hw = make_fastdiv((uint32_t)(k.tiles_w * k.tiles_h));
    k.div_c = make_fastdiv((uint32_t)k.C);
    q.grid = (int64_t)k.tiles_h * k.tiles_w * ((planes + best_ppg - 1) / best_ppg);
    int level = 0;
    for (int l = 0; l <= g.L; ++l) {
        LevelK &lv = k.level[l];
        lv.H = g.H[l]; lv.W = g.W[l];
        lv.rows = g.rows[l];
        lv.cols = g.cols[l];
        lv.pitch = g.pitch[l];
        lv.plane_stride = lv.rows * lv.pitch;
        lv.buf_off = (l & 1) ? (int32_t)g.buf_floats[0] : 0;
        lv.n_ew = 0;
        lv.vo = (l == 0) ? 1 : strip_outputs(g.dw[l].s);
        lv.items_per_row = (l == 0) ? g.nvr : lv.cols / lv.vo;
        lv.ct = std::min(lv.items_per_row, q.threads);
        lv.rt = q.threads / lv.ct;
        lv.div_ct = make_fastdiv((uint32_t)lv.ct);
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

// Bounds audit of an LDS sequence, run on the host at plan time: the rectangle of every
// level holds all windows of the level above, every level's buffer lies inside the LDS
// allocation with 16-byte aligned rows, item counts match the extents, and an index output
// in the middle of a sequence is covered by the tiles without gaps.  A plan that fails it is
// never launched.
static bool audit_lds(const Sequence &q)
{
    const LdsSeqK &k = q.lds;
    const int32_t L = k.n_levels;
    const uint64_t lds_floats = q.lds_bytes / sizeof(float);
    if (L < 1 || L > K_MAX_LEVELS || k.PPG < 1 || k.TH < 1 || k.TW < 1) return false;
    if (k.vec != 1 && k.vec != 4 && k.vec != 8) return false;
    if (k.level[L].rows != k.TH || k.level[L].cols < k.TW || k.level[L].cols % 4) return false;
    if (k.vec > 1 && k.level[0].W % k.vec) return false;
    int64_t lo_r = 0, lo_c = 0;  // most negative origin (tile 0)
    for (int l = L; l >= 1; --l) {
        const LevelK &lv = k.level[l], &pv = k.level[l - 1];
        const PoolK &p = k.pool[l];
        if (p.kh < 1 || p.kw < 1 || p.sh < 1 || p.sw < 1) return false;
        if (lv.vo != strip_outputs(p.sw)) return false;
        if (lv.cols % 4 || lv.items_per_row != lv.cols / lv.vo) return false;
        if (pv.rows < (lv.rows - 1) * p.sh + p.kh) return false;
        if (pv.cols < (lv.cols - 1) * p.sw + p.kw) return false;
        lo_r = lo_r * p.sh - p.ph;
        lo_c = lo_c * p.sw - p.pw;
        if (p.idx_slot >= 0 && l < L) {
            // tiles must cover the whole level: checked by the planner's covers_input() rule;
            // here: the rectangle is at least as large as the distance between tile origins
            int64_t step_r = k.TH, step_c = k.TW;
            for (int m = L; m > l; --m) { step_r *= k.pool[m].sh; step_c *= k.pool[m].sw; }
            if (lv.rows < step_r || lv.cols < step_c) return false;
        }
    }
    if (lo_c < -(int64_t)4096 * std::max(k.vec, 1) || lo_r < -(1 << 20)) return false;
    for (int l = 0; l < L; ++l) {
        const LevelK &lv = k.level[l];
        if (lv.pitch < lv.cols || lv.pitch % 4 || lv.buf_off % 4) return false;
        if (lv.plane_stride != lv.rows * lv.pitch) return false;
        if ((uint64_t)lv.buf_off + (uint64_t)k.PPG * lv.plane_stride > lds_floats) return false;
        if (l + 1 < L && (l & 1) == ((l + 1) & 1)) return false;
    }
    const LevelK &l0 = k.level[0];
    if (k.vec > 1) {
        // all tiles share delta0; the vectors of a row cover the rectangle; aligned over-reads of
        // up to 3 floats stay inside the row pitch
        if (k.delta0 != (int32_t)(((lo_c % k.vec) + k.vec) % k.vec)) return false;
        if (k.tiles_w > 1) {
            int64_t step_c = k.TW;
            for (int m = L; m >= 1; --m) step_c *= k.pool[m].sw;
            if (step_c % k.vec) return false;
        }
        if (l0.items_per_row * k.vec < k.delta0 + l0.cols) return false;
        if (l0.pitch < l0.items_per_row * k.vec + 4) return false;
    } else {
        if (k.delta0 != 0 || l0.items_per_row != l0.cols) return false;
    }
    for (int l = 0; l <= L; ++l) {
        const LevelK &lv = k.level[l];
        if (lv.ct < 1 || lv.rt < 1 || lv.ct * lv.rt > q.threads || lv.ct > lv.items_per_row) return false;
        if (lv.div_ct.d != (uint32_t)lv.ct) return false;
    }
    return true;
}

// ---------------------------------------------------------------------------
// Steps -> sequences (Section 4.1): steps are appended to the current sequence
// while its resource consumption stays within the device limit; otherwise the
// sequence is closed and a new one starts with that step.  The trailing sequence
// is kept.  A step-count cap implements the strategies of Section 5.1.
// ---------------------------------------------------------------------------
// Header and template-instance names (without / with index outputs) of a sequence's run-time build.
static const char *jit_names(const bs_stack *s, const Sequence &q, std::string (&expr)[2])
{
    if (q.variant == BS_VARIANT_ROWS_CHAIN) {
        expr[0] = expr[1] = xrows_chain_expr(q.chain, s->dtype);
        return "bs_xrows_device.h";
    }
    for (int w = 0; w < 2; ++w) {
        if (q.variant == BS_VARIANT_POOL_ROWS && q.n_levels == 2)
            expr[w] = q.rows2.spw > 0 ? xrows2_expr(q.rows2, s->dtype, w != 0) : rows2_expr(q.rows2, s->dtype, w != 0);
        else if (q.variant == BS_VARIANT_POOL_ROWS)
            expr[w] = q.rows.spw > 0 ? xrows_expr(q.rows, s->dtype, w != 0) : rows_expr(q.rows, s->dtype, w != 0);
        else expr[w] = lds_expr(q.lds, s->dtype, w != 0);
    }
    if (q.variant != BS_VARIANT_POOL_ROWS) return "bs_lds_device.h";
    return (q.n_levels == 2 ? q.rows2.spw : q.rows.spw) > 0 ? "bs_xrows_device.h" : "bs_rows_device.h";
}

// Decide whether the sequence runs a pre-compiled kernel or a run-time build, and (unless
// the plan is host-only) compile the latter now: without index outputs, and with them if
// the sequence has any.  A failed build marks the stack so that it is planned again without.
static bs_status prepare_jit(bs_stack *s, Sequence &q, bool host_only)
{
    q.jit = 0;
    q.jit_fn[0] = q.jit_fn[1] = nullptr;
    const bool tables = dtype_has_tables(s->dtype);
    // the sliding-window kernels (compiled in or built here) are instantiated for one column-block
    // width per storage type; a plan made for another width must never reach them
    if (q.variant == BS_VARIANT_POOL_ROWS) {
        const bool two = q.n_levels == 2, exchange = (two ? q.rows2.spw : q.rows.spw) > 0;
        const int32_t vec = exchange ? (two ? xrows2_vec(s->dtype) : xrows_vec(s->dtype))
                                     : (two ? rows2_vec(s->dtype) : rows_vec(s->dtype));
        if (q.vec != vec) return BS_ERR_UNSUPPORTED;
    }
    if (q.variant == BS_VARIANT_POOL_ROWS && q.n_levels == 2) {
        if (tables && rows2_supported(q.rows2)) return BS_OK;
    } else if (q.variant == BS_VARIANT_POOL_ROWS) {
        const PoolRowsK &k = q.rows;
        if (tables && rows_supported(k.pool, k.pre, k.n_pre, k.post, k.n_post)) return BS_OK;
    } else if (q.variant == BS_VARIANT_ROWS_CHAIN) {
        if (q.vec != xrows_vec(s->dtype)) return BS_ERR_UNSUPPORTED;
        if (xrows_chain_supported(q.chain, s->dtype)) return BS_OK;
    } else if (q.variant == BS_VARIANT_LDS_TILE) {
        if (lds_precompiled(q.lds, s->dtype) || !jit_allowed(s) || !lds_buildable(q.lds)) return BS_OK;
    } else {
        return BS_OK;
    }
    std::string expr[2];
    const char *header = jit_names(s, q, expr);
    const bool idx_variant = q.n_idx > 0;
    q.jit = 1;
    if (host_only) return BS_OK;
    for (int w = 0; w < (idx_variant ? 2 : 1); ++w) {
        const bs_status st = jit_kernel(header, expr[w], &q.jit_fn[w]);
        if (st != BS_OK) {
            s->jit_failed = true;
            return BS_ERR_JIT;
        }
    }
    return BS_OK;
}

bs_status group_sequences(bs_stack *s, const bs_plan_options &o, const Limits &lim)
{
    s->seqs.clear();
    const int32_t threads = o.threads_per_group > 0 ? o.threads_per_group : 256;
    const bool per_layer = o.breadth_first != 0;
    auto range_ops = [&](const SeqDraft &d, int32_t &first_op, int32_t &n_ops) {
        first_op = s->steps[d.first_step].first_op;
        const Step &lst = s->steps[d.first_step + d.n_steps - 1];
        n_ops = lst.first_op + lst.n_ops - first_op;
    };
    // greedy fill (Section 4.1): append steps while the sequence fits; `cap` = most steps per sequence
    auto fill = [&](int32_t cap, std::vector<SeqDraft> &drafts) -> bs_status {
        drafts.clear();
        SeqDraft cur{0, 0};
        for (int32_t i = 0; i < (int32_t)s->steps.size(); ++i) {
            if (cur.n_steps == 0) {
                cur = SeqDraft{i, 1};
            } else {
                SeqDraft trial{cur.first_step, cur.n_steps + 1};
                int32_t fo, no;
                range_ops(trial, fo, no);
                bool fits = !per_layer;
                if (fits && cap > 0 && trial.n_steps > cap) fits = false;
                if (fits && !seq_capacity_ok(s, fo, no, true)) fits = false;
                if (fits && seq_min_lds(s, fo, no, threads) > lim.max_lds_bytes) fits = false;
                // cost rule: do not trade a sequence that has a pre-compiled fast kernel for a
                // longer one that would run the much slower run-time-shape build
                if (fits && o.force_variant == BS_VARIANT_AUTO) {
                    int32_t co, cn;
                    range_ops(cur, co, cn);
                    if (seq_is_fast(s, co, cn) && !seq_is_fast(s, fo, no)) fits = false;
                }
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
        return BS_OK;
    };
    std::vector<SeqDraft> drafts;
    const bool nhwc = o.layout == BS_LAYOUT_NHWC;
    if (nhwc) {
        // channels-last kernels take one step (one pooling operation) per sequence, or two that
        // the tile kernel exists for: neighbouring steps are paired from the front
        const bs_status fs = fill(1, drafts);
        if (fs != BS_OK) return fs;
        if (!per_layer && o.max_steps_per_sequence != 1) {
            std::vector<SeqDraft> paired;
            for (size_t i = 0; i < drafts.size(); ++i) {
                if (i + 1 < drafts.size()) {
                    Sequence trial;
                    trial.in_shape[0] = s->in_shape[0];
                    trial.in_shape[1] = s->in_shape[1];
                    const SeqDraft both{drafts[i].first_step, 2};
                    range_ops(both, trial.first_op, trial.n_ops);
                    if (plan_nhwc_tile2(s, trial, o, lim) == BS_OK) {
                        paired.push_back(both);
                        ++i;
                        continue;
                    }
                }
                paired.push_back(drafts[i]);
            }
            drafts.swap(paired);
        }
    } else if (o.max_steps_per_sequence > 0 || per_layer || o.force_variant != BS_VARIANT_AUTO) {
        const bs_status fs = fill(o.max_steps_per_sequence, drafts);
        if (fs != BS_OK) return fs;
    } else {
        // Unrestricted, automatic: every further stacked step adds halo that all earlier levels
        // recompute (Section 5.1), and the multi-step kernels are bound by arithmetic, not by
        // memory, once a few steps are fused -- measured on MI355X, four to five steps per
        // sequence are fastest.  Cap sequences at K_AUTO_STEPS steps, then even out their
        // lengths (8 steps run as 4 + 4 rather than 5 + 3).
        // Chains of identical blocks that the register kernel takes are the exception: it has no LDS
        // traffic and measured fastest with as many levels as it is compiled for (64 x 64 x 56 x 56,
        // float32: 9.0 / 7.1 / 6.3 / 6.0 / 5.6 us per block with 3 / 4 / 5 / 6 / 8 levels).
        int32_t cap = K_AUTO_STEPS;
        {
            std::vector<SeqDraft> longer;
            bool all_chains = fill(K_CHAIN_MAX, longer) == BS_OK && !longer.empty();
            for (const SeqDraft &d : longer) {
                int32_t fo, no;
                range_ops(d, fo, no);
                all_chains = all_chains && (d.n_steps < BS_CHAIN_MIN || chain_applicable(s, fo, no, nullptr));
                all_chains = all_chains && (d.n_steps >= BS_CHAIN_MIN || longer.size() > 1);
            }
            if (all_chains) cap = K_CHAIN_MAX;
        }
        bs_status fs = fill(cap, drafts);
        if (fs != BS_OK) return fs;
        const int32_t n_seq = (int32_t)drafts.size(), n_steps = (int32_t)s->steps.size();
        const int32_t even = n_seq > 0 ? (n_steps + n_seq - 1) / n_seq : 0;
        if (n_seq > 1 && even < cap) {
            std::vector<SeqDraft> balanced;
            fs = fill(even, balanced);
            if (fs == BS_OK && balanced.size() == drafts.size()) drafts.swap(balanced);
        }
    }

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
        if (nhwc) {
            st = q.n_steps == 2 ? plan_nhwc_tile2(s, q, o, lim) : plan_nhwc(s, q);
        } else if (pools == 0) {
            plan_stream(s, q);
        } else if (direct_applicable(s, q.first_op, q.n_ops) && o.force_variant != BS_VARIANT_LDS_TILE) {
            plan_direct(s, q);
        } else if (BS_CHAIN_MIN < 3 && o.force_variant == BS_VARIANT_AUTO && chain_applicable(s, q.first_op, q.n_ops, nullptr)) {
            plan_chain(s, q, o);
        } else if (rows_applicable(s, q.first_op, q.n_ops, nullptr) && o.force_variant != BS_VARIANT_LDS_TILE) {
            plan_rows(s, q, o, lim);
        } else if (plane_applicable(s, q.first_op, q.n_ops) && o.force_variant != BS_VARIANT_LDS_TILE) {
            plan_direct(s, q, true);
        } else if (chain_applicable(s, q.first_op, q.n_ops, nullptr)) {
            plan_chain(s, q, o);
        } else {
            st = plan_lds(s, q, o, lim);
        }
        if (st != BS_OK) return st;
        if (!nhwc) st = prepare_jit(s, q, o.host_only != 0);
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
    if (o.force_variant < 0 || o.force_variant > BS_VARIANT_PLANE_POOL) return BS_ERR_PARAM;  // the forceable families
    if (o.max_lds_bytes > 64 * 1024) return BS_ERR_PARAM;
    if (o.jit < -1 || o.jit > 1) return BS_ERR_PARAM;
    if (o.layout != BS_LAYOUT_NCHW && o.layout != BS_LAYOUT_NHWC) return BS_ERR_PARAM;
    if (o.lane_exchange < -1 || o.lane_exchange > 0) return BS_ERR_PARAM;
    // channels-last plans have their own two kernels: nothing to force, no tiles to set
    if (o.layout == BS_LAYOUT_NHWC && o.force_variant != BS_VARIANT_AUTO) return BS_ERR_PARAM;

    stack->planned = stack->device_planned = false;
    free_backward(stack);  // it refers to this plan's operations and parameter table
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
    // Default on-chip budget per work-group: all 64 KiB a group may address.  The paper caps
    // shared memory well below what its device offers to keep occupancy (Section 4.4); here a
    // compute unit has 160 KiB, two such groups still fit, and larger tiles (less halo to
    // recompute) measured faster than more resident groups.  The tile search still prefers
    // smaller footprints among equally good tiles.
    if (lim.max_lds_bytes == 0) lim.max_lds_bytes = K_DEFAULT_LDS_BYTES;

    stack->opts = o;
    stack->jit_failed = false;
    bs_status st;
    try {
        st = build_operations(stack);
        if (st == BS_OK) st = group_steps(stack);
        if (st == BS_OK) st = group_sequences(stack, o, lim);
        // a run-time build failed: unless the caller insists on them, plan with the
        // pre-compiled and run-time-shape kernels only
        if (st == BS_ERR_JIT && o.jit == 0) st = group_sequences(stack, o, lim);
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
        // set-up for bs_stack_run_static: find this device's copy of the library's scratch array now,
        // so that the run call itself touches nothing but the launch queue
        st = static_workspace_prepare(device);
        if (st != BS_OK) return st;
        stack->device = device;
        stack->device_planned = true;
    }
    return BS_OK;
}

bs_status bs_stack_jit_check(const bs_stack *stack, const char *arch, int32_t *n_built)
{
    if (!stack) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    int32_t n = 0;
    for (const Sequence &q : stack->seqs) {
        if (!q.jit) continue;
        std::string expr[2];
        const char *header = jit_names(stack, q, expr);
        for (int w = 0; w < (q.n_idx > 0 ? 2 : 1); ++w) {
            if (!jit_check(header, expr[w], arch ? arch : "gfx950")) return BS_ERR_JIT;
            ++n;
        }
    }
    if (n_built) *n_built = n;
    return BS_OK;
}

const char *bs_jit_log(void)
{
    static thread_local std::string copy;
    copy = jit_last_log();
    return copy.c_str();
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
    r.run_time_build = q.jit;
    r.reserved = 0;
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
    case OP_LEAKY: return "LeakyReLU";
    case OP_CLAMP: return "Clamp";
    }
    return nullptr;
}

uint64_t bs_stack_workspace_bytes(const bs_stack *stack)
{
    return (stack && stack->planned) ? stack->workspace_bytes : 0;
}

}  // extern "C"
