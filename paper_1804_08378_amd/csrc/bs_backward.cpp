// Backward pass of a stack (the paper's outlook, Section 7, names training as the next step;
// the forward pass of Sections 2 and 3 fixes what it computes): the product of the upstream
// gradient with the Jacobian of the layer-by-layer forward pass, with respect to the stack's
// input and its residual operands.
//
// A fused forward pass keeps no intermediate tensor, so the backward pass recomputes what it
// needs from the stack's input.  The stack is cut into stages, each a run of element-wise
// operations followed by at most one pooling operation:
//   * the input of every stage after the first, and the picks of every max pooling, are
//     recomputed by running the stages as forward stacks of their own (the forward kernels of
//     this library, index outputs switched on) into the workspace;
//   * then one kernel per stage, last stage first, turns the gradient with respect to the
//     stage's output into the gradient with respect to its input: it re-evaluates the stage's
//     element-wise operations on the stored input to get their derivatives and gathers, for
//     every input cell, the gradients of the pooling windows that hold it.
// A stack of one stage without max pooling (BatchNorm -> Add -> ReLU, BatchNorm -> ReLU ->
// AvgPool) needs no recomputation pass at all: input, upstream gradient in, gradients out.
// Host code only; the kernel is in bs_backward.hip.
#include <algorithm>
#include <cstring>
#include <new>

#if defined(BS_BWD_AUDIT)
#include <hip/hip_runtime.h>
#endif

#include "bs_internal.h"

using namespace bs;

namespace {

inline uint64_t numel(const int64_t *sh) { return (uint64_t)sh[0] * sh[1] * sh[2] * sh[3]; }
inline uint64_t align256(uint64_t v) { return (v + 255u) & ~(uint64_t)255u; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The stage's layers as a forward stack of their own, planned with the stack's options.
bs_status make_forward(const bs_stack *s, BwdStage &g, bool host_only)
{
    std::vector<bs_layer_desc> descs((size_t)g.n_layers);
    for (int32_t i = 0; i < g.n_layers; ++i) {
        const Layer &L = s->layers[(size_t)(g.first_layer + i)];
        bs_layer_desc d = L.desc;
        d.gamma = L.gamma.data();
        d.beta = L.beta.data();
        d.running_mean = L.mean.data();
        d.running_var = L.var.data();
        d.return_indices = d.kind == BS_MAXPOOL ? 1 : 0;
        // the output size is already fixed: ceil mode is recorded only where it adds a window
        descs[(size_t)i] = d;
    }
    bs_stack *f = nullptr;
    bs_status st = bs_stack_create(descs.data(), g.n_layers, g.in_shape, s->dtype, &f);
    if (st != BS_OK) return st;
    if (std::memcmp(f->out_shape, g.out_shape, sizeof g.out_shape) != 0) {
        bs_stack_destroy(f);
        return BS_ERR_SHAPE;
    }
    bs_plan_options o = s->opts;
    o.host_only = host_only ? 1 : 0;
    o.breadth_first = 0;
    o.force_variant = BS_VARIANT_AUTO;
    st = bs_stack_plan(f, &o);
    if (st != BS_OK) {
        bs_stack_destroy(f);
        return st;
    }
    g.forward = f;
    return BS_OK;
}

// Overlapping 3 x 3 windows (padding 1, stride 1 or 2 that divides the row exactly) on row-major planes whose
// rows are whole vectors and fit one wave: the kernel whose lanes walk down the rows applies.  Average pooling
// with stride 1 stays with the gather kernel (measured on MI355X, 56 x 56 planes: 151 us against 165 us -- one
// new row per iteration does not pay for the iteration; for max pooling the saved recomputation pass does).
bool walks_rows(const bs_stack *s, const BwdStage &g)
{
    const PoolK &p = g.k.pool;
    const int32_t full = s->dtype == BS_F32 ? 4 : 8;
    return s->opts.layout != BS_LAYOUT_NHWC && s->opts.lane_exchange >= 0 &&
           (p.kind == OP_MAXPOOL || (p.kind == OP_AVGSUM && p.sh == 2)) && p.kh == 3 && p.kw == 3 && p.ph == 1 && p.pw == 1 && p.sh == p.sw && (p.sh == 1 || p.sh == 2) && g.k.W % full == 0 &&
           g.k.W / full <= 64 && g.k.Wo * p.sw == g.k.W && g.k.Ho == (g.k.H + 2 - 3) / p.sh + 1;
}

// Stage g = [element-wise list without Add, average pooling 3 x 3 / 1 / 1 that keeps the plane's size] and the stage
// behind it = [max pooling 3 x 3 / 2 / 1 alone, with the element-wise operations that joined it]: one kernel walks
// both levels down the plane (rows of whole 4-cell blocks that fit one wave).
bool walks_two_levels(const bs_stack *s, const BwdStage &g, const BwdStage &nx)
{
    const PoolK &p = g.k.pool, &q = nx.k.pool;
    return s->opts.layout != BS_LAYOUT_NHWC && s->opts.lane_exchange >= 0 && g.n_res == 0 && nx.n_res == 0 && g.k.n_post == 0 &&
           nx.k.n_ew == 0 && g.k.n_ew + nx.k.n_post <= K_BWD_EW && p.kind == OP_AVGSUM && p.kh == 3 && p.kw == 3 && p.sh == 1 &&
           p.sw == 1 && p.ph == 1 && p.pw == 1 && g.k.Ho == g.k.H && g.k.Wo == g.k.W && q.kind == OP_MAXPOOL && q.sh == 2 &&
           walks_rows(s, nx) && g.k.W % 4 == 0 && g.k.W / 4 <= 64;
}

}  // namespace

namespace bs {

void free_backward(bs_stack *s)
{
    if (!s || !s->backward) return;
    for (BwdStage &g : s->backward->stages) bs_stack_destroy(g.forward);
    delete s->backward;
    s->backward = nullptr;
}

}  // namespace bs

extern "C" bs_status bs_stack_plan_backward(bs_stack *stack)
{
    if (!stack) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    // on a host-only plan: stages, stage plans and workspace size, nothing that can run
    const bool host_only = !stack->device_planned;
    if (!host_only && current_device() != stack->device) return BS_ERR_DEVICE;
    free_backward(stack);
    BackwardPlan *plan = new (std::nothrow) BackwardPlan();
    if (!plan) return BS_ERR_ALLOC;
    stack->backward = plan;
    bs_status st = BS_OK;
    try {
        // ---- operations -> stages
        const int64_t N = stack->in_shape[0], C = stack->in_shape[1];
        BwdStage cur;
        int32_t adds = 0;
        bool open = false;
        auto begin = [&](const Op &op) {
            cur = BwdStage();
            cur.first_layer = op.layer;
            const int64_t sh[4] = {N, C, op.in_h, op.in_w};
            std::memcpy(cur.in_shape, sh, sizeof sh);
            std::memcpy(cur.out_shape, sh, sizeof sh);
            cur.k.C = (int32_t)C;
            cur.k.H = cur.k.Ho = op.in_h;
            cur.k.W = cur.k.Wo = op.in_w;
            adds = 0;
            open = true;
        };
        auto close = [&](int32_t last_layer) {
            cur.n_layers = last_layer - cur.first_layer + 1;
            plan->stages.push_back(cur);
            open = false;
        };
        for (size_t i = 0; i < stack->ops.size(); ++i) {
            const Op &op = stack->ops[i];
            if (op.kind == OP_AVGNORM) continue;  // part of the average pooling before it
            if (open && op_is_elementwise(op.kind) &&
                (cur.k.n_ew >= K_BWD_EW || (op.kind == OP_ADD && adds >= K_MAX_RES)))
                close(stack->ops[i - 1].layer);  // capacity of the argument block only
            if (!open) begin(op);
            if (op_is_elementwise(op.kind)) {
                EwOp &e = cur.k.ew[cur.k.n_ew++];
                e.kind = op.kind;
                e.arg = op.param_off;
                if (op.kind == OP_ADD) {
                    e.arg = adds;
                    cur.res_map[adds++] = op.res_slot;
                    cur.n_res = adds;
                }
                continue;
            }
            PoolK &p = cur.k.pool;
            p.kind = op.kind;
            p.kh = op.kh; p.kw = op.kw; p.sh = op.sh; p.sw = op.sw; p.ph = op.ph; p.pw = op.pw;
            p.count_include_pad = op.count_include_pad;
            p.inv_kk = 1.0f / (float)(op.kh * op.kw);
            p.idx_slot = -1;
            cur.idx_slot = op.kind == OP_MAXPOOL ? op.idx_slot : -1;
            cur.k.Ho = op.out_h;
            cur.k.Wo = op.out_w;
            cur.out_shape[2] = op.out_h;
            cur.out_shape[3] = op.out_w;
            close(op.layer);
        }
        if (open) close((int32_t)stack->layers.size() - 1);
        if (plan->stages.empty()) st = BS_ERR_UNSUPPORTED;
        // a stage of element-wise operations only (no Add) behind a max pooling whose kernel finds the picks itself
        // joins that stage: the kernel has the pooling's output at hand (the window maxima) and scales the
        // windows' gradients by the operations' derivatives there -- no kernel, no recomputed input for them
        for (size_t j = 0; j + 1 < plan->stages.size(); ++j) {
            BwdStage &g = plan->stages[j];
            const BwdStage &nx = plan->stages[j + 1];
            bool plain = nx.k.pool.kind == 0 && nx.n_res == 0 && g.k.n_ew + nx.k.n_ew <= K_BWD_EW;
            if (!plain || g.k.pool.kind != OP_MAXPOOL || !walks_rows(stack, g)) continue;
            for (int32_t q = 0; q < nx.k.n_ew; ++q) g.k.ew[g.k.n_ew + q] = nx.k.ew[q];
            g.k.n_post = nx.k.n_ew;
            g.n_layers += nx.n_layers;
            std::memcpy(g.out_shape, nx.out_shape, sizeof g.out_shape);
            plan->stages.erase(plan->stages.begin() + (long)j + 1);
        }

        // an average pooling stage in front of such a max pooling stage: both in one kernel, the plane between
        // them (and its gradient) only in registers
        for (size_t j = 0; j + 1 < plan->stages.size(); ++j) {
            BwdStage &g = plan->stages[j];
            const BwdStage &nx = plan->stages[j + 1];
            if (!walks_two_levels(stack, g, nx)) continue;
            for (int32_t q = 0; q < nx.k.n_post; ++q) g.k.ew[g.k.n_ew + q] = nx.k.ew[q];
            g.k.n_post = nx.k.n_post;
            g.k.pool2 = nx.k.pool;
            g.k.wave_rows = 2;
            g.k.Ho = nx.k.Ho;
            g.k.Wo = nx.k.Wo;
            g.idx_slot = -1;
            g.n_layers += nx.n_layers;
            std::memcpy(g.out_shape, nx.out_shape, sizeof g.out_shape);
            plan->stages.erase(plan->stages.begin() + (long)j + 1);
        }

        // ---- launch geometry, forward stacks, workspace
        const uint64_t es = dtype_size(stack->dtype);
        const int32_t full = stack->dtype == BS_F32 ? 4 : 8;
        const size_t S = plan->stages.size();
        uint64_t off = 0;
        for (size_t j = 0; j < S && st == BS_OK; ++j) {
            BwdStage &g = plan->stages[j];
            const bool nhwc = stack->opts.layout == BS_LAYOUT_NHWC;
            const PoolK &p = g.k.pool;
            const bool tiles2x2 = p.kind != 0 && p.kh == 2 && p.kw == 2 && p.sh == 2 && p.sw == 2 && p.ph == 0 && p.pw == 0 &&
                                  g.k.H == 2 * g.k.Ho && g.k.W == 2 * g.k.Wo;
            uint64_t lanes;
            g.k.nhwc = nhwc ? 1 : 0;
            if (nhwc) {
                // a lane per pixel (per window when 2 x 2 windows tile the plane) and channel vector
                g.vec = g.k.C % full == 0 ? full : 1;
                // (with two or more Adds in the stage the window-owning kernel would keep 4 pixels x vec channels of
                // every residual's factors in registers and spill: those stages gather with recorded picks)
                g.k.direct = tiles2x2 && g.vec == full && g.n_res <= 1;
                lanes = numel(g.in_shape) / (uint64_t)g.vec / (g.k.direct ? 4 : 1);
                g.k.div_wv = make_fastdiv((uint32_t)(g.k.C / g.vec));
                g.k.div_w = make_fastdiv((uint32_t)(g.k.direct ? g.k.Wo : g.k.W));
            } else {
                // one 128-bit vector per lane; 16-bit rows of 4 mod 8 elements (28 x 28 planes): one 64-bit vector
                g.vec = g.k.W % full == 0 ? full : (stack->dtype != BS_F32 && g.k.W % 4 == 0 ? 4 : 1);
                // disjoint 2 x 2 windows that tile the plane: the kernel that owns whole windows
                g.k.direct = tiles2x2 && g.vec > 1;
                // no pooling and rows that are no whole vectors (the 28 x 28, 14 x 14, 7 x 7 planes of
                // 16-bit networks): vectors over the whole tensor, which may straddle two planes
                const int64_t hw = (int64_t)g.k.H * g.k.W;
                if (p.kind == 0 && g.vec != full && numel(g.in_shape) % (uint64_t)full == 0 && hw >= full) {
                    g.vec = full;
                    g.k.flat = 1;
                    g.k.div_w = make_fastdiv((uint32_t)hw);
                }
                lanes = numel(g.in_shape) / (uint64_t)g.vec / (g.k.direct ? 2 : 1);
                g.k.div_wv = make_fastdiv((uint32_t)(g.k.flat ? 1 : g.k.W / g.vec));
                if (g.k.wave_rows == 2) {
                    // two pooling levels in one kernel: 4 cells per lane whatever the element size (registers)
                    BwdK &k = g.k;
                    g.vec = 4;
                    k.div_wv = make_fastdiv((uint32_t)(k.W / 4));
                    k.cbs = k.W / 4;
                    k.spw = 64 / k.cbs;
                    const int64_t planes = g.in_shape[0] * g.in_shape[1];
                    const int32_t rows = (k.H + 1) / 2;  // window rows of the max pooling that cover the plane's rows
                    int32_t rc = std::min(K_BWD_ROWS2_RC, rows);
                    k.chunks = (rows + rc - 1) / rc;
                    k.rc = (rows + k.chunks - 1) / k.chunks;
                    k.chunks = (rows + k.rc - 1) / k.rc;
                    k.units = (uint32_t)(planes * k.chunks);
                    k.div_cbs = make_fastdiv((uint32_t)k.cbs);
                    k.div_chunks = make_fastdiv((uint32_t)k.chunks);
                    lanes = (uint64_t)k.units * (uint64_t)k.cbs;
                } else
                // overlapping 3 x 3 windows on rows that fit one wave: the kernel whose lanes walk down the rows
                if (walks_rows(stack, g) && g.vec == full) {
                    BwdK &k = g.k;
                    k.wave_rows = 1;
                    k.cbs = k.W / full;
                    k.spw = 64 / k.cbs;
                    // window rows per chunk: a chunk also visits the window rows just above and below it
                    const int64_t planes = g.in_shape[0] * g.in_shape[1];
                    const int32_t rows = (k.H + p.sh - 1) / p.sh;  // window rows that cover the plane's rows
                    int32_t rc = std::min(K_BWD_MAXROWS_RC, rows);
                    k.chunks = (rows + rc - 1) / rc;
                    k.rc = (rows + k.chunks - 1) / k.chunks;
                    k.chunks = (rows + k.rc - 1) / k.rc;
                    k.units = (uint32_t)(planes * k.chunks);
                    k.div_cbs = make_fastdiv((uint32_t)k.cbs);
                    k.div_chunks = make_fastdiv((uint32_t)k.chunks);
                    lanes = (uint64_t)k.units * (uint64_t)k.cbs;
                }
            }
            if (lanes > 0x7fffffffull) { st = BS_ERR_UNSUPPORTED; break; }
            g.k.total = (uint32_t)lanes;
            g.k.div_h = make_fastdiv((uint32_t)(g.k.direct ? g.k.Ho : g.k.H));
            g.k.div_c = make_fastdiv((uint32_t)g.k.C);
            g.threads = 256;
            g.grid = (int64_t)((lanes + 255) / 256);
            if (g.k.wave_rows) g.grid = ((int64_t)g.k.units + 4 * g.k.spw - 1) / (4 * g.k.spw);  // whole segments per wave
            const bool is_max = p.kind == OP_MAXPOOL && !g.k.direct && !g.k.wave_rows;  // recorded picks needed
            // the buffers are sized by these shapes: a stage must end where the next one begins
            const int64_t *next = j + 1 < S ? plan->stages[j + 1].in_shape : stack->out_shape;
            if (std::memcmp(g.out_shape, next, sizeof g.out_shape) != 0) { st = BS_ERR_SHAPE; break; }
            if (j + 1 < S || is_max) st = make_forward(stack, g, host_only);
            if (st != BS_OK) break;
            if (j > 0) {
                g.a_off = off;
                off += align256(numel(g.in_shape) * es);
                g.g_off = off;
                off += align256(numel(g.in_shape) * es);
            }
            if (is_max) {
                g.idx_off = off;
                off += align256(numel(g.out_shape) * 4);
            }
            if (g.forward) plan->fwd_ws_bytes = std::max(plan->fwd_ws_bytes, g.forward->workspace_bytes);
        }
        if (st == BS_OK) {
            if (plan->stages[S - 1].forward) {
                plan->last_out_off = off;
                off += align256(numel(plan->stages[S - 1].out_shape) * es);
            }
            plan->fwd_ws_off = off;
            off += align256(plan->fwd_ws_bytes);
            plan->workspace_bytes = off;
        }
    } catch (const std::bad_alloc &) {
        st = BS_ERR_ALLOC;
    }
    if (st != BS_OK) free_backward(stack);
    return st;
}

#if defined(BS_BWD_AUDIT)
// Audit builds: 64 device counters, one per checked access site of the backward kernels.
static uint32_t *audit_counters()
{
    static uint32_t *p = nullptr;
    if (!p && hipMalloc(reinterpret_cast<void **>(&p), 64 * sizeof(uint32_t)) == hipSuccess) (void)hipMemset(p, 0, 64 * sizeof(uint32_t));
    return p;
}
extern "C" __attribute__((visibility("default"))) int32_t bs_backward_audit_read(uint32_t *out64)
{
    uint32_t *p = audit_counters();
    return p && hipMemcpy(out64, p, 64 * sizeof(uint32_t), hipMemcpyDeviceToHost) == hipSuccess ? 0 : 1;
}
#endif

extern "C" uint64_t bs_stack_backward_workspace_bytes(const bs_stack *stack)
{
    return stack && stack->backward ? stack->backward->workspace_bytes : 0;
}

extern "C" int32_t bs_stack_backward_num_stages(const bs_stack *stack)
{
    return stack && stack->backward ? (int32_t)stack->backward->stages.size() : -1;
}

extern "C" bs_status bs_stack_backward(const bs_stack *stack, const void *in, const void *const *residuals,
                                       const int32_t *const *indices, const void *grad_out, void *grad_in,
                                       void *const *grad_residuals, void *workspace, uint64_t workspace_bytes,
                                       void *stream)
{
    return bs_stack_backward_strided(stack, in, 0, residuals, indices, grad_out, 0, grad_in, 0, grad_residuals, workspace,
                                     workspace_bytes, stream);
}

extern "C" bs_status bs_stack_backward_strided(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                               const void *const *residuals, const int32_t *const *indices,
                                               const void *grad_out, int64_t grad_out_batch_stride, void *grad_in,
                                               int64_t grad_in_batch_stride, void *const *grad_residuals, void *workspace,
                                               uint64_t workspace_bytes, void *stream)
{
    if (!stack || !in || !grad_out) return BS_ERR_NULL;
    if (!stack->planned || !stack->device_planned || !stack->backward) return BS_ERR_NOT_PLANNED;
    if (current_device() != stack->device) return BS_ERR_DEVICE;
    const BackwardPlan &plan = *stack->backward;
    if (stack->n_res > 0 && !residuals) return BS_ERR_NULL;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (!residuals[i]) return BS_ERR_NULL;

    // ---- the caller's buffers: strides, alignment, workspace, no output over an input or another output
    const uint64_t es = dtype_size(stack->dtype);
    TensorBytes ins[2 + BS_MAX_RESIDUALS + 1 + BS_MAX_INDEX_OUTPUTS], outs[1 + BS_MAX_RESIDUALS];
    int n_in = 0, n_out = 0;
    bs_status bst = resolve_slice(stack, stack->in_shape, in, in_batch_stride, ins[n_in++]);
    if (bst != BS_OK) return bst;
    bst = resolve_slice(stack, stack->out_shape, grad_out, grad_out_batch_stride, ins[n_in++]);
    if (bst != BS_OK) return bst;
    auto dense = [](const void *p, uint64_t bytes) { return TensorBytes{p, 1, bytes, bytes}; };
    for (int32_t i = 0; i < stack->n_res; ++i) ins[n_in++] = dense(residuals[i], numel(stack->res_shape[i]) * es);
    if (grad_in) {
        bst = resolve_slice(stack, stack->in_shape, grad_in, grad_in_batch_stride, outs[n_out++]);
        if (bst != BS_OK) return bst;
    }
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (grad_residuals && grad_residuals[i]) outs[n_out++] = dense(grad_residuals[i], numel(stack->res_shape[i]) * es);
    if (plan.workspace_bytes > 0) {
        if (!workspace || workspace_bytes < plan.workspace_bytes) return BS_ERR_WORKSPACE;
        ins[n_in++] = dense(workspace, plan.workspace_bytes);
    }
    for (int32_t i = 0; i < stack->n_idx; ++i)
        if (indices && indices[i]) ins[n_in++] = dense(indices[i], numel(stack->idx_shape[i]) * 4);
    for (int i = 0; i < n_in; ++i)
        if (!aligned16(ins[i].p)) return BS_ERR_ALIGN;
    for (int i = 0; i < n_out; ++i) {
        if (!aligned16(outs[i].p)) return BS_ERR_ALIGN;
        for (int j = 0; j < n_in; ++j)
            if (tensors_overlap(outs[i], ins[j])) return BS_ERR_ALIAS;
        for (int j = 0; j < i; ++j)
            if (tensors_overlap(outs[i], outs[j])) return BS_ERR_ALIAS;
    }
    // what the kernels add per image (row-major) or per pixel (channels-last) to reach a slice's elements
    const bool nhwc = stack->opts.layout == BS_LAYOUT_NHWC;
    auto extra = [&](const int64_t *shape, int64_t stride) -> uint32_t {
        const int64_t image = shape[1] * shape[2] * shape[3];
        return (uint32_t)(nhwc ? (stride - image) / (shape[2] * shape[3]) : stride - image);
    };
    const uint32_t a_extra = extra(stack->in_shape, in_batch_stride), gin_extra = grad_in ? extra(stack->in_shape, grad_in_batch_stride) : 0,
                   gout_extra = extra(stack->out_shape, grad_out_batch_stride);

    char *ws = static_cast<char *>(workspace);
    const size_t S = plan.stages.size();
    // picks the caller kept from the forward pass (index outputs of bs_stack_run), per stage
    auto kept = [&](const BwdStage &g) -> const int32_t * {
        return indices && g.idx_slot >= 0 ? indices[g.idx_slot] : nullptr;
    };
    // ---- recompute: the input of every stage after the first, the picks of every max pooling
    for (size_t j = 0; j < S; ++j) {
        const BwdStage &g = plan.stages[j];
        if (!g.forward) continue;
        // the last stage is run forward for its picks alone: not when the caller kept them
        if (j + 1 == S && kept(g)) continue;
        const void *a = j == 0 ? in : ws + g.a_off;
        void *out = j + 1 < S ? ws + plan.stages[j + 1].a_off : ws + plan.last_out_off;
        const void *res[K_MAX_RES] = {nullptr, nullptr, nullptr, nullptr};
        for (int32_t r = 0; r < g.n_res; ++r) res[r] = residuals[g.res_map[r]];
        const bool picks = g.k.pool.kind == OP_MAXPOOL && !g.k.direct && !g.k.wave_rows;
        int32_t *idx[1] = {picks ? reinterpret_cast<int32_t *>(ws + g.idx_off) : nullptr};
        const bs_status st = bs_stack_run_strided(g.forward, a, j == 0 ? in_batch_stride : 0, res, out, 0,
                                                  g.forward->n_idx > 0 ? idx : nullptr, ws + plan.fwd_ws_off, plan.fwd_ws_bytes, stream);
        if (st != BS_OK) return st;
    }
    // ---- gradients, last stage first
    for (size_t j = S; j-- > 0;) {
        const BwdStage &g = plan.stages[j];
        BwdK k = g.k;
        k.a = j == 0 ? in : ws + g.a_off;
        k.g_out = j + 1 == S ? grad_out : ws + plan.stages[j + 1].g_off;
        k.g_in = j == 0 ? grad_in : ws + g.g_off;
        k.idx = g.k.pool.kind == OP_MAXPOOL && !g.k.direct && !g.k.wave_rows ? reinterpret_cast<const int32_t *>(ws + g.idx_off) : nullptr;
        if (k.idx && j + 1 == S && kept(g)) k.idx = kept(g);
        k.params = stack->dev_params;
        k.a_extra = j == 0 ? a_extra : 0;
        k.gin_extra = j == 0 ? gin_extra : 0;
        k.gout_extra = j + 1 == S ? gout_extra : 0;
#if defined(BS_BWD_AUDIT)
        {
            auto reach = [&](const TensorBytes &t) { return (uint32_t)(((t.images - 1) * t.stride_bytes + t.image_bytes) / es); };
            k.audit_lim[0] = j == 0 ? reach(ins[0]) : (uint32_t)numel(g.in_shape);
            k.audit_lim[1] = j + 1 == S ? reach(ins[1]) : (uint32_t)numel(g.out_shape);
            k.audit_lim[2] = j == 0 && grad_in ? reach(outs[0]) : (uint32_t)numel(g.in_shape);
            k.audit = audit_counters();
        }
#endif
        bool wanted = k.g_in != nullptr;
        for (int32_t r = 0; r < g.n_res; ++r) {
            k.res[r] = residuals[g.res_map[r]];
            k.g_res[r] = grad_residuals ? grad_residuals[g.res_map[r]] : nullptr;
            wanted = wanted || k.g_res[r] != nullptr;
        }
        if (!wanted) continue;  // first stage, and the caller asked for none of its gradients
        const bs_status st = launch_backward_stage(k, stack->dtype, g.vec, g.grid, g.threads, stream);
        if (st != BS_OK) return st;
    }
    return BS_OK;
}
