// Execution phase (Section 4.2): check the caller's buffers, then enqueue the
// sequences of the stack one after the other on the caller's stream.  Intermediate
// tensors between sequences alternate between the two halves of the workspace.
// Nothing here synchronises or allocates.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "bs_internal.h"

using namespace bs;

// Device memory for callers that may not allocate (bs_stack_run_static): the workspace between
// sequences lives in this array instead of a caller's buffer.  Every GPU the library's code
// object is loaded on holds its own copy, at its own address, until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; g_scratch_ptr[device] is the memory.
static __device__ __align__(256) unsigned char scratch[BS_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int K_MAX_DEVICES = 64;
void *g_scratch_ptr[K_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Address of `scratch` on `device`, which must be the current device.  Resolved once per device.
bs_status scratch_address(int device, void **out)
{
    if (device < 0 || device >= K_MAX_DEVICES) return BS_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_hip_error((int32_t)e);
            return BS_ERR_HIP;
        }
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return BS_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool overlap(const void *a, uint64_t na, const void *b, uint64_t nb)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
}

inline uint64_t numel(const int64_t *sh) { return (uint64_t)sh[0] * sh[1] * sh[2] * sh[3]; }

// A tensor of `images` images of `image_bytes` each, consecutive images `stride_bytes` apart.
struct Span {
    const void *p;
    uint64_t images, image_bytes, stride_bytes;
    uint64_t extent() const { return (images - 1) * stride_bytes + image_bytes; }
    bool dense() const { return stride_bytes == image_bytes; }
};

// Do the two tensors share a byte?  Exact for dense tensors; for strided ones it may say yes
// for disjoint layouts it cannot prove disjoint (never no for overlapping ones).
bool spans_overlap(const Span &a, const Span &b)
{
    if (!overlap(a.p, a.extent(), b.p, b.extent())) return false;
    if (a.dense() && b.dense()) return true;
    if (a.stride_bytes != b.stride_bytes) return true;
    // Same stride S: image i of a covers [pa + i*S, +la), image j of b covers [pb + j*S, +lb).
    // With d = (pb - pa) mod S they are disjoint for all i, j when la <= d and d + lb <= S.
    const uint64_t S = a.stride_bytes;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a.p), pb = reinterpret_cast<uintptr_t>(b.p);
    const uint64_t d = pb >= pa ? (pb - pa) % S : (S - (pa - pb) % S) % S;
    return !(a.image_bytes <= d && d + b.image_bytes <= S);
}

// Everything bs_stack_run checks about its pointer arguments; compares addresses only.  On
// success the batch strides are resolved (0 -> dense).
bs_status check_buffers(const bs_stack *stack, const void *in, int64_t &in_stride,
                        const void *const *residuals, const void *out, int64_t &out_stride,
                        int32_t *const *indices, const void *workspace, uint64_t workspace_bytes)
{
    if (stack->n_res > 0 && !residuals) return BS_ERR_NULL;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (!residuals[i]) return BS_ERR_NULL;

    const uint64_t es = dtype_size(stack->dtype);
    const uint64_t images = (uint64_t)stack->in_shape[0];
    const uint64_t in_image = numel(stack->in_shape) / images, out_image = numel(stack->out_shape) / images;
    if (in_stride == 0) in_stride = (int64_t)in_image;
    if (out_stride == 0) out_stride = (int64_t)out_image;
    if (in_stride < (int64_t)in_image || out_stride < (int64_t)out_image) return BS_ERR_SHAPE;
    const bool nhwc = stack->opts.layout == BS_LAYOUT_NHWC;
    if (nhwc) {
        // a channel slice of a channels-last tensor: every pixel of the larger tensor holds the
        // slice's C channels and skips the rest, so the batch stride is a whole number of pixels
        const int64_t hw_in = stack->in_shape[2] * stack->in_shape[3], hw_out = stack->out_shape[2] * stack->out_shape[3];
        if (in_stride % hw_in != 0 || out_stride % hw_out != 0) return BS_ERR_SHAPE;
        if ((uint64_t)(in_stride / hw_in) * es % 16 != 0 && in_stride != (int64_t)in_image) return BS_ERR_ALIGN;
        if ((uint64_t)(out_stride / hw_out) * es % 16 != 0 && out_stride != (int64_t)out_image) return BS_ERR_ALIGN;
        if ((uint64_t)in_stride * images > 0x7fffffffull || (uint64_t)out_stride * images > 0x7fffffffull) return BS_ERR_SHAPE;
    }
    if (in_stride > 0x7fffffffll || out_stride > 0x7fffffffll) return BS_ERR_SHAPE;
    Span sin{in, images, in_image * es, (uint64_t)in_stride * es};
    Span sout{out, images, out_image * es, (uint64_t)out_stride * es};
    if (nhwc) {
        // the bytes of a channels-last slice's image are spread over the larger tensor's image:
        // from its first pixel to the slice's channels of its last pixel
        auto spread = [&](const int64_t *sh, int64_t stride) {
            const uint64_t hw = (uint64_t)(sh[2] * sh[3]);
            return ((hw - 1) * ((uint64_t)stride / hw) + (uint64_t)sh[1]) * es;
        };
        if (!sin.dense()) sin.image_bytes = spread(stack->in_shape, in_stride);
        if (!sout.dense()) sout.image_bytes = spread(stack->out_shape, out_stride);
    }

    if (!aligned16(in) || !aligned16(out)) return BS_ERR_ALIGN;
    if (sin.stride_bytes % 16 != 0 && !sin.dense()) return BS_ERR_ALIGN;
    if (sout.stride_bytes % 16 != 0 && !sout.dense()) return BS_ERR_ALIGN;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (!aligned16(residuals[i])) return BS_ERR_ALIGN;
    if (indices)
        for (int32_t i = 0; i < stack->n_idx; ++i)
            if (indices[i] && !aligned16(indices[i])) return BS_ERR_ALIGN;
    if (stack->workspace_bytes > 0) {
        if (!workspace || workspace_bytes < stack->workspace_bytes) return BS_ERR_WORKSPACE;
        if (!aligned16(workspace)) return BS_ERR_ALIGN;
    }

    const bool in_place = in == out && sin.stride_bytes == sout.stride_bytes && !stack->has_pool;
    if (!in_place && spans_overlap(sin, sout)) return BS_ERR_ALIAS;
    for (int32_t i = 0; i < stack->n_res; ++i) {
        const uint64_t b = numel(stack->res_shape[i]) * es;
        if (spans_overlap(Span{residuals[i], 1, b, b}, sout)) return BS_ERR_ALIAS;
    }
    if (stack->workspace_bytes > 0) {
        const Span ws{workspace, 1, stack->workspace_bytes, stack->workspace_bytes};
        if (spans_overlap(ws, sout) || spans_overlap(ws, sin)) return BS_ERR_ALIAS;
    }
    // index outputs are written like `out`: they may share bytes with nothing else
    if (indices) {
        for (int32_t i = 0; i < stack->n_idx; ++i) {
            if (!indices[i]) continue;
            const uint64_t b = numel(stack->idx_shape[i]) * 4;
            const Span si{indices[i], 1, b, b};
            if (spans_overlap(si, sin) || spans_overlap(si, sout)) return BS_ERR_ALIAS;
            for (int32_t j = 0; j < stack->n_res; ++j) {
                const uint64_t rb = numel(stack->res_shape[j]) * es;
                if (spans_overlap(si, Span{residuals[j], 1, rb, rb})) return BS_ERR_ALIAS;
            }
            if (stack->workspace_bytes > 0 &&
                spans_overlap(si, Span{workspace, 1, stack->workspace_bytes, stack->workspace_bytes}))
                return BS_ERR_ALIAS;
            for (int32_t j = 0; j < i; ++j) {
                if (!indices[j]) continue;
                const uint64_t jb = numel(stack->idx_shape[j]) * 4;
                if (spans_overlap(si, Span{indices[j], 1, jb, jb})) return BS_ERR_ALIAS;
            }
        }
    }

    return BS_OK;
}

bs_status run(const bs_stack *stack, const void *in, int64_t in_stride, const void *const *residuals,
              void *out, int64_t out_stride, int32_t *const *indices, void *workspace,
              uint64_t workspace_bytes, void *stream)
{
    if (!stack || !in || !out) return BS_ERR_NULL;
    if (!stack->planned || !stack->device_planned) return BS_ERR_NOT_PLANNED;
    if (current_device() != stack->device) return BS_ERR_DEVICE;
    const bs_status cs = check_buffers(stack, in, in_stride, residuals, out, out_stride, indices, workspace,
                                       workspace_bytes);
    if (cs != BS_OK) return cs;
    const uint64_t images = (uint64_t)stack->in_shape[0];
    const uint64_t in_image = numel(stack->in_shape) / images, out_image = numel(stack->out_shape) / images;

    const size_t n = stack->seqs.size();
    const bool traced = trace_enabled();
    const void *cur_in = in;
    for (size_t i = 0; i < n; ++i) {
        void *cur_out = out;
        if (i + 1 < n) {
            char *half = static_cast<char *>(workspace) + ((i & 1) ? stack->ws_half_bytes : 0);
            cur_out = half;
        }
        // only the stack's own input and output can be slices; the workspace halves are dense
        const uint32_t in_extra = i == 0 ? (uint32_t)((uint64_t)in_stride - in_image) : 0u;
        const uint32_t out_extra = i + 1 == n ? (uint32_t)((uint64_t)out_stride - out_image) : 0u;
        if (traced) trace_push_sequence(stack->seqs[i], i, n);
        bs_status st = launch_sequence(stack, stack->seqs[i], cur_in, cur_out, in_extra, out_extra,
                                       residuals, indices, stream);
        if (traced) trace_pop();
        if (st != BS_OK) return st;
        cur_in = cur_out;
    }
    return BS_OK;
}

}  // namespace

namespace bs {

// A tensor of `shape` (N, C, H, W) that may be a channel slice of a larger one in the plan's layout: resolves the
// batch stride (elements; 0 -> dense), checks it as bs_stack_run_strided does and describes the bytes it covers.
bs_status resolve_slice(const bs_stack *stack, const int64_t *shape, const void *p, int64_t &stride, TensorBytes &out)
{
    const uint64_t es = dtype_size(stack->dtype);
    const uint64_t images = (uint64_t)shape[0], image = numel(shape) / images;
    if (stride == 0) stride = (int64_t)image;
    if (stride < (int64_t)image || stride > 0x7fffffffll) return BS_ERR_SHAPE;
    if (!aligned16(p)) return BS_ERR_ALIGN;
    out = TensorBytes{p, images, image * es, (uint64_t)stride * es};
    const bool dense = stride == (int64_t)image;
    if (stack->opts.layout == BS_LAYOUT_NHWC) {
        const int64_t hw = shape[2] * shape[3];
        if (stride % hw != 0) return BS_ERR_SHAPE;
        if (!dense && (uint64_t)(stride / hw) * es % 16 != 0) return BS_ERR_ALIGN;
        if ((uint64_t)stride * images > 0x7fffffffull) return BS_ERR_SHAPE;
        // the bytes of a channels-last slice's image: from its first pixel to the slice's channels of its last pixel
        if (!dense) out.image_bytes = ((uint64_t)(hw - 1) * ((uint64_t)stride / (uint64_t)hw) + (uint64_t)shape[1]) * es;
    } else if (!dense && out.stride_bytes % 16 != 0) {
        return BS_ERR_ALIGN;
    }
    return BS_OK;
}

bool tensors_overlap(const TensorBytes &a, const TensorBytes &b)
{
    return spans_overlap(Span{a.p, a.images, a.image_bytes, a.stride_bytes}, Span{b.p, b.images, b.image_bytes, b.stride_bytes});
}

}  // namespace bs


extern "C" bs_status bs_stack_run(const bs_stack *stack, const void *in, const void *const *residuals,
                                  void *out, int32_t *const *indices, void *workspace,
                                  uint64_t workspace_bytes, void *stream)
{
    return run(stack, in, 0, residuals, out, 0, indices, workspace, workspace_bytes, stream);
}

extern "C" uint64_t bs_static_workspace_capacity(void) { return BS_STATIC_WORKSPACE_BYTES; }

bs_status bs::static_workspace_prepare(int device)
{
    void *ptr = nullptr;
    return scratch_address(device, &ptr);
}

extern "C" bs_status bs_stack_run_static(const bs_stack *stack, const void *in, const void *const *residuals,
                                         void *out, int32_t *const *indices, void *stream)
{
    if (!stack) return BS_ERR_NULL;
    if (!stack->planned || !stack->device_planned) return BS_ERR_NOT_PLANNED;
    if (stack->workspace_bytes > BS_STATIC_WORKSPACE_BYTES) return BS_ERR_WORKSPACE;
    if (current_device() != stack->device) return BS_ERR_DEVICE;
    void *ptr = nullptr;  // resolved by bs_stack_plan on this device; here only if that was skipped
    const bs_status st = scratch_address(stack->device, &ptr);
    if (st != BS_OK) return st;
    return run(stack, in, 0, residuals, out, 0, indices, ptr, BS_STATIC_WORKSPACE_BYTES, stream);
}

extern "C" bs_status bs_stack_run_strided(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                          const void *const *residuals, void *out,
                                          int64_t out_batch_stride, int32_t *const *indices,
                                          void *workspace, uint64_t workspace_bytes, void *stream)
{
    return run(stack, in, in_batch_stride, residuals, out, out_batch_stride, indices, workspace,
               workspace_bytes, stream);
}

extern "C" bs_status bs_stack_check_buffers(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                            const void *const *residuals, const void *out,
                                            int64_t out_batch_stride, int32_t *const *indices,
                                            const void *workspace, uint64_t workspace_bytes)
{
    if (!stack || !in || !out) return BS_ERR_NULL;
    if (!stack->planned) return BS_ERR_NOT_PLANNED;
    return check_buffers(stack, in, in_batch_stride, residuals, out, out_batch_stride, indices, workspace,
                         workspace_bytes);
}
