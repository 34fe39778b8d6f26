// Execution phase (Section 4.2): check the caller's buffers, then enqueue the
// sequences of the stack one after the other on the caller's stream.  Intermediate
// tensors between sequences alternate between the two halves of the workspace.
// Nothing here synchronises or allocates.
#include <cstdint>

#include "bs_internal.h"

using namespace bs;

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline bool overlap(const void *a, uint64_t na, const void *b, uint64_t nb)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + nb && y < x + na;
}

static inline uint64_t numel(const int64_t *sh) { return (uint64_t)sh[0] * sh[1] * sh[2] * sh[3]; }

extern "C" bs_status bs_stack_run(const bs_stack *stack, const void *in, const void *const *residuals,
                                  void *out, int32_t *const *indices, void *workspace,
                                  uint64_t workspace_bytes, void *stream)
{
    if (!stack || !in || !out) return BS_ERR_NULL;
    if (!stack->planned || !stack->device_planned) return BS_ERR_NOT_PLANNED;
    if (current_device() != stack->device) return BS_ERR_DEVICE;
    if (stack->n_res > 0 && !residuals) return BS_ERR_NULL;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (!residuals[i]) return BS_ERR_NULL;
    if (!aligned16(in) || !aligned16(out)) return BS_ERR_ALIGN;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (!aligned16(residuals[i])) return BS_ERR_ALIGN;
    if (indices)
        for (int32_t i = 0; i < stack->n_idx; ++i)
            if (indices[i] && !aligned16(indices[i])) return BS_ERR_ALIGN;
    if (stack->workspace_bytes > 0) {
        if (!workspace || workspace_bytes < stack->workspace_bytes) return BS_ERR_WORKSPACE;
        if (!aligned16(workspace)) return BS_ERR_ALIGN;
    }
    const uint64_t es = dtype_size(stack->dtype);
    const uint64_t in_bytes = numel(stack->in_shape) * es, out_bytes = numel(stack->out_shape) * es;
    if (overlap(in, in_bytes, out, out_bytes) && !(in == out && !stack->has_pool)) return BS_ERR_ALIAS;
    for (int32_t i = 0; i < stack->n_res; ++i)
        if (overlap(residuals[i], numel(stack->res_shape[i]) * es, out, out_bytes)) return BS_ERR_ALIAS;
    if (stack->workspace_bytes > 0 &&
        (overlap(workspace, stack->workspace_bytes, out, out_bytes) ||
         overlap(workspace, stack->workspace_bytes, in, in_bytes)))
        return BS_ERR_ALIAS;

    const size_t n = stack->seqs.size();
    const bool traced = trace_enabled();
    const void *cur_in = in;
    for (size_t i = 0; i < n; ++i) {
        void *cur_out = out;
        if (i + 1 < n) {
            char *half = static_cast<char *>(workspace) + ((i & 1) ? stack->ws_half_bytes : 0);
            cur_out = half;
        }
        if (traced) trace_push_sequence(stack->seqs[i], i, n);
        bs_status st = launch_sequence(stack, stack->seqs[i], cur_in, cur_out, residuals, indices, stream);
        if (traced) trace_pop();
        if (st != BS_OK) return st;
        cur_in = cur_out;
    }
    return BS_OK;
}
