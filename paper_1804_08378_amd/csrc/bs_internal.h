// Internal declarations shared by the host side (stack, planner, run) and the HIP
// kernels of libbrainslug_hip.  Nothing here is part of the public C ABI.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "brainslug.h"
#include "bs_kargs.h"

namespace bs {

struct Op {
    int32_t kind = 0;
    int32_t layer = -1;       // index in the layer list
    int32_t kh = 1, kw = 1, sh = 1, sw = 1, ph = 0, pw = 0;
    int32_t count_include_pad = 1;  // average: 0 in-range cells, 1 kh * kw, 2 cells inside the padded plane
    int32_t ceil = 0;         // ceil mode added a last window that overhangs the padded plane
    int32_t idx_slot = -1;    // stack-wide index-output number (max pool with return_indices)
    int32_t res_slot = -1;    // stack-wide residual number (Add)
    int32_t param_off = -1;   // BN: float offset of scale[C] in the parameter table; shift follows
    int32_t in_h = 0, in_w = 0, out_h = 0, out_w = 0;  // plane size before / after this op
};

struct Step {
    int32_t first_op = 0, n_ops = 0, pool_op = -1, sequence = -1;
};

FastDiv make_fastdiv(uint32_t d);

struct Sequence {
    int32_t first_step = 0, n_steps = 0;
    int32_t first_op = 0, n_ops = 0;
    int32_t first_layer = 0, n_layers = 0;
    int32_t variant = 0;
    int32_t n_levels = 0;
    int32_t tile_rows = 0, tile_cols = 0, planes_per_group = 1;
    int32_t halo_rows = 0, halo_cols = 0;
    int32_t threads = 256;
    int32_t vec = 1;
    int64_t grid = 0;
    uint64_t lds_bytes = 0;
    int64_t in_shape[4] = {0, 0, 0, 0}, out_shape[4] = {0, 0, 0, 0};
    double redundancy = 1.0;
    // which stack-wide residual / index slots the sequence-local slots refer to
    int32_t n_res = 0, res_map[K_MAX_RES] = {-1, -1, -1, -1};
    int32_t n_idx = 0, idx_map[K_MAX_IDX] = {-1, -1, -1, -1};
    // argument blocks; pointers are filled in at run time
    StreamK stream{};
    PoolDirectK direct{};
    PoolRowsK rows{};
    PoolRows2K rows2{};
    RowsChainK chain{};
    LdsSeqK lds{};
    NhwcK nhwc{};
    NhwcTile2K nhwc2{};
    // run-time build (hipFunction_t) without / with index outputs; null = pre-compiled kernel
    int32_t jit = 0;
    void *jit_fn[2] = {nullptr, nullptr};
};

struct Layer {
    bs_layer_desc desc{};
    std::vector<float> gamma, beta, mean, var;
    std::vector<float> scale, shift;  // folded
    int64_t in_shape[4] = {0, 0, 0, 0}, out_shape[4] = {0, 0, 0, 0};
};

// Backward pass: the stack cut into stages (element-wise operations, then at most one pooling
// operation).  Stage j's input is recomputed by forward stacks over the stages before it.
struct BwdStage {
    int32_t first_layer = 0, n_layers = 0;
    int64_t in_shape[4] = {0, 0, 0, 0}, out_shape[4] = {0, 0, 0, 0};
    BwdK k{};
    int32_t n_res = 0, res_map[K_MAX_RES] = {-1, -1, -1, -1};  // stack-wide residual numbers
    int32_t vec = 1, threads = 256;
    int64_t grid = 0;
    bs_stack *forward = nullptr;  // this stage alone as a forward stack (null: its output and picks are not needed)
    int32_t idx_slot = -1;        // the stack's index output that holds this stage's max-pooling picks, if it has one
    uint64_t a_off = 0;           // workspace offsets: the stage's input (stages >= 1),
    uint64_t idx_off = 0;         // the picks of its max pooling,
    uint64_t g_off = 0;           // the gradient with respect to its input (stages >= 1)
};

struct BackwardPlan {
    std::vector<BwdStage> stages;
    uint64_t workspace_bytes = 0;
    uint64_t last_out_off = 0;    // output of the last stage's forward stack (only its picks are used)
    uint64_t fwd_ws_off = 0, fwd_ws_bytes = 0;  // workspace of the forward stacks
};

struct Limits {
    uint64_t max_lds_bytes = 0;
    int32_t num_cus = 0;
};

}  // namespace bs

struct bs_stack {
    std::vector<bs::Layer> layers;
    int64_t in_shape[4] = {0, 0, 0, 0}, out_shape[4] = {0, 0, 0, 0};
    int32_t dtype = BS_F32;
    int32_t n_res = 0, n_idx = 0;
    int64_t res_shape[BS_MAX_RESIDUALS][4] = {};
    int64_t idx_shape[BS_MAX_INDEX_OUTPUTS][4] = {};
    bool has_pool = false;

    // plan
    bool planned = false, device_planned = false;
    int device = -1;
    bs_plan_options opts{};
    std::vector<bs::Op> ops;
    std::vector<bs::Step> steps;
    std::vector<bs::Sequence> seqs;
    std::vector<float> host_params;  // [scale(C), shift(C)] per BatchNorm, in op order
    float *dev_params = nullptr;
    uint64_t workspace_bytes = 0;
    uint64_t ws_half_bytes = 0;  // size of each of the two ping-pong halves
    uint64_t algorithmic_bytes = 0;
    bool jit_failed = false;  // a run-time build failed during this plan: plan again without
    bs::BackwardPlan *backward = nullptr;  // bs_stack_plan_backward
};

namespace bs {

size_t dtype_size(int32_t dtype);
// The signature tables of the sliding-window and tile kernels are compiled into the library
// for float32 and bfloat16; binary16 stacks get those kernels as run-time builds.
inline bool dtype_has_tables(int32_t dtype) { return dtype == BS_F32 || dtype == BS_BF16; }
// Column-block width (elements per lane and row) of the one- / two-level sliding-window kernels.
inline int32_t rows_vec(int32_t dtype) { return dtype == BS_F32 ? 4 : K_ROWS_VEC16; }
inline int32_t rows2_vec(int32_t dtype) { return dtype == BS_F32 ? K_ROWS2_VEC32 : K_ROWS2_VEC16; }
// the same for the kernels whose lanes exchange edge columns
inline int32_t xrows_vec(int32_t dtype) { return dtype == BS_F32 ? K_XROWS_VEC32 : K_XROWS_VEC16; }
inline int32_t xrows2_vec(int32_t dtype) { return dtype == BS_F32 ? K_XROWS2_VEC32 : K_XROWS2_VEC16; }

// planner (host only)
bs_status build_operations(bs_stack *s);
bs_status group_steps(bs_stack *s);
bs_status group_sequences(bs_stack *s, const bs_plan_options &o, const Limits &lim);

// device side (bs_kernels.hip)
bs_status device_limits(Limits *lim, int *device);
int current_device();  // -1 if it cannot be queried
bs_status upload_params(bs_stack *s);
void free_params(bs_stack *s);
// in_extra / out_extra: elements between the end of one image and the start of the next in
// the sequence's input / output (0 = dense)
bs_status launch_sequence(const bs_stack *s, const Sequence &q, const void *in, void *out,
                          uint32_t in_extra, uint32_t out_extra, const void *const *res,
                          int32_t *const *idx, void *stream);
void set_hip_error(int32_t e);
// bs_run.cpp: the bytes of a tensor of `images` images of `image_bytes` each, `stride_bytes` apart (a channel slice
// when the stride exceeds the image), how the strided entry points validate one, and whether two share a byte
// (exact for dense tensors; never "no" for overlapping ones)
struct TensorBytes {
    const void *p;
    uint64_t images, image_bytes, stride_bytes;
};
bs_status resolve_slice(const bs_stack *stack, const int64_t *shape, const void *p, int64_t &stride, TensorBytes &out);
bool tensors_overlap(const TensorBytes &a, const TensorBytes &b);
// bs_run.cpp: resolve the address of the library's static scratch array on `device` (the current one)
bs_status static_workspace_prepare(int device);
// bs_nhwc.hip: channels-last kernels (element-wise, and one pooling step per sequence)
void nhwc_block(const PoolK &p, int32_t vec, int32_t dtype, int32_t &ohb, int32_t &owb);  // output pixels per lane
int32_t nhwc_plane_group(int64_t hw, int32_t vec, const PoolK &p, int32_t H, int32_t W, int32_t Ho, int32_t Wo);
bs_status launch_nhwc(const NhwcK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, uint64_t lds_bytes,
                      void *stream);
// bs_nhwc_tile.hip: channels-last, two pooling steps per sequence
bool nhwc_tile2_supported(const PoolK &pool1, const PoolK &pool2);
// bs_nhwc_rows.hip: the same pair of steps in registers, for the windows and lists it is compiled for
bool nhwc_rows2_supported(const NhwcTile2K &k, int32_t dtype);
bs_status launch_nhwc_rows2(const NhwcTile2K &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, void *stream);
bool nhwc_tile2_sizes_ok(int64_t H, int64_t W, int64_t C, int64_t extra_per_pixel, int32_t dtype);
void nhwc_tile2_shape(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t (&r0)[2], int32_t (&r1)[2], int32_t (&cells)[2],
                      int32_t (&bw)[2]);
bool nhwc_tile2_fits(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t pl);
uint64_t nhwc_tile2_lds(const PoolK &p1, const PoolK &p2, int32_t th, int32_t tw, int32_t cvb, int32_t n_bn, int32_t vec);
bs_status launch_nhwc_tile2(const NhwcTile2K &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, uint64_t lds_bytes,
                            void *stream);
// bs_rows.hip: *_supported = the signature is in the pre-compiled table; *_buildable = the
// kernel template can be instantiated for it at run time; *_expr = that instance's name
bool rows_supported(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post);
bool rows_buildable(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post, int32_t vec);
std::string rows_expr(const PoolRowsK &k, int32_t dtype, bool want_idx);
bs_status launch_rows(const PoolRowsK &k, int32_t dtype, int64_t grid, int32_t threads, void *stream);
// bs_rows2.hip
bool rows2_supported(const PoolRows2K &k);
bool rows2_buildable(const PoolRows2K &k, int32_t vec);
std::string rows2_expr(const PoolRows2K &k, int32_t dtype, bool want_idx);
bs_status launch_rows2(const PoolRows2K &k, int32_t dtype, int64_t grid, int32_t threads, void *stream);
// bs_xrows.hip: the sliding-window kernels whose lanes exchange edge columns (rows of at most 64 column
// blocks); their pre-compiled signatures are those of rows_supported / rows2_supported.
// *_launchable = the argument block and the launch shape are what the kernel assumes
bool xrows_buildable(const PoolK &pool, const EwOp *pre, int32_t n_pre, const EwOp *post, int32_t n_post, int32_t vec);
bool xrows2_buildable(const PoolRows2K &k, int32_t vec);
std::string xrows_expr(const PoolRowsK &k, int32_t dtype, bool want_idx);
std::string xrows2_expr(const PoolRows2K &k, int32_t dtype, bool want_idx);
bool xrows_launchable(const PoolRowsK &k, int32_t dtype, int64_t grid, int32_t threads);
bool xrows2_launchable(const PoolRows2K &k, int32_t dtype, int64_t grid, int32_t threads);
bs_status launch_xrows(const PoolRowsK &k, int32_t dtype, int64_t grid, int32_t threads, void *stream);
bs_status launch_xrows2(const PoolRows2K &k, int32_t dtype, int64_t grid, int32_t threads, void *stream);
// the chain kernel: is there an instance for this pooling shape, list and depth / launch it
bool xrows_chain_supported(const RowsChainK &k, int32_t dtype);
bool xrows_chain_buildable(const RowsChainK &k, int32_t vec);
bool xrows_chain_launchable(const RowsChainK &k, int32_t dtype, int64_t grid, int32_t threads);
std::string xrows_chain_expr(const RowsChainK &k, int32_t dtype);
bs_status launch_xrows_chain(const RowsChainK &k, int32_t dtype, int64_t grid, int32_t threads, void *stream);
// bs_lds.hip
bool lds_fast_path(const LdsSeqK &k);
bool lds_precompiled(const LdsSeqK &k, int32_t dtype);
bool lds_buildable(const LdsSeqK &k);
std::string lds_expr(const LdsSeqK &k, int32_t dtype, bool want_idx);
bs_status launch_lds(const LdsSeqK &k, int32_t dtype, int64_t grid, int32_t threads, uint64_t lds_bytes, void *stream);
// bs_backward.cpp / bs_backward.hip
void free_backward(bs_stack *s);
bs_status launch_backward_stage(const BwdK &k, int32_t dtype, int32_t vec, int64_t grid, int32_t threads, void *stream);
// bs_trace.cpp
bool trace_enabled();
void trace_push_sequence(const Sequence &q, size_t index, size_t count);
void trace_pop();
// bs_jit.cpp
bool jit_enabled();
std::string jit_last_log();
bool jit_check(const std::string &header, const std::string &expr, const std::string &arch);
bs_status jit_kernel(const std::string &header, const std::string &expr, void **fn);
bs_status jit_launch(void *fn, const void *args, size_t arg_bytes, int64_t grid, int32_t threads, uint64_t lds_bytes,
                     void *stream);

}  // namespace bs
