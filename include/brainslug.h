/*
 * brainslug.h -- C ABI of libbrainslug_hip: depth-first execution of a stack of
 * consecutive non-convolution CNN layers on one AMD MI355X (gfx950).
 *
 * Method: BrainSlug (arXiv 1804.08378).  A "stack" is a run of consecutive
 * optimizable layers (Section 3.2): element-wise layers (inference BatchNorm,
 * ReLU, residual Add) and pooling layers (max, average).  Instead of executing
 * the stack layer by layer through main memory (Figure 2), every tile of the
 * activation is taken through all layers in registers / on-chip memory
 * (Figure 3), so the tensor crosses HBM once in and once out.  The results are
 * those of the layer-by-layer execution (Sections 1, 3, 6).
 *
 * Life cycle (Sections 4.1 "compile phase" and 4.2 "execution phase"):
 *     bs_stack_create   layer list + input shape -> handle (host only)
 *     bs_stack_plan     layers -> operations -> steps -> sequences -> tiles;
 *                       uploads the folded BatchNorm parameters
 *     bs_stack_run      enqueue the sequence kernels on a HIP stream
 *                       (bs_stack_run_strided: on channel slices of larger tensors)
 *     bs_stack_destroy
 *
 * Conventions
 *   - Tensors are dense, NCHW or (a plan option) NHWC, float32, bfloat16 or float16 (bs_dtype).  All tensors of one
 *     stack share the dtype; BatchNorm parameters are always float32.
 *   - "host" / "device" at each pointer says where the memory lives.  The caller
 *     owns every buffer it passes; the library copies what it keeps.
 *   - Enumerations cross the boundary as int32_t (bs_dtype in bs_stack_create, bs_variant and bs_layout in
 *     the option block), sizes as uint64_t and the HIP stream as void *, so that the header needs no HIP
 *     header and has one layout for every compiler.
 *   - Every function returning bs_status returns BS_OK (0) on success and leaves
 *     its outputs untouched on failure.  No function throws or aborts.
 *   - A handle may be used from one thread at a time for create/plan/destroy;
 *     bs_stack_run on a planned handle does not modify it and may be called
 *     concurrently on different streams with different buffers.
 */
#ifndef BRAINSLUG_H
#define BRAINSLUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BS_API __attribute__((visibility("default")))

#define BS_MAX_LAYERS 256      /* layers per stack                                  */
#define BS_MAX_RESIDUALS 16    /* BS_ADD layers per stack                           */
#define BS_MAX_INDEX_OUTPUTS 16 /* max-pool layers with return_indices per stack    */
#define BS_STATIC_WORKSPACE_BYTES (64ull << 20) /* size of the library-owned workspace of bs_stack_run_static */

typedef enum bs_status {
    BS_OK = 0,
    BS_ERR_NULL = 1,        /* a required pointer is NULL                                  */
    BS_ERR_SHAPE = 2,       /* non-positive dimension, or a pooling output dimension < 1   */
    BS_ERR_PARAM = 3,       /* k < 1, s < 1, p > k/2, var + eps <= 0, non-finite parameter */
    BS_ERR_UNSUPPORTED = 4, /* dilation != 1, unknown kind/dtype, too many layers          */
    BS_ERR_NOT_PLANNED = 5, /* run / info before a successful device plan                  */
    BS_ERR_NO_FIT = 6,      /* a step does not fit the on-chip budget at the smallest tile */
    BS_ERR_ALIGN = 7,       /* a device pointer is not 16-byte aligned                     */
    BS_ERR_WORKSPACE = 8,   /* workspace missing or too small                              */
    BS_ERR_HIP = 9,         /* a HIP call failed; see bs_last_hip_error()                  */
    BS_ERR_ALLOC = 10,      /* host allocation failed                                      */
    BS_ERR_RANGE = 11,      /* an index argument is out of range                           */
    BS_ERR_ALIAS = 12,      /* out overlaps an input where that is not allowed             */
    BS_ERR_JIT = 13,        /* a run-time kernel build the caller required has failed      */
    BS_ERR_DEVICE = 14      /* the current HIP device is not the one the stack was planned on */
} bs_status;

/* Storage type of every tensor of a stack; the arithmetic is float32 for all three, each
 * layer output rounded (nearest-even) to the storage type. */
typedef enum bs_dtype { BS_F32 = 0, BS_BF16 = 1, BS_F16 = 2 /* IEEE binary16 */ } bs_dtype;

typedef enum bs_layer_kind {
    BS_BATCHNORM = 1, /* inference BatchNorm: y = (x - mean) / sqrt(var + eps) * gamma + beta  */
    BS_RELU = 2,      /* y = x > 0 ? x : +0   (Section 2: f(x) = max(0, x))                    */
    BS_ADD = 3,       /* y = x + r, r = the next residual tensor passed to bs_stack_run        */
    BS_MAXPOOL = 4,   /* Section 2 pooling, maximum; optional argmax output                    */
    BS_AVGPOOL = 5,   /* Section 2 pooling, average (window sum, then normalisation; Listing 2) */
    BS_LEAKY_RELU = 6, /* y = x > 0 ? x : x * negative_slope                                   */
    BS_CLAMP = 7      /* y = min(max(x, clamp_min), clamp_max): ReLU6, hard tanh               */
} bs_layer_kind;

/*
 * One layer.  Unused fields must be zero.
 *
 * BS_BATCHNORM: gamma, beta, running_mean, running_var are HOST pointers to C
 *   floats each (C = channels of the input shape); copied by bs_stack_create.
 *   The library folds them once, in float64, into scale = gamma / sqrt(var + eps)
 *   and shift = beta - mean * scale, each rounded once to float32, and evaluates
 *   y = fma(x, scale, shift) in float32.
 * BS_LEAKY_RELU / BS_CLAMP: further element-wise activations (Section 2 lists the class as
 *   "BatchNorm, ReLU, ..."); finite parameters, clamp_min <= clamp_max.  A value not above
 *   clamp_min (NaN included) becomes clamp_min.
 * BS_MAXPOOL / BS_AVGPOOL: window kh x kw, stride sh x sw, zero/ignored padding
 *   ph x pw on each side (p <= k/2), output size H_out = (H + 2p - k) / s + 1 rounded
 *   down, or with ceil_mode != 0 rounded up unless the extra window would start at or
 *   beyond H + p (a last window may then overhang the padded input; its cells outside
 *   the input count like padding).
 *   Padding cells are never a maximum candidate and add nothing to an average.
 *   Max: first maximum in row-major window order wins; with return_indices the
 *   layer also yields int32 ih * W + iw of the winner in its own input plane.
 *   Avg: float32 sum over the in-range cells in row-major order, multiplied by the
 *   float32 reciprocal of the number of window cells inside the padded input
 *   (count_include_pad != 0: kh * kw, fewer only for an overhanging ceil-mode window)
 *   or of the number of in-range cells (count_include_pad == 0).
 *   A dilation other than 0 / 1 is rejected (BS_ERR_UNSUPPORTED).
 */
typedef struct bs_layer_desc {
    int32_t kind; /* bs_layer_kind */
    int32_t kh, kw, sh, sw, ph, pw;
    int32_t count_include_pad;
    int32_t return_indices;
    int32_t ceil_mode;
    int32_t dilation_h, dilation_w;
    double eps;
    const float *gamma;        /* host */
    const float *beta;         /* host */
    const float *running_mean; /* host */
    const float *running_var;  /* host */
    float negative_slope;      /* BS_LEAKY_RELU */
    float clamp_min, clamp_max; /* BS_CLAMP */
    float reserved;
} bs_layer_desc;

typedef struct bs_stack bs_stack; /* opaque */

/* Kernel families a sequence can be mapped to (Section 4.1, last paragraph: a
 * single-step sequence streams values from operation to operation; a multi-step
 * sequence keeps a cached buffer and synchronises between steps). */
typedef enum bs_variant {
    BS_VARIANT_AUTO = 0,
    BS_VARIANT_STREAM = 1,      /* element-wise only: 128-bit streaming, registers only         */
    BS_VARIANT_POOL_DIRECT = 2, /* one step, disjoint windows (k == s, p == 0): registers only   */
    BS_VARIANT_LDS_TILE = 3,    /* tiles with halos staged in LDS, ping-pong buffers, barriers   */
    BS_VARIANT_POOL_ROWS = 4,   /* one or two pooling steps with overlapping / padded windows: rows slide in registers, no LDS */
    BS_VARIANT_PLANE_POOL = 5,  /* one step whose window is the whole (small) plane: one lane per plane       */
    BS_VARIANT_NHWC_STREAM = 6, /* channels-last plans only: element-wise, one channel vector per lane   */
    BS_VARIANT_NHWC_POOL = 7,   /* channels-last plans only: one pooling step, a lane = one output pixel x one channel vector */
    BS_VARIANT_NHWC_TILE = 8,   /* channels-last plans only: two pooling steps, tiles of both planes with halos staged in LDS */
    BS_VARIANT_ROWS_CHAIN = 9,  /* two and more identical max-pooling steps that keep the plane's size, each with the same
                                   kinds of element-wise operations behind it: rows ripple through all levels in registers */
    BS_VARIANT_NHWC_ROWS = 10   /* channels-last plans only: two 3 x 3 pooling steps (the first with stride 1, the second a
                                   maximum) on images at most 64 pixels wide: rows slide in registers, a lane = one pixel
                                   column x one channel vector, no LDS */
} bs_variant;

/* Memory order of every tensor of a planned stack (shapes are always given as N, C, H, W). */
typedef enum bs_layout {
    BS_LAYOUT_NCHW = 0, /* N, C, H, W: the width is contiguous                                       */
    BS_LAYOUT_NHWC = 1  /* N, H, W, C: the channels of a pixel are contiguous ("channels last")      */
} bs_layout;

/*
 * Planner options; NULL or all-zero = automatic.
 *   max_lds_bytes           on-chip budget per work-group (Section 4.1 "resource limit")
 *   max_steps_per_sequence  the strategy knob of Section 5.1 (1, 5, 0 = unrestricted)
 *   threads_per_group       64..512, multiple of 64 (0 = 256); the pooling kernels take at most 256, the
 *                           channels-last two-pool kernels have work-groups of their own size
 *   num_cus                 compute units to size grids for (0 = query the current device)
 *   breadth_first           != 0: one sequence per layer, i.e. the layer-by-layer execution
 *                           of Figure 2 with every intermediate in the workspace
 *   force_variant           bs_variant to use wherever it is applicable (tests)
 *   tile_rows, tile_cols, planes_per_group
 *                           final-output tile of LDS sequences (0 = automatic)
 *   host_only               != 0: plan without touching any device; such a plan can be
 *                           inspected but bs_stack_run returns BS_ERR_NOT_PLANNED
 *   jit                     run-time kernel builds (Section 4.1: code is generated for the
 *                           stack and compiled when it is optimised).  A sequence whose
 *                           signature (pooling shapes, element-wise lists) has no instance
 *                           compiled into the library gets one built with hipRTC during
 *                           bs_stack_plan; builds are shared by all stacks of the process.
 *                           0 = automatic: on unless the environment has BS_JIT=0; if a
 *                           build fails the plan falls back to the slower kernels that read
 *                           shapes at run time.  1 = required: a failed build makes
 *                           bs_stack_plan return BS_ERR_JIT.  -1 = off for this plan.
 *   layout                  bs_layout of the input, the residual operands, the output and the
 *                           index outputs.  BS_LAYOUT_NHWC plans run one step (one pooling
 *                           operation with the element-wise operations around it) per
 *                           sequence, or two neighbouring steps in one BS_VARIANT_NHWC_TILE
 *                           sequence when both windows are 3 x 3 (stride 1 or 2) or 2 x 2
 *                           (stride 2), the first pool has no index output and C is a
 *                           multiple of the 128-bit vector (never with
 *                           max_steps_per_sequence = 1 or breadth_first); force_variant must
 *                           be automatic and jit is ignored.  For that variant tile_rows and
 *                           tile_cols are upper bounds of the output tile and
 *                           planes_per_group the channels per work-group; its work-groups
 *                           walk runs of tiles, and the grid reported by bs_stack_sequence_info
 *                           is an upper bound (at most as many groups are launched as the
 *                           device holds at once).  A channel slice of a channels-last tensor
 *                           skips the other channels in every pixel: bs_stack_run_strided
 *                           takes its batch stride, which must be H * W times the larger
 *                           tensor's channel count.  Index outputs hold the same values
 *                           (ih * W + iw) in channels-last order.  With 16-bit storage a pair of
 *                           3 x 3 steps with padding 1 -- the first with stride 1, the second a
 *                           maximum with stride 1 or 2, no index output, images at most 64 pixels
 *                           wide -- runs as one BS_VARIANT_NHWC_ROWS sequence instead (rows in
 *                           registers, no LDS); tile_rows is then the number of output rows per
 *                           work-group.
 *   lane_exchange           sliding-window (BS_VARIANT_POOL_ROWS) sequences on planes whose rows fit one
 *                           wave as 128-bit column blocks (at most 64 of them): 0 = the lanes pass
 *                           their edge columns to their neighbours inside the wave (each input
 *                           element is loaded and computed once); -1 = every lane loads and
 *                           recomputes the columns next to its block itself, as for wider planes.
 *                           Channels-last plans: -1 = no BS_VARIANT_NHWC_ROWS sequences (the pairs
 *                           they would take run as BS_VARIANT_NHWC_TILE).
 */
typedef struct bs_plan_options {
    uint64_t max_lds_bytes;
    int32_t max_steps_per_sequence;
    int32_t threads_per_group;
    int32_t num_cus;
    int32_t breadth_first;
    int32_t force_variant;
    int32_t tile_rows, tile_cols, planes_per_group;
    int32_t host_only;
    int32_t jit;
    int32_t layout;
    int32_t lane_exchange;
    int32_t reserved[2];
} bs_plan_options;

typedef struct bs_plan_info {
    int32_t n_operations; /* layers mapped to basic operations (AvgPool = sum + normalisation) */
    int32_t n_steps;
    int32_t n_sequences;
    int32_t device_planned;     /* 1 when bs_stack_run may be called                       */
    uint64_t workspace_bytes;   /* device bytes bs_stack_run needs between sequences       */
    uint64_t algorithmic_bytes; /* input + residuals + output (+ indices) of the whole stack */
} bs_plan_info;

typedef struct bs_step_info {
    int32_t first_operation, n_operations; /* range in the operation list                  */
    int32_t pool_operation;                /* index of its non-element-wise op, or -1      */
    int32_t sequence;                      /* sequence it was put into                     */
} bs_step_info;

typedef struct bs_sequence_info {
    int32_t first_step, n_steps;
    int32_t first_layer, n_layers;
    int32_t variant;                 /* bs_variant                                         */
    int32_t n_levels;                /* pooling operations inside (LDS hand-offs + 1)      */
    int32_t tile_rows, tile_cols;    /* final-output tile per work-group (LDS variant)     */
    int32_t planes_per_group;
    int32_t halo_rows, halo_cols;    /* input rows/cols an interior tile loads beyond tile*stride */
    int32_t threads_per_group;
    int64_t grid;                    /* work-groups                                        */
    uint64_t lds_bytes;
    int64_t in_shape[4], out_shape[4];
    double redundancy;               /* elements loaded (with halos) / elements of the input */
    int32_t run_time_build;          /* 1: the kernel was (or, host-only, would be) built for this
                                        signature at plan time; 0: compiled into the library   */
    int32_t reserved;
} bs_sequence_info;


/*
 * Create a stack from `n_layers` layer descriptions and the NCHW input shape
 * (Section 4.3: the front-end hands the optimizer a run of optimizable layers
 * with their parameters).  Pure host call; no device is touched.  `layers`,
 * `in_shape` and every parameter array are read during the call only.
 * Errors: BS_ERR_NULL, BS_ERR_SHAPE, BS_ERR_PARAM, BS_ERR_UNSUPPORTED, BS_ERR_ALLOC.
 */
BS_API bs_status bs_stack_create(const bs_layer_desc *layers, int32_t n_layers,
                                 const int64_t in_shape[4], int32_t dtype /* bs_dtype */, bs_stack **out);

/* End of a stack's life (Section 4.2: the plan made in the compile phase serves every later
 * execution of the network; nothing of it outlives the handle): frees the handle, its host
 * copies, its plans and its device parameter table.  NULL is allowed. */
BS_API void bs_stack_destroy(bs_stack *stack);

/* Output size of the stack (Section 4.2: the scheduler calculates the output
 * size; the caller's framework allocates). */
BS_API bs_status bs_stack_output_shape(const bs_stack *stack, int64_t out_shape[4]);
/* Number of BS_ADD layers = residual tensors bs_stack_run expects (-1 if stack is NULL). */
BS_API int32_t bs_stack_num_residuals(const bs_stack *stack);
/* Shape residual tensor `i` must have (that of the i-th BS_ADD layer's input). */
BS_API bs_status bs_stack_residual_shape(const bs_stack *stack, int32_t i, int64_t shape[4]);
/* Number of max-pool layers with return_indices (-1 if stack is NULL). */
BS_API int32_t bs_stack_num_index_outputs(const bs_stack *stack);
/* Shape of index output `i` (the output shape of that max-pool layer), int32 elements. */
BS_API bs_status bs_stack_index_shape(const bs_stack *stack, int32_t i, int64_t shape[4]);
/* Folded BatchNorm parameters of layer `layer` (host float arrays of C elements, either may be
 * NULL): what the kernels multiply and add.  BS_ERR_RANGE if that layer is not a BatchNorm. */
BS_API bs_status bs_stack_folded_bn(const bs_stack *stack, int32_t layer, float *scale, float *shift);

/*
 * Plan the stack (Section 4.1, collapse process): map layers to operations, group
 * operations into steps (any number of element-wise operations and at most one
 * non-element-wise one per step), group steps into sequences that fit the on-chip
 * budget, and choose kernel variant and tile geometry per sequence.  Unless
 * opts->host_only is set it queries the current HIP device for limits that opts
 * leaves at 0 and uploads the folded BatchNorm parameters (library-owned device
 * memory, freed by bs_stack_destroy or a re-plan).  May be called again.
 * Errors: BS_ERR_NULL, BS_ERR_PARAM (bad option), BS_ERR_NO_FIT, BS_ERR_HIP, BS_ERR_ALLOC,
 *         BS_ERR_JIT (opts->jit == 1 only; bs_jit_log() has the compiler output).
 */
BS_API bs_status bs_stack_plan(bs_stack *stack, const bs_plan_options *opts);

/* What the collapse process of Section 4.1 made of the stack: the counts of operations, steps
 * and sequences (Listing 1), each step's operation range (Listing 2 prints exactly this
 * partition), and per sequence the kernel family, tile, halo, on-chip bytes and grid the
 * resource model chose.  Host only.  Errors: BS_ERR_NULL, BS_ERR_NOT_PLANNED, BS_ERR_RANGE. */
BS_API bs_status bs_stack_plan_info(const bs_stack *stack, bs_plan_info *info);
BS_API bs_status bs_stack_step_info(const bs_stack *stack, int32_t step, bs_step_info *info);
BS_API bs_status bs_stack_sequence_info(const bs_stack *stack, int32_t sequence, bs_sequence_info *info);
/* Static name of operation `op` of the plan ("BatchNorm", "ReLU", "Add", "MaxPooling",
 * "AvgPooling", "AvgNormalization"), or NULL when out of range / not planned. */
BS_API const char *bs_stack_operation_name(const bs_stack *stack, int32_t op);
/* Device bytes bs_stack_run needs as workspace: sequences run one after the other (Section 4.2)
 * and hand the tensor between them through main memory, alternating between two halves of the
 * workspace; 0 when the stack is one sequence.  The caller's framework allocates it, like the
 * output (Section 4.2). */
BS_API uint64_t bs_stack_workspace_bytes(const bs_stack *stack);

/*
 * Enqueue the stack on `stream` (a hipStream_t passed as void*; NULL = the null
 * stream) of the device the plan was made on.  Never synchronises, never
 * allocates, returns as soon as the kernels are queued; sequences of one stack
 * run one after the other (Section 4.2).
 *   in         device, dense NCHW of the create-time shape and dtype
 *   residuals  host array of bs_stack_num_residuals() DEVICE pointers, in layer
 *              order (may be NULL when there are none)
 *   out        device, bs_stack_output_shape() elements of the stack dtype.
 *              Must not overlap any input, except that a stack without pooling
 *              layers may run in place (out == in)
 *   indices    host array of bs_stack_num_index_outputs() DEVICE int32 pointers;
 *              the array or single entries may be NULL to skip those outputs
 *   workspace  device, >= bs_stack_workspace_bytes() (NULL allowed when that is 0)
 * All device pointers must be 16-byte aligned.
 * The device that was current in bs_stack_plan (it holds the parameter table and the kernels
 * built for the stack) must be current again.
 * Errors: BS_ERR_NULL, BS_ERR_NOT_PLANNED, BS_ERR_DEVICE, BS_ERR_ALIGN, BS_ERR_WORKSPACE,
 *         BS_ERR_ALIAS, BS_ERR_HIP (launch failure; raw code in bs_last_hip_error()).
 */
BS_API bs_status bs_stack_run(const bs_stack *stack, const void *in, const void *const *residuals,
                              void *out, int32_t *const *indices, void *workspace,
                              uint64_t workspace_bytes, void *stream);

/*
 * bs_stack_run for callers that cannot allocate device memory and therefore have no workspace
 * to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The intermediate tensors between sequences go to a library-owned array of
 * BS_STATIC_WORKSPACE_BYTES (64 MiB) that is part of the library's device code: every GPU the
 * library runs on holds one copy from the moment the code is loaded there until the process
 * ends.  bs_stack_plan looks up the array's address on its device; this call allocates and frees
 * nothing (no hipMalloc / hipFree, no allocating library routine), never synchronises, and only
 * enqueues the sequence kernels, exactly those of bs_stack_run.
 *   in, residuals, out, indices, stream   as in bs_stack_run (caller-owned, dense)
 * A stack whose bs_stack_workspace_bytes() exceeds BS_STATIC_WORKSPACE_BYTES is refused with
 * BS_ERR_WORKSPACE (nothing is enqueued); a stack that is one sequence uses no workspace at all.
 * All calls on one GPU share that GPU's array.  It keeps the last call's contents; nothing in
 * it has to start at zero, because every sequence writes its whole output before the next one
 * reads it.  Two calls that need the workspace and overlap in time on one GPU (different
 * streams, or a graph replay beside an eager call) race on it: the caller must order them.
 * Errors: those of bs_stack_run.
 */
BS_API bs_status bs_stack_run_static(const bs_stack *stack, const void *in, const void *const *residuals,
                                     void *out, int32_t *const *indices, void *stream);
/* BS_STATIC_WORKSPACE_BYTES of the loaded library. */
BS_API uint64_t bs_static_workspace_capacity(void);

/*
 * bs_stack_run for an input and / or an output that is a channel slice of a larger NCHW
 * tensor, read and written in place: what a DenseNet-style concatenation buffer needs
 * (Section 5, DenseNet-121: every dense layer's BatchNorm -> ReLU reads the first channels
 * of the block's buffer; the stem's pooling writes into it), so that the stack still moves
 * the tensor through main memory once (Section 3) with no gather / scatter copy around it.
 *   in, out            device pointers to the first element of the slice (image 0, channel 0
 *                      of the stack's own C channels)
 *   in_batch_stride    elements between the starts of consecutive images of the input:
 *   out_batch_stride   0 = dense (C*H*W of that tensor), else >= C*H*W; the stride times the
 *                      element size must be a multiple of 16 bytes (BS_ERR_ALIGN)
 * Channels, rows and columns of a slice stay dense (a slice along the channel axis).  For a
 * channels-last plan the slice lies inside every pixel of the larger tensor instead: the batch
 * stride must be H * W * (channels of the larger tensor), that channel count times the element
 * size a multiple of 16 bytes, and N * stride at most 2^31 - 1 (BS_ERR_SHAPE / BS_ERR_ALIGN).
 * Residual operands, index outputs and the workspace are dense, as in bs_stack_run.
 * `out` must not overlap an input; two slices of one buffer with the same batch stride count
 * as disjoint when their per-image byte ranges are.  In place (out == in, equal strides) is
 * allowed for a stack without pooling layers.
 * Errors: those of bs_stack_run; BS_ERR_SHAPE for a stride below C*H*W or above 2^31 - 1.
 */
BS_API bs_status bs_stack_run_strided(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                      const void *const *residuals, void *out,
                                      int64_t out_batch_stride, int32_t *const *indices,
                                      void *workspace, uint64_t workspace_bytes, void *stream);

/*
 * The argument checks of bs_stack_run_strided alone: nothing is enqueued, no device is touched
 * and no pointer is dereferenced (addresses are only compared), so it also works on a
 * host-only plan.  Returns what bs_stack_run_strided would return for these arguments before
 * its first launch, device checks (BS_ERR_DEVICE) aside.
 */
BS_API bs_status bs_stack_check_buffers(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                        const void *const *residuals, const void *out,
                                        int64_t out_batch_stride, int32_t *const *indices,
                                        const void *workspace, uint64_t workspace_bytes);

/*
 * Backward pass (Section 7 names training as the method's next step; Sections 2 and 3 fix the
 * forward pass whose Jacobian this applies): plan it, once, after bs_stack_plan on the same
 * device.  The stack is cut into stages (element-wise operations, then at most one pooling
 * operation); stages whose output or max-pooling picks the backward pass needs get forward
 * plans of their own (library-owned, freed by bs_stack_destroy or the next bs_stack_plan).
 * For the plan's memory layout (row-major or channels-last; all tensors of bs_stack_backward are
 * then in that layout, dense).  BatchNorm is the inference-mode layer (constant folded
 * parameters): gradients are produced for the stack's input and its residual operands, none
 * for BatchNorm parameters.
 * After a host-only plan it builds the stages, their (host-only) forward plans and the workspace size, which
 * bs_stack_backward_num_stages / _workspace_bytes report; bs_stack_backward then returns BS_ERR_NOT_PLANNED.
 * Errors: BS_ERR_NULL, BS_ERR_NOT_PLANNED (no plan), BS_ERR_UNSUPPORTED (a tensor of 2^31
 *         lanes), BS_ERR_DEVICE, BS_ERR_ALLOC, and those of bs_stack_plan for the stage plans.
 */
BS_API bs_status bs_stack_plan_backward(bs_stack *stack);
/* Device bytes bs_stack_backward needs as workspace (0: none, or no backward plan). */
BS_API uint64_t bs_stack_backward_workspace_bytes(const bs_stack *stack);
/* Stages of the backward plan (-1 without one). */
BS_API int32_t bs_stack_backward_num_stages(const bs_stack *stack);

/*
 * Enqueue the backward pass on `stream`: given the stack's input and residual operands of the
 * forward pass and the gradient of a scalar with respect to the stack's output, compute its
 * gradients with respect to the input and the residual operands -- grad_out times the
 * Jacobian of the layer-by-layer forward pass, storage rounding taken as the identity.  The
 * forward pass is not needed beforehand and nothing of it is kept: intermediate values and
 * max-pooling picks are recomputed from `in` (first maximum in row-major window order, as in
 * bs_stack_run).  ReLU passes the gradient where its input is > 0, clamp where
 * lo <= input <= hi; average pooling uses the forward pass's divisor per window; overlapping
 * windows add up.  Arithmetic is float32, each result rounded once to the stack dtype.
 *   in, residuals    device, as in bs_stack_run (dense, the forward pass's values)
 *   indices          host array of bs_stack_num_index_outputs() DEVICE int32 pointers: index outputs
 *                    that bs_stack_run wrote for this `in` (the saved picks of max-pooling layers
 *                    created with return_indices); the array or single entries may be NULL.  Where
 *                    given for the stack's last pooling layer, the forward run that would recompute
 *                    them is skipped; they are trusted (a cell index outside its window or plane
 *                    only misroutes that gradient, it is never used as an address)
 *   grad_out         device, dense, bs_stack_output_shape() elements of the stack dtype
 *   grad_in          device, dense, the input's shape and dtype; NULL = not wanted
 *   grad_residuals   host array of bs_stack_num_residuals() DEVICE pointers (shapes of the
 *                    residual operands); the array or single entries may be NULL = not wanted
 *   workspace        device, >= bs_stack_backward_workspace_bytes() (NULL allowed when 0)
 * All device pointers 16-byte aligned; no output may overlap an input, the workspace or
 * another output.  Never synchronises, never allocates.  The device of the plan must be current.
 * Errors: BS_ERR_NULL, BS_ERR_NOT_PLANNED (no backward plan), BS_ERR_DEVICE, BS_ERR_ALIGN,
 *         BS_ERR_WORKSPACE, BS_ERR_ALIAS, BS_ERR_HIP.
 */
BS_API bs_status bs_stack_backward(const bs_stack *stack, const void *in, const void *const *residuals,
                                   const int32_t *const *indices, const void *grad_out, void *grad_in,
                                   void *const *grad_residuals, void *workspace, uint64_t workspace_bytes,
                                   void *stream);

/*
 * bs_stack_backward for operands that are channel slices of larger tensors (Section 5, DenseNet-121:
 * the dense layers' BatchNorm -> ReLU read a prefix of the block's concatenation buffer, and the
 * gradients of the buffer's channel ranges are slices of one gradient buffer): `in`, `grad_out`
 * and `grad_in` are read and written in place, with batch strides as in bs_stack_run_strided
 * (0 = dense; row-major: elements between consecutive images; channels-last: H * W times the
 * larger tensor's channel count).  Residual operands, their gradients, saved indices and the
 * workspace are dense.  No output may overlap an input, the workspace or another output; two
 * slices of one buffer with the same batch stride count as disjoint when their per-image byte
 * ranges are.  A stage without pooling on planes that are no whole number of 128-bit vectors
 * takes slices only when C * H * W is one (BS_ERR_UNSUPPORTED otherwise).
 * Errors: those of bs_stack_backward; BS_ERR_SHAPE / BS_ERR_ALIGN for the strides as in
 *         bs_stack_run_strided.
 */
BS_API bs_status bs_stack_backward_strided(const bs_stack *stack, const void *in, int64_t in_batch_stride,
                                           const void *const *residuals, const int32_t *const *indices,
                                           const void *grad_out, int64_t grad_out_batch_stride, void *grad_in,
                                           int64_t grad_in_batch_stride, void *const *grad_residuals, void *workspace,
                                           uint64_t workspace_bytes, void *stream);

/*
 * Compile, without loading them and without touching any device, all run-time builds the
 * current plan (device or host-only) asks for, for GPU architecture `arch` ("gfx950"; NULL =
 * "gfx950").  A way to check on a machine without a GPU that a stack's kernels build.
 * `n_built`, if not NULL, receives the number of kernels compiled.
 * Errors: BS_ERR_NULL, BS_ERR_NOT_PLANNED (no plan at all), BS_ERR_JIT (see bs_jit_log()).
 */
BS_API bs_status bs_stack_jit_check(const bs_stack *stack, const char *arch, int32_t *n_built);
/* Compiler output of the calling process's last failed run-time build ("" if none); the
 * pointer stays valid until the calling thread's next call of this function. */
BS_API const char *bs_jit_log(void);

/*
 * Measurement aid (the resource model of Section 4.1 and the utilisation trade-offs of Section 4.4
 * need the device's issue rates, which no query reports): enqueue a kernel in which every wave
 * issues 8 * `iterations` instruction groups of one kind and nothing else, on
 * `waves_per_simd` (1..8) waves per SIMD of every compute unit.  The caller times the launch;
 * cycles per group per SIMD = time * clock / (8 * iterations * waves_per_simd).
 *   kind         bs_probe_kind
 *   sink         device, >= compute units * waves_per_simd * 256 floats (one store per lane)
 * Errors: BS_ERR_NULL, BS_ERR_PARAM, BS_ERR_RANGE (kind), BS_ERR_WORKSPACE (sink too small), BS_ERR_HIP.
 */
typedef enum bs_probe_kind {
    BS_PROBE_ADD = 0,           /* v_add_f32 (two-operand encoding)                          */
    BS_PROBE_FMA = 1,           /* v_fma_f32 (three-operand encoding)                        */
    BS_PROBE_MAX3 = 2,          /* v_max3_f32                                                */
    BS_PROBE_SELECT_VCC = 3,    /* v_cndmask_b32 reading its lane mask from VCC              */
    BS_PROBE_SELECT_SGPR = 4,   /* v_cndmask_b32 reading its lane mask from a scalar pair    */
    BS_PROBE_LANE_SHIFT = 5,    /* v_mov_b32 with a one-lane wave shift (DPP)                */
    BS_PROBE_ADD_SCALAR = 6,    /* group = v_add_f32 + one scalar ALU instruction            */
    BS_PROBE_ADD_BRANCH = 7,    /* group = v_add_f32 + one not-taken scalar branch           */
    BS_PROBE_DEPENDENT_ADD = 8  /* v_add_f32 on one register: every add waits for the last   */
} bs_probe_kind;
BS_API bs_status bs_probe_issue_rate(int32_t kind, int32_t waves_per_simd, int32_t iterations, float *sink,
                                     uint64_t sink_floats, void *stream);

/*
 * Measurement aid (the roofline the streaming kernels are priced against): enqueue a kernel with no
 * arithmetic in which every lane reads `reads_per_write` (1, 2 or 4) 128-bit vectors from `in` --
 * that many streams, each contiguous across the lanes, non-temporal loads as in the streaming
 * kernels -- and writes one vector to `out`: 4 = the four-bytes-in-per-byte-out pattern of a 2 x 2
 * pooling step, 1 = a copy.  read_only != 0: the same loads, nothing written (out is still needed
 * and must hold out_bytes).  The caller times the launch; bytes moved = out_bytes * reads_per_write
 * (+ out_bytes unless read_only).
 *   in, out      device, 16-byte aligned, not overlapping; in_bytes >= out_bytes * reads_per_write
 *   out_bytes    a multiple of 16, at most 2^31 - 1 vectors
 * Errors: BS_ERR_NULL, BS_ERR_PARAM, BS_ERR_WORKSPACE (in too small), BS_ERR_ALIGN, BS_ERR_HIP.
 */
BS_API bs_status bs_probe_stream(int32_t reads_per_write, int32_t read_only, const void *in, uint64_t in_bytes, void *out,
                                 uint64_t out_bytes, void *stream);

/* Static, never NULL. */
BS_API const char *bs_status_string(bs_status status);
BS_API const char *bs_version(void);
/* Raw hipError_t of the calling thread's last failed HIP call inside the library (0 if none). */
BS_API int32_t bs_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BRAINSLUG_H */
