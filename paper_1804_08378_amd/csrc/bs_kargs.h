// Kernel argument blocks and the few constants and helpers that host code and device code
// share.  Plain data only and no standard-library headers: this file is also compiled at run
// time (hipRTC) when a stack signature gets its own kernel build.
#pragma once

#if defined(__HIPCC_RTC__)
typedef signed int int32_t;
typedef unsigned int uint32_t;
typedef unsigned short uint16_t;
typedef long long int64_t;
typedef unsigned long long uint64_t;
#else
#include <cstdint>
#endif

namespace bs {

// ---------------------------------------------------------------------------
// Basic operations a layer maps to (Section 4.1 "collapse process": layers are
// mapped onto element-wise and non-element-wise operations; Listing 2 shows
// average pooling as AvgPooling + AvgNormalization).
// ---------------------------------------------------------------------------
enum OpKind : int32_t {
    OP_BN = 1,
    OP_RELU = 2,
    OP_ADD = 3,
    OP_MAXPOOL = 4,
    OP_AVGSUM = 5,   // non-element-wise: window sum
    OP_AVGNORM = 6,  // element-wise: multiply by 1/divisor
    OP_LEAKY = 7,    // element-wise: x > 0 ? x : x * slope
    OP_CLAMP = 8,    // element-wise: min(max(x, lo), hi)
};

// Element-wise lists are packed into template arguments one base-K_EW_BASE digit per operation
// (the operation kind; first operation in the lowest digit, 0 = end).
constexpr int K_EW_BASE = 16;
// number of operations in such a code, and the kind of its q-th operation
constexpr int ew_code_len(int code)
{
    int n = 0;
    while (code > 0) {
        ++n;
        code /= K_EW_BASE;
    }
    return n;
}
constexpr int ew_code_kind(int code, int q)
{
    for (int i = 0; i < q; ++i) code /= K_EW_BASE;
    return code % K_EW_BASE;
}

inline bool op_is_elementwise(int32_t k) { return k != OP_MAXPOOL && k != OP_AVGSUM; }

// ---------------------------------------------------------------------------
// Kernel argument blocks (plain data, passed by value at launch).
// ---------------------------------------------------------------------------
constexpr int K_MAX_LEVELS = 8;   // pooling operations in one LDS sequence
constexpr int K_MAX_EW = 6;       // element-wise operations attached to one level
constexpr int K_MAX_STREAM_EW = 16;
constexpr int K_MAX_RES = 4;      // residual tensors one sequence can read
constexpr int K_MAX_IDX = 4;      // index tensors one sequence can write
constexpr int K_STREAM_U = 2;     // 128-bit vectors per lane in stream_kernel (measured on MI355X: 1 is 3..9 points of HBM peak slower, 4 is 1..3 slower with 16-bit storage)
#if !defined(BS_ROWS_OR)
#define BS_ROWS_OR 2
#endif
// Measured on MI355X (ResNet stem, float32 / bfloat16 / with indices float32, us): 2 rows 46.1 / 27.5 / 64.8, 3 rows 46.5 / 29.2 / 64.7,
// 4 rows 46.8 / 29.2 / 62.6.
constexpr int K_ROWS_OR = BS_ROWS_OR;     // output rows per lane per iteration of the one-level sliding-window kernels (all their input rows are requested at once)
constexpr int K_ROWS2_RC = 4;    // output rows per lane in pool_rows2_kernel
// Elements per lane and row (the lane's column block) of the sliding-window kernels for 16-bit
// storage: one 128-bit load, as for float32 (4).  Measured on MI355X, 64-bit blocks (twice the
// lanes) are 15..30 % slower for the one-level kernel.
constexpr int K_ROWS_VEC16 = 8;
constexpr int K_ROWS2_VEC16 = 8;
constexpr int K_ROWS2_VEC32 = 4;  // float32 in the two-level kernel (8, two loads per row, measured 5 % slower: registers)
// Column block of the sliding-window kernels whose lanes exchange edge columns (whole 128-bit vectors).
constexpr int K_XROWS_VEC32 = 4, K_XROWS_VEC16 = 8;    // one pooling operation
constexpr int K_XROWS2_VEC32 = 4, K_XROWS2_VEC16 = 8;  // two pooling operations (float32 with 8: measured 4 .. 9 % slower)
// Output rows per lane in pool_xrows2_kernel.  Longer chunks recompute less, but the kernel is bound by
// instruction issue and wants many waves: measured best on 56 x 56 planes.
constexpr int K_XROWS2_RC32 = 2, K_XROWS2_RC16 = 4;
// Channel vectors (waves) per work-group of nhwc_rows2_kernel and output rows per chunk.  Measured on MI355X (halo_stress
// channels-last, 28 output rows, bfloat16 / binary16, us) -- 8 waves (the 128 bytes of one cache line): 4 rows 74 / 59,
// 7 rows 68 / 56, 14 rows 64 / 55; 4 waves: 60 / 56, 57 / 55, 64 / 55; 2 waves: 87 / 88, 80 / 81, 82 / 78.  With eight waves and the
// bfloat16 instance's 168 registers (three waves per SIMD) only one work-group fits a compute unit.
#if !defined(BS_NHWC_ROWS_WAVES)
#define BS_NHWC_ROWS_WAVES 4
#endif
constexpr int K_NHWC_ROWS_WAVES = BS_NHWC_ROWS_WAVES;
constexpr int K_NHWC_ROWS_RC = 7;
constexpr int K_LDS_RB = 2;       // consecutive rows one lane pools per strip in the specialised LDS kernels
constexpr int K_DIRECT_U = 1;     // units per lane in pool_direct_kernel (2 measured 1..2 % slower on the VGG stacks)
constexpr int K_PLANE_WALK_CELLS = 16;  // whole-plane pooling: planes up to this many cells are walked in global
                                        // memory by one lane each, larger ones are staged through LDS

// n / d for 0 <= n < 2^31 by multiply-high and shift.
struct FastDiv {
    uint32_t mul = 0, shift = 0, d = 1;
};

struct EwOp {
    int32_t kind;  // OP_BN, OP_RELU, OP_ADD, OP_LEAKY, OP_CLAMP
    int32_t arg;   // BN: offset of scale[] in the parameter table (shift[] follows); leaky ReLU / clamp:
                   // offset of [slope] / [lo, hi] there; Add: residual slot of the sequence
};

struct PoolK {
    int32_t kind;  // OP_MAXPOOL or OP_AVGSUM (normalisation included)
    int32_t kh, kw, sh, sw, ph, pw;
    int32_t count_include_pad;
    int32_t idx_slot;  // slot in LdsSeqK::idx, or -1
    float inv_kk;      // 1.0f / (kh * kw)
};

// One level of an LDS sequence.  The region a work-group keeps of level l is a fixed-size
// rectangle rows x cols whose origin (which may lie outside the plane: padding) follows
// from the tile by origin[l-1] = origin[l] * stride - pad.
struct LevelK {
    int32_t H, W;            // plane size at this level
    int32_t rows, cols;      // region extent; cols is a multiple of 4 for levels >= 1
    int32_t pitch;           // LDS row pitch in floats (multiple of 4)
    int32_t plane_stride;    // rows * pitch
    int32_t buf_off;         // float offset of this level's buffer in dynamic LDS
    int32_t n_ew;
    EwOp ew[K_MAX_EW];       // applied to a value once it exists at this level
    int32_t vo;              // outputs one lane produces per strip at this level (levels >= 1)
    int32_t items_per_row;   // level 0: global vectors per region row; else strips of vo outputs
    int32_t ct, rt;          // lane grid of a phase: ct = min(items_per_row, threads) lanes along a
                             // row, rt = threads / ct rows in flight
    FastDiv div_ct;          // by ct
};

struct LdsSeqK {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    const void *res[K_MAX_RES];
    int32_t *idx[K_MAX_IDX];
    int32_t n_levels;  // L >= 1 pooling operations; levels 0..L
    int32_t NC, C;
    int32_t TH, TW, tiles_h, tiles_w, PPG;
    int32_t vec;       // elements per 128-bit access used for the level-0 load (1 = scalar)
    int32_t delta0;    // level-0 LDS column of the region's first column: the LDS row starts at the
                       // 128-bit global vector that contains it (0 when vec == 1)
    FastDiv div_tiles_w, div_tiles_hw, div_c;
    LevelK level[K_MAX_LEVELS + 1];
    PoolK pool[K_MAX_LEVELS + 1];  // pool[l] produces level l from level l-1 (l >= 1)
};

struct StreamK {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    const void *res[K_MAX_RES];
    int32_t n_ew;
    EwOp ew[K_MAX_STREAM_EW];
    uint32_t total;     // vectors (or elements when vec == 1)
    int32_t C;
    FastDiv div_plane;  // by H*W/vec (flat: by H*W)
    FastDiv div_c;
    int32_t flat;       // 1: H*W is no multiple of vec; vectors run over the whole tensor and may straddle two planes
};

struct PoolDirectK {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    const void *res[K_MAX_RES];
    int32_t *idx;
    int32_t n_pre, n_post;
    EwOp pre[K_MAX_EW], post[K_MAX_EW];
    PoolK pool;
    int32_t C, H, W, Ho, Wo;
    uint32_t total;      // units = planes * Ho * (W / vec); planes for the whole-plane kernels
    FastDiv div_wv;      // by W / vec (whole-plane kernel staged through LDS: by H * W)
    FastDiv div_ho;      // by Ho
    FastDiv div_c;
    int32_t ppg, pitch;  // whole-plane kernel staged through LDS: planes per work-group, LDS floats per plane (odd)
};

struct PoolRowsK {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    int32_t *idx;
    int32_t n_pre, n_post;
    EwOp pre[K_MAX_EW], post[K_MAX_EW];
    PoolK pool;
    int32_t C, H, W, Ho, Wo;
    int32_t rc;       // output rows one lane walks down
    int32_t chunks;   // chunks per plane = ceil(Ho / rc)
    int32_t cbs;      // 128-bit column blocks per input row = W / vec
    uint32_t total;   // lanes with work = planes * chunks * cbs
    FastDiv div_cbs, div_chunks, div_c;
    // lane-exchange kernel only (spw == 0: the kernel that loads its edge columns)
    int32_t spw;      // (plane, chunk) segments of cbs lanes per wave = 64 / cbs
    uint32_t units;   // segments = planes * chunks
};

// Two pooling operations in one register sliding-window kernel: pre, pool1, mid, pool2, post.
struct PoolRows2K {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    int32_t *idx;     // index output of pool2 (pool1 never has one here)
    int32_t n_pre, n_mid, n_post;
    EwOp pre[K_MAX_EW], mid[K_MAX_EW], post[K_MAX_EW];
    PoolK pool1, pool2;
    int32_t C, H, W, H1, W1, Ho, Wo;  // input plane, plane between the pools, output plane
    int32_t rc;       // output rows one lane walks down
    int32_t chunks;   // chunks per plane = ceil(Ho / rc)
    int32_t cbs;      // 128-bit column blocks per input row = W / vec
    uint32_t total;   // lanes with work = planes * chunks * cbs
    FastDiv div_cbs, div_chunks, div_c;
    // lane-exchange kernel only (spw == 0: the kernel that loads its edge columns)
    int32_t spw;      // (plane, chunk) segments of cbs lanes per wave = 64 / cbs
    uint32_t units;   // segments = planes * chunks
};

// A chain of identical pooling steps that keep the plane's size (window k, stride 1, padding (k - 1) / 2), each followed
// by the same kinds of element-wise operations: the stacked blocks of Section 5.1 in the register kernel whose lanes
// exchange edge columns.  A lane walks down a chunk of rc output rows and the n_levels * (kh - 1) / 2 rows above and below it.
constexpr int K_CHAIN_MAX = 8;
struct RowsChainK {
    const void *in;
    void *out;
    const float *params;
    uint32_t in_extra, out_extra;  // elements to skip per image beyond a dense one: batch stride - C*H*W (0 = dense)
    int32_t n_levels;              // pooling steps, 1 .. K_CHAIN_MAX
    int32_t n_ew;                  // element-wise operations behind each of them
    EwOp ew[K_CHAIN_MAX][K_MAX_EW];
    PoolK pool;
    int32_t C, H, W;
    int32_t rc, chunks, cbs, spw;  // as in PoolRows2K
    uint32_t units;
    FastDiv div_cbs, div_chunks, div_c;
};

// Channels-last (N, H, W, C in memory) sequences: element-wise only (pool.kind == 0, the list
// in `pre`) or one pooling operation with element-wise operations before and after it.
struct NhwcK {
    const void *in;
    void *out;
    const float *params;
    const void *res[K_MAX_RES];
    int32_t *idx;
    int32_t n_pre, n_post;
    EwOp pre[K_MAX_STREAM_EW], post[K_MAX_EW];
    PoolK pool;
    int32_t C, H, W, Ho, Wo;
    uint32_t total;   // lanes with work: (output) pixels * channel vectors
    FastDiv div_cv;   // by channel vectors per pixel = C / vec
    FastDiv div_wo, div_ho;
    uint32_t in_xp, out_xp;  // elements to skip per pixel beyond the sequence's own C channels: the tensor is a
                             // channel slice of one with C + in_xp (C + out_xp) channels (0 = dense)
    int32_t cv_group; // whole-plane pooling staged through LDS: channel vectors per work-group (0: not that kernel);
                      // div_wo then divides by the work-groups per image
};

// Channels-last sequence of two pooling steps in one kernel (bs_nhwc_tile.hip): a tile is TH x TW
// output pixels of one image and `cvb` consecutive channel vectors; a work-group keeps the rectangles
// of the input plane (r0h x r0w cells) and of the plane between the pools (r1h x r1w) under a tile in
// LDS and walks a run of consecutive tiles.
constexpr int K_TILE_MAX_BN = 3 * K_MAX_EW;
struct NhwcTile2K {
    const void *in;
    void *out;
    const float *params;
    const void *res[K_MAX_RES];
    int32_t *idx;                // picks of the second pool (a max pool), or null
    int32_t n_pre, n_mid, n_post;
    EwOp pre[K_MAX_EW], mid[K_MAX_EW], post[K_MAX_EW];
    PoolK pool1, pool2;
    int32_t C, H, W, H1, W1, Ho, Wo;
    int32_t TH, TW, r0h, r0w, r1h, r1w;
    int32_t cvb, pl;             // channel vectors per work-group; pixel lanes = threads / cvb
    int32_t cvgs, tiles_h, tiles_w;  // channel-vector groups (C / vec / cvb), tiles per image
    uint32_t total_tiles;        // cvgs * N * tiles_h * tiles_w, numbered in that order
    uint32_t lds1_off, par_off;  // first LDS vector of the second rectangle, of the staged BatchNorm parameters
    int32_t n_bn;                // BatchNorm operations of the three lists, in order
    int32_t bn_base[3];          // how many of them precede the lists pre, mid, post
    int32_t bn_arg[K_TILE_MAX_BN];   // where their scale[] starts in the parameter table (shift[] follows)
    FastDiv div_cvb, div_r0w, div_n, div_tiles_w, div_tiles_h;
    FastDiv div_bw1, div_bw2;    // by the blocks per rectangle row of the two pooling levels
    uint32_t in_xp, out_xp;      // as in NhwcK
    // nhwc_rows2_kernel (no tiles: a work-group is cvb channel vectors of a chunk of rc output rows of one image;
    // work-groups numbered (image * chunks + chunk) * cvgs + group)
    int32_t rc, chunks;
    FastDiv div_cvgs, div_chunks;
};

// Backward pass of one stage: element-wise operations followed by at most one pooling
// operation (pool.kind == 0: none).  Dense tensors only, row-major (NCHW) or channels-last.
constexpr int K_BWD_EW = 16;
#if !defined(BS_MAXROWS_RC)
#define BS_MAXROWS_RC 8
#endif
// Window rows per chunk of the backward kernel that finds max-pooling picks itself.  Measured on MI355X (ResNet stem, 56 window
// rows, float32 / bfloat16): 8 -> 94 / 73 us, 14 -> 99 / 73, 28 -> 95 / 76, 56 -> 101 / 107.
constexpr int K_BWD_MAXROWS_RC = BS_MAXROWS_RC;
#if !defined(BS_ROWS2_RC)
#define BS_ROWS2_RC 28
#endif
// ... of the kernel that walks two pooling levels at once (a chunk revisits two window rows).  Measured on MI355X, 56 x 56 planes
// (28 window rows), float32: 7 -> 145 us, 14 -> 134 us, 28 -> 130 us; with the BatchNorm parameters read once per lane: 132, 122, 116 us.
constexpr int K_BWD_ROWS2_RC = BS_ROWS2_RC;
struct BwdK {
    const void *a;        // the stage's input of the forward pass
    const void *g_out;    // gradient with respect to the stage's output
    void *g_in;           // gradient with respect to the stage's input (null: not wanted)
    const int32_t *idx;   // max pooling: the forward pass's picks (cell index inside the input plane)
    const float *params;
    const void *res[K_MAX_RES];   // residual operands of the stage's Add operations, in order
    void *g_res[K_MAX_RES];       // their gradients (null: not wanted)
    int32_t n_ew;
    EwOp ew[K_BWD_EW];    // Add: arg is unused, the n-th Add of the list uses res[n]
    PoolK pool;
    int32_t C, H, W, Ho, Wo;
    uint32_t total;       // lanes with work = planes * H * (W / vec); direct: planes * Ho * (W / vec)
    FastDiv div_wv;       // by W / vec
    FastDiv div_h, div_c; // by H (direct: by Ho), by C
    int32_t direct;       // 1: disjoint 2 x 2 windows that tile the plane; a lane owns whole windows and
                          // finds the max-pooling picks itself (idx unused)
    int32_t nhwc;         // 1: channels-last tensors.  A lane owns `vec` consecutive channels of one pixel (direct:
                          // of one window's four pixels); total = pixels (direct: windows) * (C / vec), div_wv
                          // divides by C / vec, div_h by H (direct: Ho), div_w by W (direct: Wo)
    FastDiv div_w;
    int32_t flat;         // 1 (row-major, no pooling): planes are no whole number of vectors; the tensor is one run of
                          // `vec`-element vectors that may begin in one plane and end in the next; total = vectors,
                          // div_w divides by H * W
    // wave_rows = 1 (row-major, pooling 3 x 3 with padding 1 and stride 1 or 2, rows of at most 64 vectors): a lane
    // owns one column block and walks down a chunk of rows with the rows of the current windows in registers; max
    // pooling: it finds every window's pick itself (idx unused); gradients that belong to its neighbours' columns
    // travel inside the wave.  A wave holds spw = 64 / cbs (plane, chunk) segments of cbs lanes; a chunk is rc window rows.
    // The stage input, the gradient with respect to it and the upstream gradient may be channel slices of larger
    // tensors (first stage / last stage of bs_stack_backward_strided).  Row-major: elements every image starts later
    // than in a dense tensor, for each image before it; channels-last: elements to skip per pixel beyond the C channels.
    uint32_t a_extra, gin_extra, gout_extra;
    // audit builds (-DBS_BWD_AUDIT): elements reachable from a / g_out / g_in, and where offsets beyond them are counted
    uint32_t audit_lim[3];
    uint32_t *audit;
    int32_t wave_rows;    // 2: two stages in one kernel -- `pool` (average 3 x 3 / 1 / 1) behind ew[0 .. n_ew), then `pool2` (max
                          // 3 x 3 / 2 / 1) with ew[n_ew .. n_ew + n_post) behind it; H x W: the input plane, Ho x Wo: the max pooling's output
    PoolK pool2;
    int32_t n_post;       // wave_rows, max pooling: element-wise operations (no Add) that follow the pooling, ew[n_ew .. n_ew + n_post):
                          // g_out is the gradient with respect to their output
    int32_t cbs, spw, chunks, rc;
    uint32_t units;       // planes * chunks
    FastDiv div_cbs, div_chunks;
};

#if defined(__HIPCC__)
#define BS_HD __host__ __device__ inline
#else
#define BS_HD inline
#endif

// Outputs one lane produces per strip of a pooling phase, by column stride.  Two per lane for
// stride 2 would make consecutive lanes read LDS four floats apart (no bank conflicts), but it
// doubles the per-output address and predicate work; measured on MI355X four per lane is faster
// for every benchmark stack, so the rule is constant.  Planner, audit and kernels all use it.
#if defined(__HIPCC__)
__host__ __device__
#endif
constexpr int32_t strip_outputs(int32_t /*sw*/)
{
    return 4;
}

BS_HD void origin_step(const PoolK &p, int32_t &r0, int32_t &c0)
{
    r0 = r0 * p.sh - p.ph;
    c0 = c0 * p.sw - p.pw;
}

}  // namespace bs
