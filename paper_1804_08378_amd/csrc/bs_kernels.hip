// HIP kernels (gfx950 / CDNA4, wave64) for depth-first execution of a sequence of
// steps, and their launchers.
//
// Kernel families, following the two code-generation cases of Section 4.1 (single-step
// sequence: values pass from operation to operation directly; multi-step sequence: cached
// buffer + synchronisation between steps) and the GPU building blocks of Section 4.4
// (element-wise; non-stacked pooling; stacked pooling with two on-chip buffers swapped
// after each step).  In this file:
//
//   stream_kernel       element-wise only.  128-bit loads/stores, everything in registers.
//   pool_direct_kernel  one pooling operation with disjoint windows (k == s, p == 0)
//                       plus element-wise operations before and after it.  Each lane
//                       owns whole windows: KH 128-bit row loads give VEC/KW outputs.
//   plane_pool_kernel   one pooling operation whose window is the whole (small) plane:
//                       one lane per plane.
//
// In their own files: the register sliding-window kernels for one or two pooling
// operations with overlapping / padded windows (bs_rows_device.h) and the LDS tile
// kernels for any sequence (bs_lds_device.h), both also built at plan time for
// signatures that have no instance compiled into the library (bs_jit.cpp).
//
// Arithmetic is float32 with one fixed operation order per layer so that results do
// not depend on the tiling: BatchNorm is one fused multiply-add with host-folded
// scale/shift, the average's sum runs row-major over the in-range cells from +0 and is
// multiplied by a float32 reciprocal, max takes the first maximum in row-major order.
// With bfloat16 storage every layer's output is rounded to bfloat16 (nearest-even).
// No MFMA: the path moves 5..12 bytes per element and does ~10 flops on them.
#include "bs_device.h"
#include "bs_internal.h"

namespace bs {

// ------------------------------------------------------ element-wise operations
// Apply a list of element-wise operations to U register vectors at once.  The list is
// wave-uniform, so interpreting it costs scalar instructions only.  Lanes that have no
// work carry c = 0 / off = 0 (safe addresses) and simply compute values nobody stores:
// no load here is predicated.
//   c[u]    channel of vector u (BatchNorm parameters)
//   off[u]  element offset of vector u in this level's tensors (residual loads)
//   CODE    >= 0: the list's kinds as a code of base-K_EW_BASE digits (n_ew is ignored): the list unrolls into
//           straight code and only the arguments come from `ew`; -1: kinds and length are read at run time
template <int DT, int VEC, int U, int CODE = -1>
BS_DEV void apply_ew(float (&x)[U][VEC], const int32_t (&c)[U], const uint32_t (&off)[U],
                     const EwOp *ew, int32_t n_ew, const float *__restrict__ params, int32_t C,
                     const void *const *res)
{
    auto one = [&](const int32_t kind, const int32_t arg) {
        if (kind == OP_BN) {
            float sc[U], sh[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                sc[u] = params[arg + c[u]];
                sh[u] = params[arg + C + c[u]];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = __builtin_fmaf(x[u][i], sc[u], sh[u]);
                round_store_all<DT, VEC>(x[u]);
            }
        } else if (kind == OP_RELU) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = __builtin_fmaxf(x[u][i], 0.0f);  // NaN, -0 -> +0
        } else if (kind == OP_LEAKY) {
            const float slope = params[arg];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(x[u][i] > 0.0f ? x[u][i] : x[u][i] * slope);
        } else if (kind == OP_CLAMP) {
            const float lo = params[arg], hi = params[arg + 1];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i)  // v_max / v_min: a NaN becomes lo
                    x[u][i] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[u][i], lo), hi));
        } else {  // OP_ADD
            const void *rp = res[arg];
            Raw<DT, VEC> rr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) rr[u] = load_raw<DT, VEC, true>(rp, off[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float r[VEC];
                unpack<DT, VEC>(rr[u], r);
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u][i] = round_store<DT>(x[u][i] + r[i]);
            }
        }
    };
    if constexpr (CODE >= 0) {
#pragma unroll
        for (int j = 0; j < ew_code_len(CODE); ++j) one(ew_code_kind(CODE, j), ew[j].arg);
    } else {
#pragma clang loop unroll(disable)
        for (int32_t j = 0; j < n_ew; ++j) one(ew[j].kind, ew[j].arg);
    }
}

// =============================================================================
// stream_kernel: element-wise only sequence.  A work-group takes nthr * U
// consecutive 128-bit vectors; lane t handles vectors t, t + nthr, ...
// CODE: the kinds of the list's operations as a compile-time code (apply_ew), or -1.
// =============================================================================
template <int DT, int VEC, int U, int CODE = -1>
__global__ __launch_bounds__(512) void stream_kernel(const StreamK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    Raw<DT, VEC> raw[U];
    bool valid[U];
    uint32_t off[U], img[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        i = valid[u] ? i : 0u;
        off[u] = i * VEC;
        const uint32_t plane = fdiv(i, k.div_plane);
        img[u] = fdiv(plane, k.div_c);
        c[u] = (int32_t)(plane - img[u] * (uint32_t)k.C);
        raw[u] = load_raw<DT, VEC, true>(image_base<DT>(k.in, img[u], k.in_extra), off[u]);
    }
    float x[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) unpack<DT, VEC>(raw[u], x[u]);
    apply_ew<DT, VEC, U, CODE>(x, c, off, k.ew, k.n_ew, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (valid[u]) store_elems<DT, VEC>(image_base<DT>(k.out, img[u], k.out_extra), off[u], x[u]);
}

// =============================================================================
// stream_flat_kernel: the same for planes whose size is no multiple of the vector width (the
// 35 x 35, 17 x 17, 147 x 147 grids of Inception-style networks).  The tensor is taken as one
// run of 128-bit vectors; a vector may begin in one plane and end in the next (never further:
// a plane has at least VEC cells), so BatchNorm picks each element's parameters from the two
// channels involved.  With 16-bit storage this doubles the throughput of the scalar kernel.
// Dense tensors only (a vector may straddle two images as well).
// =============================================================================
template <int DT, int VEC, int U>
__global__ __launch_bounds__(512) void stream_flat_kernel(const StreamK k)
{
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t hw = k.div_plane.d;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        const bool valid = i < k.total;
        i = valid ? i : 0u;
        const uint32_t off = i * VEC;
        const uint32_t plane = fdiv(off, k.div_plane);
        const uint32_t nfirst = hw - (off - plane * hw);  // elements of the vector that lie in `plane`
        const uint32_t c0 = plane - fdiv(plane, k.div_c) * (uint32_t)k.C;
        const uint32_t c1 = c0 + 1 == (uint32_t)k.C ? 0u : c0 + 1;
        float x[VEC];
        unpack<DT, VEC>(load_raw<DT, VEC, true>(k.in, off), x);
#pragma clang loop unroll(disable)
        for (int32_t j = 0; j < k.n_ew; ++j) {
            const int32_t kind = k.ew[j].kind, arg = k.ew[j].arg;
            if (kind == OP_BN) {
                const float sc0 = k.params[arg + c0], sh0 = k.params[arg + k.C + c0];
                const float sc1 = k.params[arg + c1], sh1 = k.params[arg + k.C + c1];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const bool first = (uint32_t)e < nfirst;
                    x[e] = round_store<DT>(__builtin_fmaf(x[e], first ? sc0 : sc1, first ? sh0 : sh1));
                }
            } else if (kind == OP_RELU) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = __builtin_fmaxf(x[e], 0.0f);
            } else if (kind == OP_LEAKY) {
                const float slope = k.params[arg];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(x[e] > 0.0f ? x[e] : x[e] * slope);
            } else if (kind == OP_CLAMP) {
                const float lo = k.params[arg], hi = k.params[arg + 1];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(__builtin_fminf(__builtin_fmaxf(x[e], lo), hi));
            } else {  // OP_ADD
                float r[VEC];
                unpack<DT, VEC>(load_raw<DT, VEC, true>(k.res[arg], off), r);
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = round_store<DT>(x[e] + r[e]);
            }
        }
        if (valid) store_elems<DT, VEC>(k.out, off, x);
    }
}

// =============================================================================
// pool_direct_kernel: [element-wise]* pool(k == s, p == 0) [element-wise]*,
// windows disjoint, one 128-bit column block (VEC input columns) per unit.
// unit = (plane, output row oh, column block cv); it reads KH rows x VEC columns and
// produces VEC / KW outputs.  Consecutive lanes take consecutive column blocks, so each
// row load of a wave is one contiguous run.
// =============================================================================
// SIG selects how the element-wise lists are executed: 0 interprets k.pre / k.post at
// run time; 1 is compiled for "BatchNorm, ReLU, pool" with nothing after the pool (the
// VGG stack, the DenseNet transition), whose BatchNorm parameters are requested together
// with the data so a wave makes one round trip to memory instead of two.
template <int DT, int VEC, int KH, int KW, int U, int SIG>
__global__ __launch_bounds__(512) void pool_direct_kernel(const PoolDirectK k)
{
    constexpr int NO = VEC / KW;  // outputs per unit
    const uint32_t nthr = blockDim.x;
    const uint32_t base = blockIdx.x * (nthr * U) + threadIdx.x;
    const uint32_t wv = k.div_wv.d;

    Raw<DT, VEC> raw[U][KH];
    bool valid[U];
    uint32_t in_off[U], out_off[U], idx0[U], img[U];
    int32_t c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t i = base + u * nthr;
        valid[u] = i < k.total;
        i = valid[u] ? i : 0u;
        const uint32_t t = fdiv(i, k.div_wv);
        const uint32_t cv = i - t * wv;
        const uint32_t plane = fdiv(t, k.div_ho);
        const uint32_t oh = t - plane * (uint32_t)k.Ho;
        img[u] = fdiv(plane, k.div_c);
        c[u] = (int32_t)(plane - img[u] * (uint32_t)k.C);
        idx0[u] = (oh * KH) * (uint32_t)k.W + cv * VEC;  // first cell of the unit in its plane
        in_off[u] = plane * (uint32_t)(k.H * k.W) + idx0[u];
        out_off[u] = (plane * (uint32_t)k.Ho + oh) * (uint32_t)k.Wo + cv * NO;
        const void *inp = image_base<DT>(k.in, img[u], k.in_extra);
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) raw[u][dh] = load_raw<DT, VEC, true>(inp, in_off[u] + dh * (uint32_t)k.W);
    }
    float sc[U], sh[U];
    if constexpr (SIG == 1) {
        const int32_t arg = k.pre[0].arg;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sc[u] = k.params[arg + c[u]];
            sh[u] = k.params[arg + k.C + c[u]];
        }
    }

    float y[U][NO];
    int32_t yi[U][NO];
    const bool is_max = k.pool.kind == OP_MAXPOOL;
    const bool want_idx = k.idx != nullptr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float x[KH][VEC];
        int32_t c1[KH];
        uint32_t o1[KH];
#pragma unroll
        for (int dh = 0; dh < KH; ++dh) {
            c1[dh] = c[u];
            o1[dh] = in_off[u] + dh * (uint32_t)k.W;
            unpack<DT, VEC>(raw[u][dh], x[dh]);
        }
        if constexpr (SIG == 1) {
#pragma unroll
            for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    x[dh][i] = __builtin_fmaxf(round_store<DT>(__builtin_fmaf(x[dh][i], sc[u], sh[u])), 0.0f);
        } else {
            apply_ew<DT, VEC, KH>(x, c1, o1, k.pre, k.n_pre, k.params, k.C, k.res);
        }
        if (is_max) {
            if (want_idx) {
#pragma unroll
                for (int j = 0; j < NO; ++j) {
                    float best = -INFINITY;
                    int32_t bi = (int32_t)idx0[u] + j * KW;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            const float v = x[dh][j * KW + dw];
                            const bool g = v > best;
                            best = g ? v : best;
                            bi = g ? (int32_t)(idx0[u] + dh * (uint32_t)k.W) + j * KW + dw : bi;
                        }
                    y[u][j] = best;
                    yi[u][j] = bi;
                }
            } else {
#pragma unroll
                for (int j = 0; j < NO; ++j) {
                    float best = -INFINITY;
#pragma unroll
                    for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                        for (int dw = 0; dw < KW; ++dw) {
                            best = __builtin_fmaxf(best, x[dh][j * KW + dw]);
                        }
                    y[u][j] = best;
                    yi[u][j] = 0;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NO; ++j) {
                float sum = 0.0f;
#pragma unroll
                for (int dh = 0; dh < KH; ++dh)
#pragma unroll
                    for (int dw = 0; dw < KW; ++dw) sum = sum + x[dh][j * KW + dw];
                y[u][j] = round_store<DT>(sum * k.pool.inv_kk);
                yi[u][j] = 0;
            }
        }
    }
    if constexpr (SIG == 0) apply_ew<DT, NO, U>(y, c, out_off, k.post, k.n_post, k.params, k.C, k.res);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (!valid[u]) continue;
        store_elems<DT, NO>(image_base<DT>(k.out, img[u], k.out_extra), out_off[u], y[u]);
        if (want_idx && is_max) {
            store_indices<NO>(k.idx + out_off[u], yi[u]);
        }
    }
}

// =============================================================================
// plane_pool_kernel: [element-wise]* pool(window = the whole plane) [element-wise]*, the
// global pooling at the end of a network.  One lane per plane walks the plane in row-major
// order (the order in which the average's sum and the first-maximum rule are defined), eight
// elements requested at a time; planes are small here (the planner sends large ones to the
// tile kernels).  A plane is contiguous, so a lane's loads fall into a few cache lines.
// =============================================================================
template <int DT>
__global__ __launch_bounds__(256) void plane_pool_kernel(const PoolDirectK k)
{
    constexpr int U = 8;
    uint32_t plane = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = plane < k.total;
    plane = live ? plane : 0u;
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c1[1] = {(int32_t)(plane - img * (uint32_t)k.C)};
    const uint32_t hw = (uint32_t)(k.H * k.W), base = plane * hw;
    const void *inp = image_base<DT>(k.in, img, k.in_extra);
    const bool is_max = k.pool.kind == OP_MAXPOOL;
    float acc = is_max ? -INFINITY : 0.0f;
    int32_t bi = 0;  // first cell of the plane
    for (uint32_t i0 = 0; i0 < hw; i0 += U) {
        Raw<DT, 1> raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) raw[u] = load_raw<DT, 1>(inp, base + min(i0 + u, hw - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float x[1][1];
            unpack<DT, 1>(raw[u], x[0]);
            const uint32_t o1[1] = {base + min(i0 + u, hw - 1)};
            apply_ew<DT, 1, 1>(x, c1, o1, k.pre, k.n_pre, k.params, k.C, k.res);
            const float v = x[0][0];
            if (i0 + u < hw) {
                if (is_max) {
                    const bool g = v > acc;
                    acc = g ? v : acc;
                    bi = g ? (int32_t)(i0 + u) : bi;
                } else {
                    acc = acc + v;
                }
            }
        }
    }
    float y[1][1] = {{is_max ? acc : round_store<DT>(acc * k.pool.inv_kk)}};
    const uint32_t oo[1] = {plane};  // Ho = Wo = 1: the output (and a residual of its shape) is indexed by plane
    apply_ew<DT, 1, 1>(y, c1, oo, k.post, k.n_post, k.params, k.C, k.res);
    if (live) {
        store_elems<DT, 1>(image_base<DT>(k.out, img, k.out_extra), plane, y[0]);
        if (k.idx && is_max) k.idx[plane] = bi;
    }
}

// =============================================================================
// plane_pool_lds_kernel: the same operation for planes of more than a few cells.  A lane that
// walks its plane in global memory waits for one memory round trip per handful of cells; here
// a work-group takes k.ppg consecutive planes (one contiguous range of a dense tensor), all its
// lanes fetch that range together -- coalesced, one round trip, at most eight cells per lane --
// and leave the values, after the element-wise operations in front of the pool, in LDS; then
// lane p walks plane p in LDS, in the same row-major order.  The LDS pitch of a plane is odd, so
// the lanes of the second phase hit different banks.
// =============================================================================
template <int DT>
__global__ __launch_bounds__(256) void plane_pool_lds_kernel(const PoolDirectK k)
{
    extern __shared__ float staged[];
    constexpr int U = 8;
    const uint32_t hw = (uint32_t)(k.H * k.W);
    const uint32_t p0 = blockIdx.x * (uint32_t)k.ppg;
    const uint32_t np = min((uint32_t)k.ppg, k.total - p0);  // planes of this group (the grid covers k.total exactly)
    const uint32_t n = np * hw;                              // cells of this group
    for (uint32_t e0 = threadIdx.x; e0 < n; e0 += blockDim.x * U) {
        Raw<DT, 1> raw[U];
        uint32_t off[U], pl[U];
        int32_t c[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t e = min(e0 + u * blockDim.x, n - 1);  // lanes past the end repeat the last cell
            pl[u] = fdiv(e, k.div_wv);                           // plane within the group
            const uint32_t plane = p0 + pl[u];
            const uint32_t img = fdiv(plane, k.div_c);
            c[u] = (int32_t)(plane - img * (uint32_t)k.C);
            off[u] = p0 * hw + e;
            raw[u] = load_raw<DT, 1>(image_base<DT>(k.in, img, k.in_extra), off[u]);
        }
        float x[U][1];
#pragma unroll
        for (int u = 0; u < U; ++u) unpack<DT, 1>(raw[u], x[u]);
        apply_ew<DT, 1, U>(x, c, off, k.pre, k.n_pre, k.params, k.C, k.res);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t e = e0 + u * blockDim.x;
            if (e < n) staged[pl[u] * (uint32_t)k.pitch + (e - pl[u] * hw)] = x[u][0];
        }
    }
    __syncthreads();
    if (threadIdx.x >= np) return;
    const uint32_t plane = p0 + threadIdx.x;
    const uint32_t img = fdiv(plane, k.div_c);
    const int32_t c1[1] = {(int32_t)(plane - img * (uint32_t)k.C)};
    const float *cells = staged + threadIdx.x * (uint32_t)k.pitch;
    const bool is_max = k.pool.kind == OP_MAXPOOL;
    float acc = is_max ? -INFINITY : 0.0f;
    int32_t bi = 0;  // first cell of the plane
    for (uint32_t i0 = 0; i0 < hw; i0 += U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = cells[min(i0 + u, hw - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i0 + u < hw) {
                if (is_max) {
                    const bool g = v[u] > acc;
                    acc = g ? v[u] : acc;
                    bi = g ? (int32_t)(i0 + u) : bi;
                } else {
                    acc = acc + v[u];
                }
            }
    }
    float y[1][1] = {{is_max ? acc : round_store<DT>(acc * k.pool.inv_kk)}};
    const uint32_t oo[1] = {plane};
    apply_ew<DT, 1, 1>(y, c1, oo, k.post, k.n_post, k.params, k.C, k.res);
    store_elems<DT, 1>(image_base<DT>(k.out, img, k.out_extra), plane, y[0]);
    if (k.idx && is_max) k.idx[plane] = bi;
}

// =============================================================================
// Host side: device queries, parameter upload, launchers.
// =============================================================================
static bs_status hip_fail(hipError_t e)
{
    set_hip_error((int32_t)e);
    (void)hipGetLastError();
    return BS_ERR_HIP;
}

bs_status device_limits(Limits *lim, int *device)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e);
    int smem = 0;
    e = hipDeviceGetAttribute(&smem, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return hip_fail(e);
    lim->num_cus = cus;
    lim->max_lds_bytes = (uint64_t)smem;
    *device = dev;
    return BS_OK;
}

int current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return dev;
}

bs_status upload_params(bs_stack *s)
{
    free_params(s);
    if (s->host_params.empty()) return BS_OK;
    const size_t bytes = s->host_params.size() * sizeof(float);
    float *d = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&d), bytes);
    if (e != hipSuccess) return hip_fail(e);
    // synchronous copy from pageable memory: complete when it returns
    e = hipMemcpy(d, s->host_params.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(d);
        return hip_fail(e);
    }
    s->dev_params = d;
    return BS_OK;
}

void free_params(bs_stack *s)
{
    if (s->dev_params) {
        (void)hipFree(s->dev_params);
        s->dev_params = nullptr;
    }
}

template <int DT, int VEC, int KH>
static void launch_direct_kw(const PoolDirectK &k, int kw, dim3 grid, dim3 block, hipStream_t st)
{
    if constexpr (VEC == 8) {
        if (kw == 8) { pool_direct_kernel<DT, VEC, KH, 8, K_DIRECT_U, 0><<<grid, block, 0, st>>>(k); return; }
    }
    if constexpr (KH == 2) {
        const bool bn_relu_pool = k.n_pre == 2 && k.pre[0].kind == OP_BN && k.pre[1].kind == OP_RELU && k.n_post == 0;
        if (kw == 2 && bn_relu_pool) { pool_direct_kernel<DT, VEC, 2, 2, K_DIRECT_U, 1><<<grid, block, 0, st>>>(k); return; }
    }
    if (kw == 1) pool_direct_kernel<DT, VEC, KH, 1, K_DIRECT_U, 0><<<grid, block, 0, st>>>(k);
    else if (kw == 2) pool_direct_kernel<DT, VEC, KH, 2, K_DIRECT_U, 0><<<grid, block, 0, st>>>(k);
    else pool_direct_kernel<DT, VEC, KH, 4, K_DIRECT_U, 0><<<grid, block, 0, st>>>(k);
}

template <int DT, int VEC>
static void launch_direct(const PoolDirectK &k, dim3 grid, dim3 block, hipStream_t st)
{
    switch (k.pool.kh) {
    case 1: launch_direct_kw<DT, VEC, 1>(k, k.pool.kw, grid, block, st); break;
    case 2: launch_direct_kw<DT, VEC, 2>(k, k.pool.kw, grid, block, st); break;
    case 3: launch_direct_kw<DT, VEC, 3>(k, k.pool.kw, grid, block, st); break;
    default: launch_direct_kw<DT, VEC, 4>(k, k.pool.kw, grid, block, st); break;
    }
}

// Launch the sequence's run-time build (compiled at plan time) with argument block `args`.
static bs_status launch_built(const Sequence &q, bool want_idx, const void *args, size_t bytes, void *stream)
{
    void *fn = q.jit_fn[want_idx ? 1 : 0];
    if (!fn) return BS_ERR_NOT_PLANNED;
    return jit_launch(fn, args, bytes, q.grid, q.threads, q.lds_bytes, stream);
}

// stream_kernel with full-width vectors: the lists of the common networks -- BatchNorm, ReLU (DenseNet) and
// BatchNorm, Add, ReLU (ResNet) -- are compiled in, any other list is read at run time.
template <int DT, int VEC>
static void launch_stream(const StreamK &k, dim3 grid, dim3 block, hipStream_t st)
{
    constexpr int BN_RELU = OP_BN + OP_RELU * K_EW_BASE, BN_ADD_RELU = OP_BN + (OP_ADD + OP_RELU * K_EW_BASE) * K_EW_BASE;
    int32_t code = 0, digit = 1;
    for (int32_t j = 0; j < k.n_ew && j < 4; ++j, digit *= K_EW_BASE) code += k.ew[j].kind * digit;
    if (k.n_ew == 2 && code == BN_RELU) stream_kernel<DT, VEC, K_STREAM_U, BN_RELU><<<grid, block, 0, st>>>(k);
    else if (k.n_ew == 3 && code == BN_ADD_RELU) stream_kernel<DT, VEC, K_STREAM_U, BN_ADD_RELU><<<grid, block, 0, st>>>(k);
    else stream_kernel<DT, VEC, K_STREAM_U><<<grid, block, 0, st>>>(k);
}

bs_status launch_sequence(const bs_stack *s, const Sequence &q, const void *in, void *out,
                          uint32_t in_extra, uint32_t out_extra, const void *const *res,
                          int32_t *const *idx, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t dtype = s->dtype;
    if (q.grid < 1 || q.grid > 0x7fffffffll) return BS_ERR_UNSUPPORTED;
    const dim3 grid((uint32_t)q.grid), block((uint32_t)q.threads);
    const void *rp[K_MAX_RES] = {nullptr, nullptr, nullptr, nullptr};
    for (int32_t j = 0; j < q.n_res; ++j) rp[j] = res[q.res_map[j]];
    int32_t *ip[K_MAX_IDX] = {nullptr, nullptr, nullptr, nullptr};
    for (int32_t j = 0; j < q.n_idx; ++j) ip[j] = idx ? idx[q.idx_map[j]] : nullptr;

    switch (q.variant) {
    case BS_VARIANT_STREAM: {
        // vector widths the compiled instances exist for (guards against a plan / kernel mismatch)
        if (q.vec != 1 && q.vec != (dtype == BS_F32 ? 4 : 8)) return BS_ERR_UNSUPPORTED;
        StreamK k = q.stream;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        if (k.flat) {
            // planned for vectors that run over plane boundaries: dense tensors only
            if (q.vec != (dtype == BS_F32 ? 4 : 8) || (int64_t)k.div_plane.d < q.vec) return BS_ERR_UNSUPPORTED;
            if (in_extra != 0 || out_extra != 0) {
                // channel slices: the scalar kernel, whose argument block differs in the element count only
                k.total *= (uint32_t)q.vec;
                k.flat = 0;
                const int64_t per_group = (int64_t)q.threads * K_STREAM_U;
                const dim3 g1((uint32_t)(((int64_t)k.total + per_group - 1) / per_group));
                if (dtype == BS_BF16) stream_kernel<DT_BF16, 1, K_STREAM_U><<<g1, block, 0, st>>>(k);
                else if (dtype == BS_F16) stream_kernel<DT_F16, 1, K_STREAM_U><<<g1, block, 0, st>>>(k);
                else stream_kernel<DT_F32, 1, K_STREAM_U><<<g1, block, 0, st>>>(k);
            } else if (dtype == BS_BF16) {
                stream_flat_kernel<DT_BF16, 8, K_STREAM_U><<<grid, block, 0, st>>>(k);
            } else if (dtype == BS_F16) {
                stream_flat_kernel<DT_F16, 8, K_STREAM_U><<<grid, block, 0, st>>>(k);
            } else {
                stream_flat_kernel<DT_F32, 4, K_STREAM_U><<<grid, block, 0, st>>>(k);
            }
            break;
        }
        if (dtype == BS_BF16) {
            if (q.vec == 8) launch_stream<DT_BF16, 8>(k, grid, block, st);
            else stream_kernel<DT_BF16, 1, K_STREAM_U><<<grid, block, 0, st>>>(k);
        } else if (dtype == BS_F16) {
            if (q.vec == 8) launch_stream<DT_F16, 8>(k, grid, block, st);
            else stream_kernel<DT_F16, 1, K_STREAM_U><<<grid, block, 0, st>>>(k);
        } else {
            if (q.vec == 4) launch_stream<DT_F32, 4>(k, grid, block, st);
            else stream_kernel<DT_F32, 1, K_STREAM_U><<<grid, block, 0, st>>>(k);
        }
        break;
    }
    case BS_VARIANT_POOL_DIRECT: {
        // column blocks the instances exist for: one 128-bit vector, or one 64-bit vector with 16-bit storage
        if ((q.vec != (dtype == BS_F32 ? 4 : 8) && !(dtype != BS_F32 && q.vec == 4)) || q.vec % q.direct.pool.kw != 0 ||
            (int64_t)q.direct.div_wv.d * q.vec != q.direct.W)
            return BS_ERR_UNSUPPORTED;
        PoolDirectK k = q.direct;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        k.idx = ip[0];
        if (dtype == BS_BF16) {
            if (q.vec == 8) launch_direct<DT_BF16, 8>(k, grid, block, st);
            else launch_direct<DT_BF16, 4>(k, grid, block, st);
        } else if (dtype == BS_F16) {
            if (q.vec == 8) launch_direct<DT_F16, 8>(k, grid, block, st);
            else launch_direct<DT_F16, 4>(k, grid, block, st);
        } else {
            launch_direct<DT_F32, 4>(k, grid, block, st);
        }
        break;
    }
    case BS_VARIANT_PLANE_POOL: {
        PoolDirectK k = q.direct;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        k.idx = ip[0];
        if (k.ppg > 0) {
            // staged through LDS: the argument block must describe what the kernel assumes
            const int64_t hw = (int64_t)k.H * k.W;
            if (k.pitch < hw || k.ppg > q.threads || (int64_t)k.div_wv.d != hw || q.lds_bytes < (uint64_t)k.ppg * k.pitch * 4 ||
                q.grid != ((int64_t)k.total + k.ppg - 1) / k.ppg)
                return BS_ERR_UNSUPPORTED;
            const size_t lds = (size_t)q.lds_bytes;
            if (dtype == BS_BF16) plane_pool_lds_kernel<DT_BF16><<<grid, block, lds, st>>>(k);
            else if (dtype == BS_F16) plane_pool_lds_kernel<DT_F16><<<grid, block, lds, st>>>(k);
            else plane_pool_lds_kernel<DT_F32><<<grid, block, lds, st>>>(k);
            break;
        }
        if (dtype == BS_BF16) plane_pool_kernel<DT_BF16><<<grid, block, 0, st>>>(k);
        else if (dtype == BS_F16) plane_pool_kernel<DT_F16><<<grid, block, 0, st>>>(k);
        else plane_pool_kernel<DT_F32><<<grid, block, 0, st>>>(k);
        break;
    }
    case BS_VARIANT_POOL_ROWS: {
        if (q.n_levels == 2) {
            PoolRows2K k = q.rows2;
            k.in = in; k.out = out; k.params = s->dev_params;
            k.in_extra = in_extra; k.out_extra = out_extra;
            k.idx = ip[0];
            const bool want_idx = k.idx != nullptr && k.pool2.kind == OP_MAXPOOL;
            if (k.spw > 0 && !xrows2_launchable(k, dtype, q.grid, q.threads)) return BS_ERR_UNSUPPORTED;
            const bs_status ls = q.jit ? launch_built(q, want_idx, &k, sizeof k, stream)
                                       : (k.spw > 0 ? launch_xrows2(k, dtype, q.grid, q.threads, stream)
                                                    : launch_rows2(k, dtype, q.grid, q.threads, stream));
            if (ls != BS_OK) return ls;
            break;
        }
        PoolRowsK k = q.rows;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        k.idx = ip[0];
        const bool want_idx = k.idx != nullptr && k.pool.kind == OP_MAXPOOL;
        if (k.spw > 0 && !xrows_launchable(k, dtype, q.grid, q.threads)) return BS_ERR_UNSUPPORTED;
        const bs_status ls = q.jit ? launch_built(q, want_idx, &k, sizeof k, stream)
                                   : (k.spw > 0 ? launch_xrows(k, dtype, q.grid, q.threads, stream)
                                                : launch_rows(k, dtype, q.grid, q.threads, stream));
        if (ls != BS_OK) return ls;
        break;
    }
    case BS_VARIANT_ROWS_CHAIN: {
        RowsChainK k = q.chain;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        if (!xrows_chain_launchable(k, dtype, q.grid, q.threads)) return BS_ERR_UNSUPPORTED;
        const bs_status ls = q.jit ? launch_built(q, false, &k, sizeof k, stream) : launch_xrows_chain(k, dtype, q.grid, q.threads, stream);
        if (ls != BS_OK) return ls;
        break;
    }
    case BS_VARIANT_LDS_TILE: {
        LdsSeqK k = q.lds;
        k.in = in; k.out = out; k.params = s->dev_params;
        k.in_extra = in_extra; k.out_extra = out_extra;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        for (int j = 0; j < K_MAX_IDX; ++j) k.idx[j] = ip[j];
        bool want_idx = false;
        for (int j = 0; j < q.n_idx; ++j) want_idx = want_idx || ip[j] != nullptr;
        const bs_status ls = q.jit ? launch_built(q, want_idx, &k, sizeof k, stream)
                                   : launch_lds(k, dtype, q.grid, q.threads, q.lds_bytes, stream);
        if (ls != BS_OK) return ls;
        break;
    }
    case BS_VARIANT_NHWC_STREAM:
    case BS_VARIANT_NHWC_POOL: {
        NhwcK k = q.nhwc;
        // a channel slice of a channels-last tensor: the batch stride is a whole number of pixels
        // of the larger tensor (checked by the caller), the slice skips the same count per pixel
        const uint32_t hw_in = (uint32_t)(q.in_shape[2] * q.in_shape[3]), hw_out = (uint32_t)(q.out_shape[2] * q.out_shape[3]);
        if (in_extra % hw_in != 0 || out_extra % hw_out != 0) return BS_ERR_UNSUPPORTED;
        k.in_xp = in_extra / hw_in;
        k.out_xp = out_extra / hw_out;
        k.in = in; k.out = out; k.params = s->dev_params;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        k.idx = ip[0];
        const bs_status ls = launch_nhwc(k, dtype, q.vec, q.grid, q.threads, q.lds_bytes, stream);
        if (ls != BS_OK) return ls;
        break;
    }
    case BS_VARIANT_NHWC_TILE: {
        NhwcTile2K k = q.nhwc2;
        const uint32_t hw_in = (uint32_t)(q.in_shape[2] * q.in_shape[3]), hw_out = (uint32_t)(q.out_shape[2] * q.out_shape[3]);
        if (in_extra % hw_in != 0 || out_extra % hw_out != 0) return BS_ERR_UNSUPPORTED;
        k.in_xp = in_extra / hw_in;
        k.out_xp = out_extra / hw_out;
        k.in = in; k.out = out; k.params = s->dev_params;
        for (int j = 0; j < K_MAX_RES; ++j) k.res[j] = rp[j];
        k.idx = ip[0];
        const bs_status ls = launch_nhwc_tile2(k, dtype, q.vec, q.grid, q.threads, q.lds_bytes, stream);
        if (ls != BS_OK) return ls;
        break;
    }
    case BS_VARIANT_NHWC_ROWS: {
        NhwcTile2K k = q.nhwc2;
        const uint32_t hw_in = (uint32_t)(q.in_shape[2] * q.in_shape[3]), hw_out = (uint32_t)(q.out_shape[2] * q.out_shape[3]);
        if (in_extra % hw_in != 0 || out_extra % hw_out != 0) return BS_ERR_UNSUPPORTED;
        k.in_xp = in_extra / hw_in;
        k.out_xp = out_extra / hw_out;
        k.in = in; k.out = out; k.params = s->dev_params;
        const bs_status ls = launch_nhwc_rows2(k, dtype, q.vec, q.grid, q.threads, stream);
        if (ls != BS_OK) return ls;
        break;
    }
    default:
        return BS_ERR_UNSUPPORTED;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e);
    return BS_OK;
}

}  // namespace bs
