// Issue-rate probe: how many cycles a SIMD (and a single wave) needs per instruction of a given
// kind.  The sliding-window and tile kernels of this library are bound by instruction issue,
// not by HBM; these figures are what their cost model and the roofline notes rest on.  Each
// probe kernel repeats a block of eight independent instructions of one kind (inline assembly,
// so the compiler neither removes nor reorders them) `iterations` times per wave; the caller
// times the launch and divides.  No memory traffic beyond one store per lane at the end.
#include <hip/hip_runtime.h>

#include "bs_internal.h"

namespace bs {
namespace {

#define BS_REP8(I) I(0, 1) I(1, 2) I(2, 3) I(3, 4) I(4, 5) I(5, 6) I(6, 7) I(7, 0)
#define BS_OPS : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f), "+v"(g), "+v"(h) : "v"(seed), "s"(mask)

#define I_ADD(x, y) "v_add_f32 %" #x ", %" #x ", %8\n"
#define I_FMA(x, y) "v_fma_f32 %" #x ", %" #x ", %8, %" #y "\n"
#define I_MAX3(x, y) "v_max3_f32 %" #x ", %" #x ", %" #y ", %8\n"
#define I_CND_VCC(x, y) "v_cndmask_b32 %" #x ", %" #x ", %" #y ", vcc\n"
#define I_CND_SGPR(x, y) "v_cndmask_b32_e64 %" #x ", %" #x ", %" #y ", %9\n"
#define I_DPP(x, y) "v_mov_b32_dpp %" #x ", %" #y " wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
#define I_ADD_SALU(x, y) "v_add_f32 %" #x ", %" #x ", %8\ns_add_u32 s20, s20, 1\n"
#define I_ADD_BRANCH(x, y) "v_add_f32 %" #x ", %" #x ", %8\ns_cbranch_scc1 1f\n"
#define I_CHAIN(x, y) "v_add_f32 %0, %0, %8\n"

#define BS_PROBE(NAME, PRE, INSTR, POST, ...)                                                                          \
    __global__ __launch_bounds__(256) void probe_##NAME(float *out, int iters, float seed, unsigned long long mask) \
    {                                                                                                                   \
        float a = seed + threadIdx.x, b = a + 1.0f, c = a + 2.0f, d = a + 3.0f, e = a + 4.0f, f = a + 5.0f,          \
              g = a + 6.0f, h = a + 7.0f;                                                                               \
        asm volatile("v_cmp_gt_f32 vcc, %0, %1" : : "v"(a), "v"(seed) : "vcc");                                        \
        for (int i = 0; i < iters; ++i) asm volatile(PRE BS_REP8(INSTR) POST BS_OPS : __VA_ARGS__);                    \
        out[blockIdx.x * blockDim.x + threadIdx.x] = a + b + c + d + e + f + g + h;                                    \
    }

BS_PROBE(add, "", I_ADD, "", "memory")
BS_PROBE(fma, "", I_FMA, "", "memory")
BS_PROBE(max3, "", I_MAX3, "", "memory")
BS_PROBE(cnd_vcc, "", I_CND_VCC, "", "memory")
BS_PROBE(cnd_sgpr, "", I_CND_SGPR, "", "memory")
BS_PROBE(dpp, "s_nop 1\n", I_DPP, "", "memory")
BS_PROBE(add_salu, "", I_ADD_SALU, "", "s20", "scc")
BS_PROBE(add_branch, "s_cmp_lg_u32 0, 0\n", I_ADD_BRANCH, "1:\n", "scc")
BS_PROBE(chain, "", I_CHAIN, "", "memory")

// Streaming probe: what HBM delivers for an access pattern with no arithmetic at all.  Every lane
// reads R consecutive-per-wave 128-bit vectors (non-temporal, as the streaming kernels do) and
// writes one (R = 4: four bytes read per byte written, the pattern of a 2 x 2 pooling step;
// R = 1: a copy).  READ_ONLY: the vectors are folded together and stored only if the fold hits
// a value random data never produces, so the loads stay but nothing is written.
template <int R, bool READ_ONLY>
__global__ __launch_bounds__(256) void probe_stream_kernel(const uint4 *in, uint4 *out, uint32_t n_out)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= n_out) return;
    // lane i reads vectors r * n_out + i: R streams, each contiguous across the lanes
    u4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int r = 0; r < R; ++r) acc ^= __builtin_nontemporal_load(reinterpret_cast<const u4 *>(in) + (size_t)r * n_out + i);
    if (READ_ONLY && (acc.x != 0x7fc12345u || acc.y != 0x7fc12345u)) return;
    __builtin_nontemporal_store(acc, reinterpret_cast<u4 *>(out) + i);
}

}  // namespace
}  // namespace bs

using namespace bs;

extern "C" bs_status bs_probe_stream(int32_t reads_per_write, int32_t read_only, const void *in, uint64_t in_bytes, void *out,
                                     uint64_t out_bytes, void *stream)
{
    if (!in || !out) return BS_ERR_NULL;
    if (reads_per_write != 1 && reads_per_write != 2 && reads_per_write != 4) return BS_ERR_PARAM;
    if (out_bytes == 0 || out_bytes % 16 != 0 || out_bytes / 16 > 0x7fffffffull) return BS_ERR_PARAM;
    if (in_bytes < out_bytes * (uint64_t)reads_per_write) return BS_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15u) return BS_ERR_ALIGN;
    const uint32_t n_out = (uint32_t)(out_bytes / 16);
    const dim3 g((n_out + 255u) / 256u), b(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint4 *src = static_cast<const uint4 *>(in);
    uint4 *dst = static_cast<uint4 *>(out);
    if (read_only) {
        if (reads_per_write == 1) probe_stream_kernel<1, true><<<g, b, 0, st>>>(src, dst, n_out);
        else if (reads_per_write == 2) probe_stream_kernel<2, true><<<g, b, 0, st>>>(src, dst, n_out);
        else probe_stream_kernel<4, true><<<g, b, 0, st>>>(src, dst, n_out);
    } else {
        if (reads_per_write == 1) probe_stream_kernel<1, false><<<g, b, 0, st>>>(src, dst, n_out);
        else if (reads_per_write == 2) probe_stream_kernel<2, false><<<g, b, 0, st>>>(src, dst, n_out);
        else probe_stream_kernel<4, false><<<g, b, 0, st>>>(src, dst, n_out);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error((int32_t)e);
        return BS_ERR_HIP;
    }
    return BS_OK;
}

extern "C" bs_status bs_probe_issue_rate(int32_t kind, int32_t waves_per_simd, int32_t iterations, float *sink,
                                         uint64_t sink_floats, void *stream)
{
    if (!sink) return BS_ERR_NULL;
    if (waves_per_simd < 1 || waves_per_simd > 8 || iterations < 1) return BS_ERR_PARAM;
    Limits lim;
    int device = -1;
    const bs_status ds = device_limits(&lim, &device);
    if (ds != BS_OK) return ds;
    const uint32_t blocks = (uint32_t)lim.num_cus * (uint32_t)waves_per_simd;  // 4 waves per work-group: one per SIMD
    if (sink_floats < (uint64_t)blocks * 256) return BS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned long long mask = 0x5555555555555555ull;
    switch (kind) {
    case BS_PROBE_ADD: probe_add<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_FMA: probe_fma<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_MAX3: probe_max3<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_SELECT_VCC: probe_cnd_vcc<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_SELECT_SGPR: probe_cnd_sgpr<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_LANE_SHIFT: probe_dpp<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_ADD_SCALAR: probe_add_salu<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_ADD_BRANCH: probe_add_branch<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    case BS_PROBE_DEPENDENT_ADD: probe_chain<<<blocks, 256, 0, st>>>(sink, iterations, 1.0f, mask); break;
    default: return BS_ERR_RANGE;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error((int32_t)e);
        return BS_ERR_HIP;
    }
    return BS_OK;
}
