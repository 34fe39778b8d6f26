// Optional tracing (the paper's GPU back-end hooks into the vendor's profiling library,
// Section 5.4 / appendix; here: rocTX ranges that rocprofv3 --marker-trace records).
// With BS_TRACE=1 in the environment every sequence launch of bs_stack_run is wrapped in a
// named range "bs seq <i>/<n> <variant> steps <first>..<last>".  The rocTX library is looked
// up at run time, so the library has no link-time dependency on the profiler; without
// BS_TRACE, or if rocTX cannot be loaded, tracing costs one predictable branch per launch.
#include <dlfcn.h>

#include <cstdio>
#include <cstdlib>

#include "bs_internal.h"

namespace bs {

namespace {

struct Tracer {
    int (*push)(const char *) = nullptr;
    int (*pop)() = nullptr;
};

Tracer load_tracer()
{
    Tracer t;
    const char *e = std::getenv("BS_TRACE");
    if (!e || !*e || *e == '0') return t;
    for (const char *name : {"librocprofiler-sdk-roctx.so.1", "librocprofiler-sdk-roctx.so", "libroctx64.so.4", "libroctx64.so"}) {
        void *h = dlopen(name, RTLD_NOW | RTLD_GLOBAL);
        if (!h) continue;
        t.push = reinterpret_cast<int (*)(const char *)>(dlsym(h, "roctxRangePushA"));
        t.pop = reinterpret_cast<int (*)()>(dlsym(h, "roctxRangePop"));
        if (t.push && t.pop) return t;
        t.push = nullptr;
        t.pop = nullptr;
    }
    return t;
}

const Tracer &tracer()
{
    static const Tracer t = load_tracer();
    return t;
}

const char *variant_name(int32_t v)
{
    switch (v) {
    case BS_VARIANT_STREAM: return "stream";
    case BS_VARIANT_POOL_DIRECT: return "pool_direct";
    case BS_VARIANT_LDS_TILE: return "lds_tile";
    case BS_VARIANT_POOL_ROWS: return "pool_rows";
    case BS_VARIANT_PLANE_POOL: return "plane_pool";
    case BS_VARIANT_NHWC_STREAM: return "nhwc_stream";
    case BS_VARIANT_NHWC_POOL: return "nhwc_pool";
    }
    return "?";
}

}  // namespace

bool trace_enabled() { return tracer().push != nullptr; }

void trace_push_sequence(const Sequence &q, size_t index, size_t count)
{
    char label[128];
    std::snprintf(label, sizeof label, "bs seq %zu/%zu %s%s steps %d..%d", index + 1, count, variant_name(q.variant),
                  q.jit ? " (run-time build)" : "", q.first_step, q.first_step + q.n_steps - 1);
    (void)tracer().push(label);
}

void trace_pop() { (void)tracer().pop(); }

}  // namespace bs
