// Host-side helpers: per-kernel timing with HIP events on the caller's stream (instrumentation only),
// and the once-per-device raising of a kernel's dynamic-LDS limit.
#include <dlfcn.h>

#include <mutex>
#include <vector>

#include "sgc_internal.h"

namespace sgc {

bool g_profile_on = false;

namespace {
struct Span {
    int cls;
    hipEvent_t a, b;
};
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_pool;
struct Open {
    int cls;
    hipEvent_t a;
};
std::vector<Open> g_open; // scopes nest (a panel refill inside a contraction scope)
bool g_failed = false;

hipEvent_t get_event()
{
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) {
        g_failed = true;
        return nullptr;
    }
    return e;
}
} // namespace

hipError_t raise_dynamic_lds(const void *kernel, size_t bytes)
{
    struct Done {
        const void *kernel;
        int device;
        size_t bytes;
    };
    static std::vector<Done> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    for (const Done &d : done)
        if (d.kernel == kernel && d.device == dev && d.bytes >= bytes)
            return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess)
        done.push_back(Done{kernel, dev, bytes});
    return e;
}

// ---- named ranges for external profilers (rocprofv3 --marker-trace): the marker library is looked up at run
// time so that the library does not depend on it; without it the ranges are no-ops ----
namespace {
typedef int (*roctx_push_fn)(const char *);
typedef int (*roctx_pop_fn)();
roctx_push_fn g_roctx_push = nullptr;
roctx_pop_fn g_roctx_pop = nullptr;
std::once_flag g_roctx_once;
void roctx_resolve()
{
    for (const char *name : {"librocprofiler-sdk-roctx.so.1", "librocprofiler-sdk-roctx.so", "libroctx64.so.4", "libroctx64.so"}) {
        void *h = dlopen(name, RTLD_LAZY | RTLD_LOCAL);
        if (!h)
            continue;
        roctx_push_fn push = reinterpret_cast<roctx_push_fn>(dlsym(h, "roctxRangePushA"));
        roctx_pop_fn pop = reinterpret_cast<roctx_pop_fn>(dlsym(h, "roctxRangePop"));
        if (push && pop) {
            g_roctx_push = push;
            g_roctx_pop = pop;
            return;
        }
    }
}
} // namespace

RangeScope::RangeScope(const char *name)
{
    std::call_once(g_roctx_once, roctx_resolve);
    on = g_roctx_push != nullptr;
    if (on)
        g_roctx_push(name);
}

RangeScope::~RangeScope()
{
    if (on)
        g_roctx_pop();
}

void profile_begin(int cls, hipStream_t s)
{
    hipEvent_t a = get_event();
    if (a && hipEventRecord(a, s) != hipSuccess)
        g_failed = true;
    g_open.push_back(Open{cls, a});
}

void profile_end(hipStream_t s)
{
    hipEvent_t e = get_event();
    if (e && hipEventRecord(e, s) != hipSuccess)
        g_failed = true;
    if (g_open.empty())
        return;
    const Open o = g_open.back();
    g_open.pop_back();
    if (o.a && e)
        g_spans.push_back(Span{o.cls, o.a, e});
}

} // namespace sgc

using namespace sgc;

extern "C" {

sgc_status sgc_profile_enable(int32_t on)
{
    for (auto &sp : g_spans) {
        g_pool.push_back(sp.a);
        g_pool.push_back(sp.b);
    }
    g_spans.clear();
    g_failed = false;
    g_profile_on = on != 0;
    return SGC_OK;
}

sgc_status sgc_profile_read(sgc_profile *out)
{
    if (!out)
        return SGC_ERR_NULL;
    for (int c = 0; c < SGC_PROFILE_CLASSES; ++c) {
        out->ms[c] = 0.0;
        out->launches[c] = 0;
    }
    sgc_status st = g_failed ? SGC_ERR_DEVICE : SGC_OK;
    for (auto &sp : g_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(sp.b) != hipSuccess || hipEventElapsedTime(&ms, sp.a, sp.b) != hipSuccess)
            st = SGC_ERR_DEVICE;
        out->ms[sp.cls] += (double)ms;
        out->launches[sp.cls] += 1;
        g_pool.push_back(sp.a);
        g_pool.push_back(sp.b);
    }
    g_spans.clear();
    return st;
}

} // extern "C"
