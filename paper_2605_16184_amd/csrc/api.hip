// Version, status strings and option defaults.
#include <vector>

#include "common.h"
#include "gemm.h"

extern "C" int asteria_version(void) { return 100; }

extern "C" const char *asteria_status_string(asteria_status s)
{
    switch (s) {
        case ASTERIA_OK: return "ok";
        case ASTERIA_INVALID_ARG: return "invalid argument";
        case ASTERIA_UNSUPPORTED: return "unsupported";
        case ASTERIA_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ASTERIA_HIP_ERROR: return "HIP runtime error";
        case ASTERIA_EXCEEDS_STATIC_SCRATCH: return "a factor exceeds the static scratch array";
    }
    return "unknown status";
}

extern "C" void asteria_root_opts_default(asteria_root_opts *o)
{
    if (!o) return;
    o->max_iters = 40;
    o->fp64_iters = -1;
    o->power_iters = 256;
    o->schedule = 1;
    o->stop_resid = 1e-2f;
    o->power_tol = 1e-3f;
    o->lambda_margin = 0.01f;
    o->lowp_from = -1;
    o->int8_slices = -1;
}

// ---- measurement aid: HIP events around every grouped-GEMM launch ----------------------------
namespace {
struct ProfileState {
    bool on = false;
    int cap = 0;
    bool open = false;            // profile_begin pushed a pair that profile_end has not closed yet
    std::vector<hipEvent_t> ev;   // 2 per recorded launch
    std::vector<int> kind;
} g_prof;
}  // namespace

static __device__ double g_i8_flops[3];
static double *g_i8_flops_ptr[asteria::MAX_DEVICES];   // device address of g_i8_flops, per device

static double *i8_flops_ptr()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= asteria::MAX_DEVICES) return nullptr;
    if (!g_i8_flops_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_i8_flops)) != hipSuccess) return nullptr;
        g_i8_flops_ptr[dev] = reinterpret_cast<double *>(p);
    }
    return g_i8_flops_ptr[dev];
}

double *asteria::profile_i8_counters() { return g_prof.on ? i8_flops_ptr() : nullptr; }

void asteria::profile_begin(int kind, hipStream_t stream)
{
    if (!g_prof.on || (int)g_prof.kind.size() >= g_prof.cap) return;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    g_prof.ev.push_back(a);
    g_prof.ev.push_back(b);
    g_prof.kind.push_back(kind);
    g_prof.open = true;
    (void)hipEventRecord(a, stream);
}

void asteria::profile_end(hipStream_t stream)
{
    // a launch skipped by the cap opened nothing: only the launch whose begin pushed a pair is closed
    if (!g_prof.on || !g_prof.open) return;
    g_prof.open = false;
    (void)hipEventRecord(g_prof.ev.back(), stream);
}

extern "C" asteria_status asteria_profile_enable(int max_launches)
{
    if (max_launches <= 0 || g_prof.on) return ASTERIA_INVALID_ARG;
    if (double *c = i8_flops_ptr()) {
        if (hipMemset(c, 0, 3 * sizeof(double)) != hipSuccess) return ASTERIA_HIP_ERROR;   // synchronous: measurement aid
    }
    g_prof.on = true;
    g_prof.cap = max_launches;
    g_prof.open = false;
    g_prof.ev.clear();
    g_prof.kind.clear();
    return ASTERIA_OK;
}

extern "C" int asteria_profile_collect(float *ms, int32_t *kind, int cap)
{
    if (!g_prof.on) return -1;
    g_prof.on = false;
    const int n = (int)g_prof.kind.size();
    int out = 0;
    for (int i = 0; i < n; ++i) {
        float t = 0.0f;
        (void)hipEventSynchronize(g_prof.ev[2 * i + 1]);
        const bool ok = hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) == hipSuccess;
        if (ok && out < cap && ms && kind) { ms[out] = t; kind[out] = g_prof.kind[i]; ++out; }
        (void)hipEventDestroy(g_prof.ev[2 * i]);
        (void)hipEventDestroy(g_prof.ev[2 * i + 1]);
    }
    g_prof.ev.clear();
    g_prof.kind.clear();
    return out;
}

extern "C" asteria_status asteria_profile_i8_flops(double *out3)
{
    if (!out3) return ASTERIA_INVALID_ARG;
    double *c = i8_flops_ptr();
    if (!c) return ASTERIA_HIP_ERROR;
    ASTERIA_HIP_TRY(hipMemcpy(out3, c, 3 * sizeof(double), hipMemcpyDeviceToHost));   // waits for the device
    return ASTERIA_OK;
}
