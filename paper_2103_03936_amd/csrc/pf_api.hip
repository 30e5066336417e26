// Status strings, error bookkeeping, per-kernel timing and the small utility kernels.
#include <string.h>

#include <vector>

#include "pf_gemm.h"

namespace pf {

static thread_local int g_last_hip_error = 0;

int set_hip_error(hipError_t e)
{
    g_last_hip_error = (int)e;
    return PF_ERR_LAUNCH;
}

// ------------------------------------------------------------------ timing
struct TimingRecord {
    const char *name;
    hipEvent_t start, stop;
};
struct TimingTotal {
    const char *name;
    int64_t launches;
    double total_ms;
};
static bool g_timing_on = false;
static std::vector<TimingRecord> g_pending;
static std::vector<TimingTotal> g_totals;

TimingScope::TimingScope(const char *name, hipStream_t s) : slot(-1), stream(s)
{
    if (!g_timing_on) return;
    TimingRecord r;
    r.name = name;
    if (hipEventCreate(&r.start) != hipSuccess) return;
    if (hipEventCreate(&r.stop) != hipSuccess) {
        (void)hipEventDestroy(r.start);
        return;
    }
    (void)hipEventRecord(r.start, s);
    g_pending.push_back(r);
    slot = (int)g_pending.size() - 1;
}

TimingScope::~TimingScope()
{
    if (slot >= 0) (void)hipEventRecord(g_pending[slot].stop, stream);
}

__global__ void splitk_reduce_kernel(const float *partial, float *out, i64 count, int ksplit, int accumulate)
{
    const i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float acc = 0.f;
    int s = 0;
    for (; s + 8 <= ksplit; s += 8) { // eight loads in flight, added in split order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(i64)(s + u) * count + i];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; s < ksplit; ++s) acc += partial[(i64)s * count + i];
    out[i] = accumulate ? (out[i] + acc) : acc;
}

__global__ void zero_f32_kernel(float *out, i64 count)
{
    const i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = 0.f;
}

int launch_splitk_reduce(hipStream_t stream, const float *partial, float *out, i64 count, int ksplit, int accumulate)
{
    int status = PF_OK;
    if (count <= 0) return status;
    dim3 grid((unsigned)((count + 255) / 256));
    PF_LAUNCH(status, "splitk_reduce", splitk_reduce_kernel, grid, dim3(256), stream, partial, out, count, ksplit,
              accumulate);
    return status;
}

int launch_zero_f32(hipStream_t stream, float *out, i64 count)
{
    int status = PF_OK;
    if (count <= 0 || !out) return status;
    dim3 grid((unsigned)((count + 255) / 256));
    PF_LAUNCH(status, "zero_f32", zero_f32_kernel, grid, dim3(256), stream, out, count);
    return status;
}

} // namespace pf

extern "C" {

const char *pf_status_string(int status)
{
    switch (status) {
    case PF_OK: return "ok";
    case PF_ERR_NULL: return "a required pointer is NULL";
    case PF_ERR_SHAPE: return "a dimension is out of range";
    case PF_ERR_UNSUPPORTED: return "dtype, layout or option not supported";
    case PF_ERR_WORKSPACE: return "workspace missing or too small";
    case PF_ERR_LAUNCH: return "HIP reported an error at launch";
    default: return "unknown status";
    }
}

int pf_last_hip_error(void) { return pf::g_last_hip_error; }

int pf_version(void) { return 1; }

void pf_timing_enable(int on) { pf::g_timing_on = on != 0; }

int pf_timing_collect(void)
{
    for (auto &r : pf::g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            bool found = false;
            for (auto &t : pf::g_totals)
                if (t.name == r.name || strcmp(t.name, r.name) == 0) {
                    t.launches += 1;
                    t.total_ms += ms;
                    found = true;
                    break;
                }
            if (!found) pf::g_totals.push_back({r.name, 1, (double)ms});
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    pf::g_pending.clear();
    return (int)pf::g_totals.size();
}

int pf_timing_entry(int i, const char **name, int64_t *launches, double *total_ms)
{
    if (i < 0 || i >= (int)pf::g_totals.size()) return PF_ERR_SHAPE;
    if (name) *name = pf::g_totals[i].name;
    if (launches) *launches = pf::g_totals[i].launches;
    if (total_ms) *total_ms = pf::g_totals[i].total_ms;
    return PF_OK;
}

void pf_timing_reset(void)
{
    pf_timing_collect();
    pf::g_totals.clear();
}

} // extern "C"
