// Library-level entry points of the C ABI that belong to no single stage: version, error text,
// scratch sizing, and the event-timing hook used by the benchmark.
#include "common.hpp"

namespace ddt {
size_t attn_ws_upper(int batch, int T, int Hq, int Hkv, int D);

Profiler &profiler()
{
    static Profiler p;
    return p;
}

static void profiler_destroy(Profiler &p)
{
    for (int k = 0; k < DDTREE_KERNEL_COUNT; ++k) {
        if (p.start[k]) {
            for (int i = 0; i < p.capacity; ++i) {
                (void)hipEventDestroy(p.start[k][i]);
                (void)hipEventDestroy(p.stop[k][i]);
            }
            delete[] p.start[k];
            delete[] p.stop[k];
            p.start[k] = p.stop[k] = nullptr;
        }
        p.count[k] = p.seen[k] = 0;
    }
    p.mask = 0;
    p.capacity = 0;
    p.every = 1;
}
}  // namespace ddt

extern "C" int ddtree_version(void) { return 100; }

extern "C" const char *ddtree_error_string(int code)
{
    switch (code) {
    case DDTREE_OK: return "ok";
    case DDTREE_ERR_ARG: return "bad argument (null pointer, shape, size or dtype)";
    case DDTREE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DDTREE_ERR_HIP: return "HIP runtime error at launch";
    default: return "unknown error code";
    }
}

extern "C" size_t ddtree_workspace_bytes(int batch, int B, int V, int N, int Hq, int Hkv, int D,
                                         int max_sum_L)
{
    using namespace ddt;
    (void)max_sum_L;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || B < 1 || B > DDTREE_MAX_B || V < 1 || N < 1 ||
        N > DDTREE_MAX_N || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 8 || D > 256 || D % 8 != 0)
        return 0;
    const int K = N < V ? N : V;
    const int T = N + 1;
    TopkPlan tp = topk_plan(batch, B, V, K);
    if (!tp.ok) return 0;
    size_t need = tp.bytes;
    const size_t a = attn_ws_upper(batch, T, Hq, Hkv, D);
    if (a > need) need = a;
    const size_t c = accept_plan(batch, T, V).bytes;
    if (c > need) need = c;
    return need < 256 ? 256 : need;
}

extern "C" size_t ddtree_verify_attn_workspace_bytes(int batch, int T, int Hq, int Hkv, int D, int dtype,
                                                    long long sum_L)
{
    using namespace ddt;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 1 || T > DDTREE_MAX_N + 1 || Hq < 1 || Hkv < 1 ||
        Hq % Hkv != 0 || D < 8 || D > 256 || D % 8 != 0 || sum_L < 0)
        return 0;
    return attn_plan(batch, T, Hq, Hkv, D, sum_L, dtype).bytes;
}

extern "C" int ddtree_profile_enable(unsigned kernel_mask, int capacity)
{
    return ddtree_profile_enable_every(kernel_mask, capacity, 1);
}

extern "C" int ddtree_profile_enable_every(unsigned kernel_mask, int capacity, int every)
{
    using namespace ddt;
    Profiler &p = profiler();
    profiler_destroy(p);
    if (kernel_mask == 0) return DDTREE_OK;
    if (capacity < 1 || capacity > (1 << 20) || (kernel_mask >> DDTREE_KERNEL_COUNT) != 0 || every < 1)
        return DDTREE_ERR_ARG;
    p.capacity = capacity;
    p.every = every;
    for (int k = 0; k < DDTREE_KERNEL_COUNT; ++k) {
        if (!(kernel_mask & (1u << k))) continue;
        p.start[k] = new hipEvent_t[capacity];
        p.stop[k] = new hipEvent_t[capacity];
        for (int i = 0; i < capacity; ++i)
            if (hipEventCreate(&p.start[k][i]) != hipSuccess || hipEventCreate(&p.stop[k][i]) != hipSuccess)
                return DDTREE_ERR_HIP;
    }
    p.mask = kernel_mask;
    return DDTREE_OK;
}

extern "C" int ddtree_profile_reset(void)
{
    ddt::Profiler &p = ddt::profiler();
    for (int k = 0; k < DDTREE_KERNEL_COUNT; ++k) p.count[k] = p.seen[k] = 0;
    return DDTREE_OK;
}

extern "C" int ddtree_profile_read(int kernel_id, float *ms_out, int max_records)
{
    ddt::Profiler &p = ddt::profiler();
    if (kernel_id < 0 || kernel_id >= DDTREE_KERNEL_COUNT || !ms_out || max_records < 0)
        return DDTREE_ERR_ARG;
    if (!(p.mask & (1u << kernel_id))) return 0;
    const int n = p.count[kernel_id] < max_records ? p.count[kernel_id] : max_records;
    for (int i = 0; i < n; ++i)
        if (hipEventElapsedTime(&ms_out[i], p.start[kernel_id][i], p.stop[kernel_id][i]) != hipSuccess)
            return DDTREE_ERR_HIP;
    return n;
}
