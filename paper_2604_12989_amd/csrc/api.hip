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

// Host-side self-check (no GPU): the attention kernel's launch arithmetic (attn.hip) and the
// invariants of the top-K and accept plans that their kernels index by.
namespace ddt {
int attn_selftest_host();
}
extern "C" int ddtree_selftest_host(void)
{
    using namespace ddt;
    if (const int rc = attn_selftest_host()) return rc;
    // top-K: chunks tile the row, stay within what a chunk workgroup holds, and their candidates
    // fit the merge workgroup; a plan that cannot be made says so
    const int Vs[] = {1, 2, 7, 64, 1000, 1024, 4096, 12288, 12289, 20000, 50001, 100000, 151936, 172032, 200003, 344064, 688128, 1000000};
    const int Ks[] = {1, 2, 16, 64, 255, 256, 257, 512, 1024};
    const int rows_[] = {1, 2, 3, 8, 16, 17, 64, 127, 128, 1024};
    for (int V : Vs)
        for (int K : Ks)
            for (int rows : rows_) {
                if (K > V) continue;
                const TopkPlan p = topk_plan(1, rows, V, K);
                if (!p.ok) {
                    // only where the candidates of a row cannot fit the merge workgroup
                    const long long c_min = (V + kTopkChunkMax - 1) / kTopkChunkMax;
                    const long long len = ((V + c_min - 1) / c_min + 3) / 4 * 4;
                    if (c_min * (K < len ? K : len) <= kTopkMergeMaxCand) return 10001;
                    continue;
                }
                if (p.row_kernel) {
                    if (rows < kTopkRowKernelMinRows) return 10002;
                    continue;
                }
                if (rows >= kTopkRowKernelMinRows) return 10003;
                if (p.chunk_len % 4 != 0 || p.chunk_len < 1 || p.chunk_len > kTopkChunkMax) return 10004;
                if ((long long)(p.chunks - 1) * p.chunk_len >= V || (long long)p.chunks * p.chunk_len < V) return 10005;
                if (p.kc != (K < p.chunk_len ? K : p.chunk_len)) return 10006;
                if ((long long)p.chunks * p.kc > kTopkMergeMaxCand) return 10007;
                // K candidates exist: the first chunk is whole unless it is the only one
                const int first_len = p.chunks > 1 ? p.chunk_len : V;
                if (p.kc < K && p.kc != p.chunk_len) return 10008;
                if (p.kc == K && first_len < K) return 10009;
                if (p.stat_off < (size_t)rows * p.chunks * p.kc * 8 || p.bytes < p.stat_off + (size_t)rows * p.chunks * 16) return 10010;
                if ((p.stat_off & 255u) || (p.bytes & 255u)) return 10011;
            }
    // accept: segments tile the row in multiples of four, scratch holds one partial per segment
    for (int V : Vs)
        for (int T : {2, 17, 65, 257, 513, 1025})
            for (int batch : {1, 16, 64})
                for (int sampled = 0; sampled < 2; ++sampled) {
                    const AcceptPlan p = accept_plan(batch, T, V, sampled != 0);
                    if (p.seg_len % 4 != 0 || p.seg_len < 1 || p.splits < 1) return 10021;
                    if ((long long)(p.splits - 1) * p.seg_len >= V || (long long)p.splits * p.seg_len < V) return 10022;
                    if (p.bytes < (size_t)batch * T * p.splits * 8 || (p.bytes & 255u)) return 10023;
                }
    return 0;
}
