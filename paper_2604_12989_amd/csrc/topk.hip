// Per-position log-softmax and exact top-K over the vocabulary (paper Section 4.3: the
// ordering q_i^(1) >= q_i^(2) >= ... of each position's distribution; Lemma 1: K ranks suffice).
//
// Two kernels.
//   chunk kernel  one workgroup per (row, vocabulary chunk): the chunk is read once from HBM
//                 (coalesced 16-byte loads) into LDS as order-preserving integer keys; the
//                 workgroup reduces max and sum-of-exp (fp64) for the row's log-sum-exp and
//                 selects the chunk's exact top-kc by a multi-level radix select held in LDS.
//   merge kernel  one workgroup per row: merges the chunk statistics into the fp64
//                 log-sum-exp, selects the row's top-K among chunks*kc candidates, ranks them
//                 (key descending, token id ascending) and writes tokens and log-probabilities.
//
// Every candidate is the 64-bit composite (key << 32) | ~token_id, so all composites of a row
// are distinct and "larger composite" is exactly "larger logit, or equal logit and smaller id".
#include "common.hpp"

namespace ddt {

constexpr int kListCap = 1024;  // a radix bin this small is finished by rank counting
constexpr int kHistBins = 4096;

TopkPlan topk_plan(int batch, int B, int V, int K)
{
    TopkPlan p{};
    p.ok = false;
    if (batch < 1 || B < 1 || V < 1 || K < 1 || K > V) return p;
    long long rows = (long long)batch * B;
    int c_min = (V + kTopkChunkMax - 1) / kTopkChunkMax;
    int want = (int)((256 + rows - 1) / rows);
    int c_cap = V / 1024 > 0 ? V / 1024 : 1;  // keep chunks at least 1024 long
    int C = want < c_cap ? want : c_cap;
    if (C < c_min) C = c_min;
    for (;;) {
        int len = (V + C - 1) / C;
        len = (len + 3) / 4 * 4;
        int real_c = (V + len - 1) / len;
        int kc = K < len ? K : len;
        if ((long long)real_c * kc <= kTopkMergeMaxCand) {
            p.chunks = real_c;
            p.chunk_len = len;
            p.kc = kc;
            break;
        }
        if (C == c_min) return p;
        --C;
    }
    p.cand_off = 0;
    size_t cand_bytes = (size_t)rows * p.chunks * p.kc * sizeof(uint64_t);
    p.stat_off = align_up(cand_bytes, 256);
    p.bytes = align_up(p.stat_off + (size_t)rows * p.chunks * 16, 256);
    p.ok = true;
    return p;
}

// ------------------------------------------------------------------------------------------
// Block-wide helpers.  NT = threads per workgroup (multiple of 64).
// ------------------------------------------------------------------------------------------

// Exclusive prefix sum of v over the workgroup's threads; *total receives the sum.
template <int NT>
__device__ int block_exclusive_scan(int v, int *s_wave /*[NT/64 + 1]*/, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int w = 0; w < NT / 64; ++w) {
            int t = s_wave[w];
            s_wave[w] = acc;
            acc += t;
        }
        s_wave[NT / 64] = acc;
    }
    __syncthreads();
    int res = s_wave[wave] + incl - v;
    *total = s_wave[NT / 64];
    __syncthreads();
    return res;
}

struct SelectScratch {
    uint32_t *hist;    // [kHistBins]
    uint64_t *list;    // [kListCap]
    int *s_wave;       // [NT/64 + 1]
    int *s_misc;       // [8]
    uint64_t *s_thr;   // [1]
};

// Returns thr such that exactly k of the n distinct composites get(i) are >= thr (1 <= k <= n).
// Radix select from the most significant bits down: 12, 12, 8 bits of the key, then 12, 12, 8
// bits of the inverted id.  A level ends the search when its threshold bin holds exactly the
// number still wanted, or few enough elements to rank them directly.
template <int NT, class Get>
__device__ uint64_t block_select_threshold(Get get, int n, int k, SelectScratch s)
{
    const int tid = threadIdx.x;
    uint64_t pmask = 0, pval = 0;
    const int shifts[6] = {52, 40, 32, 20, 8, 0};
    const int widths[6] = {12, 12, 8, 12, 12, 8};
    for (int level = 0; level < 6; ++level) {
        const int shift = shifts[level];
        const int nb = 1 << widths[level];
        for (int i = tid; i < nb; i += NT) s.hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += NT) {
            uint64_t c = get(i);
            if ((c & pmask) == pval) atomicAdd(&s.hist[(uint32_t)(c >> shift) & (nb - 1)], 1u);
        }
        __syncthreads();
        // locate the bin holding the k-th largest.  Thread t owns the `per` bins that end at
        // ahi = nb-1 - t*per, so thread 0 owns the highest bins and an exclusive scan over the
        // threads counts the elements in all higher bins.
        const int per = nb >= NT ? nb / NT : 1;
        const int ahi = nb - 1 - tid * per;
        int mine = 0;
        if (ahi >= 0)
            for (int j = 0; j < per; ++j) mine += (int)s.hist[ahi - j];
        int total;
        int above = block_exclusive_scan<NT>(mine, s.s_wave, &total);
        if (ahi >= 0 && above < k && k <= above + mine) {
            int acc = above;
            for (int j = 0; j < per; ++j) {
                int h = (int)s.hist[ahi - j];
                if (acc + h >= k) {
                    s.s_misc[1] = ahi - j;  // bin
                    s.s_misc[2] = acc;      // elements in higher bins
                    s.s_misc[3] = h;        // elements in the bin
                    break;
                }
                acc += h;
            }
        }
        __syncthreads();
        const int bin = s.s_misc[1], above_cnt = s.s_misc[2], in_bin = s.s_misc[3];
        __syncthreads();
        k -= above_cnt;
        pval |= (uint64_t)bin << shift;
        pmask |= (uint64_t)(nb - 1) << shift;
        if (in_bin == k) return pval;  // the whole bin is wanted: pval's low bits are zero
        if (in_bin <= kListCap) {
            if (tid == 0) s.s_misc[4] = 0;
            __syncthreads();
            for (int i = tid; i < n; i += NT) {
                uint64_t c = get(i);
                if ((c & pmask) == pval) s.list[atomicAdd(&s.s_misc[4], 1)] = c;
            }
            __syncthreads();
            for (int e = tid; e < in_bin; e += NT) {
                const uint64_t c = s.list[e];
                int greater = 0;
                for (int j = 0; j < in_bin; ++j) greater += s.list[j] > c ? 1 : 0;
                if (greater == k - 1) *s.s_thr = c;
            }
            __syncthreads();
            uint64_t thr = *s.s_thr;
            __syncthreads();
            return thr;
        }
    }
    return pval;  // all 64 bits fixed: a single element
}

// ------------------------------------------------------------------------------------------
// Chunk kernel
// ------------------------------------------------------------------------------------------
constexpr int kChunkThreads = 256;

__global__ __launch_bounds__(kChunkThreads) void topk_chunk_kernel(
    const float *__restrict__ logits, int V, int K, int chunk_len, int kc, int chunks,
    uint64_t *__restrict__ cand, double *__restrict__ stat)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *s_key = reinterpret_cast<uint32_t *>(smem);
    uint32_t *hist = s_key + chunk_len;
    uint64_t *list = reinterpret_cast<uint64_t *>(hist + kHistBins);
    __shared__ int s_wave[kChunkThreads / 64 + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ float s_fmax[kChunkThreads / 64];
    __shared__ double s_dsum[kChunkThreads];

    const int tid = threadIdx.x;
    const int c = blockIdx.x;
    const size_t row = (size_t)blockIdx.z * gridDim.y + blockIdx.y;
    const int start = c * chunk_len;
    const int n = min(chunk_len, V - start);
    const float *p = logits + row * (size_t)V + start;

    // ---- load the chunk: scalar head up to 16-byte alignment, float4 body, scalar tail ----
    float tmax = -INFINITY;
    int head = (int)((4 - ((reinterpret_cast<uintptr_t>(p) >> 2) & 3)) & 3);
    if (head > n) head = n;
    if (tid < head) {
        float x = p[tid];
        tmax = fmaxf(tmax, x);
        s_key[tid] = float_key(x);
    }
    const int nvec = (n - head) >> 2;
    const float4 *pv = reinterpret_cast<const float4 *>(p + head);
    // all of a thread's loads are issued before the first one is consumed (at most
    // kTopkChunkMax / 4 / kChunkThreads = 12 per thread): one HBM round trip instead of twelve
    constexpr int kMaxVec = kTopkChunkMax / 4 / kChunkThreads;
    float4 xv[kMaxVec];
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
        const int j = tid + u * kChunkThreads;
        xv[u] = j < nvec ? pv[j] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
        const int j = tid + u * kChunkThreads;
        if (j < nvec) {
            const float4 x = xv[u];
            tmax = fmaxf(fmaxf(tmax, x.x), fmaxf(x.y, fmaxf(x.z, x.w)));
            const int o = head + 4 * j;
            s_key[o + 0] = float_key(x.x);
            s_key[o + 1] = float_key(x.y);
            s_key[o + 2] = float_key(x.z);
            s_key[o + 3] = float_key(x.w);
        }
    }
    const int tail0 = head + 4 * nvec;
    if (tid < n - tail0) {
        float x = p[tail0 + tid];
        tmax = fmaxf(tmax, x);
        s_key[tail0 + tid] = float_key(x);
    }
    // ---- chunk max ----
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, d, 64));
    if ((tid & 63) == 0) s_fmax[tid >> 6] = tmax;
    __syncthreads();
    float cmax = s_fmax[0];
#pragma unroll
    for (int w = 1; w < kChunkThreads / 64; ++w) cmax = fmaxf(cmax, s_fmax[w]);
    // ---- sum of exp(x - cmax) in fp64, fixed reduction order ----
    double acc = 0.0;
    for (int i = tid; i < n; i += kChunkThreads)
        acc += exp((double)key_float(s_key[i]) - (double)cmax);
    s_dsum[tid] = acc;
    __syncthreads();
    for (int d = kChunkThreads / 2; d >= 1; d >>= 1) {
        if (tid < d) s_dsum[tid] += s_dsum[tid + d];
        __syncthreads();
    }
    if (tid == 0) {
        double *st = stat + (row * chunks + c) * 2;
        st[0] = (double)cmax;
        st[1] = s_dsum[0];
    }
    // ---- exact top-kc of the chunk ----
    uint64_t *out = cand + (row * chunks + c) * (size_t)kc;
    const uint32_t base_id = (uint32_t)start;
    auto get = [&](int i) -> uint64_t {
        return ((uint64_t)s_key[i] << 32) | (uint64_t)(uint32_t)(~(base_id + (uint32_t)i));
    };
    if (n <= kc) {
        for (int i = tid; i < kc; i += kChunkThreads) out[i] = i < n ? get(i) : 0ull;
        return;
    }
    SelectScratch sc{hist, list, s_wave, s_misc, &s_thr};
    const uint64_t thr = block_select_threshold<kChunkThreads>(get, n, kc, sc);
    if (tid == 0) s_misc[5] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kChunkThreads) {
        uint64_t cc = get(i);
        if (cc >= thr) {
            int pos = atomicAdd(&s_misc[5], 1);
            if (pos < kc) out[pos] = cc;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Merge kernel
// ------------------------------------------------------------------------------------------
constexpr int kMergeThreads = 1024;

__global__ __launch_bounds__(kMergeThreads) void topk_merge_kernel(
    const uint64_t *__restrict__ cand, const double *__restrict__ stat, int K, int kc, int chunks,
    int32_t *__restrict__ topk_tok, float *__restrict__ topk_lp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int n = chunks * kc;
    uint64_t *s_cand = reinterpret_cast<uint64_t *>(smem);
    uint64_t *s_sel = s_cand + n;                       // [K]
    uint64_t *list = s_sel + K;                         // [kListCap]
    uint32_t *hist = reinterpret_cast<uint32_t *>(list + kListCap);  // [kHistBins]
    int *s_rank = reinterpret_cast<int *>(hist + kHistBins);         // [K]
    __shared__ int s_wave[kMergeThreads / 64 + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ double s_lse;

    const int tid = threadIdx.x;
    const size_t row = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t *in = cand + row * (size_t)n;
    {
        // candidates of the row (at most kTopkMergeMaxCand): loads issued back to back
        constexpr int kMaxLd = (kTopkMergeMaxCand + kMergeThreads - 1) / kMergeThreads;
        uint64_t cv[kMaxLd];
#pragma unroll
        for (int u = 0; u < kMaxLd; ++u) {
            const int i = tid + u * kMergeThreads;
            cv[u] = i < n ? in[i] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < kMaxLd; ++u) {
            const int i = tid + u * kMergeThreads;
            if (i < n) s_cand[i] = cv[u];
        }
    }
    for (int i = tid; i < K; i += kMergeThreads) s_rank[i] = 0;
    if (tid == 0) {
        const double *st = stat + row * (size_t)chunks * 2;
        double m = st[0];
        for (int c = 1; c < chunks; ++c) m = fmax(m, st[2 * c]);
        double S = 0.0;
        for (int c = 0; c < chunks; ++c) S += st[2 * c + 1] * exp(st[2 * c] - m);
        s_lse = m + log(S);
        s_misc[5] = 0;
    }
    __syncthreads();
    auto get = [&](int i) -> uint64_t { return s_cand[i]; };
    SelectScratch sc{hist, list, s_wave, s_misc, &s_thr};
    uint64_t thr = 0;
    if (n > K) thr = block_select_threshold<kMergeThreads>(get, n, K, sc);
    // n == K can only happen with a single chunk holding exactly K elements: keep them all
    for (int i = tid; i < n; i += kMergeThreads) {
        uint64_t c = s_cand[i];
        if (c >= thr && c != 0ull) {
            int pos = atomicAdd(&s_misc[5], 1);
            if (pos < K) s_sel[pos] = c;
        }
    }
    __syncthreads();
    // rank by counting: K*K comparisons spread over the workgroup
    const int parts = kMergeThreads / K > 0 ? kMergeThreads / K : 1;
    for (int idx = tid; idx < K * parts; idx += kMergeThreads) {
        const int e = idx % K, part = idx / K;
        const int j0 = (int)((long long)K * part / parts), j1 = (int)((long long)K * (part + 1) / parts);
        const uint64_t c = s_sel[e];
        int greater = 0;
        for (int j = j0; j < j1; ++j) greater += s_sel[j] > c ? 1 : 0;
        atomicAdd(&s_rank[e], greater);
    }
    __syncthreads();
    const double lse = s_lse;
    for (int e = tid; e < K; e += kMergeThreads) {
        const uint64_t c = s_sel[e];
        const int r = s_rank[e];
        topk_tok[row * (size_t)K + r] = (int32_t)(~(uint32_t)c);
        topk_lp[row * (size_t)K + r] = (float)((double)key_float((uint32_t)(c >> 32)) - lse);
    }
}

}  // namespace ddt

extern "C" int ddtree_topk(const float *logits, int batch, int B, int V, int K, int32_t *topk_tok,
                           float *topk_lp, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace ddt;
    if (!logits || !topk_tok || !topk_lp) return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || B < 1 || B > DDTREE_MAX_B || V < 1 || K < 1 ||
        K > V || K > DDTREE_MAX_N)
        return DDTREE_ERR_ARG;
    TopkPlan p = topk_plan(batch, B, V, K);
    if (!p.ok) return DDTREE_ERR_ARG;
    if (!ws_ok(workspace, workspace_bytes, p.bytes)) return DDTREE_ERR_WORKSPACE;
    uint64_t *cand = reinterpret_cast<uint64_t *>(static_cast<char *>(workspace) + p.cand_off);
    double *stat = reinterpret_cast<double *>(static_cast<char *>(workspace) + p.stat_off);

    static bool attr_set = false;
    const size_t lds_chunk = (size_t)p.chunk_len * 4 + kHistBins * 4 + kListCap * 8;
    const size_t lds_merge =
        (size_t)p.chunks * p.kc * 8 + (size_t)K * 8 + kListCap * 8 + kHistBins * 4 + (size_t)K * 4;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(topk_chunk_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(topk_merge_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) != hipSuccess)
            return DDTREE_ERR_HIP;
        attr_set = true;
    }
    hipStream_t st = as_stream(stream);
    DDT_LAUNCH(DDTREE_KERNEL_TOPK_CHUNK, st, topk_chunk_kernel, dim3(p.chunks, B, batch), dim3(kChunkThreads), lds_chunk, st,
                       logits, V, K, p.chunk_len, p.kc, p.chunks, cand, stat);
    DDT_LAUNCH(DDTREE_KERNEL_TOPK_MERGE, st, topk_merge_kernel, dim3(B, batch), dim3(kMergeThreads), lds_merge, st, cand,
                       stat, K, p.kc, p.chunks, topk_tok, topk_lp);
    return launch_status();
}
