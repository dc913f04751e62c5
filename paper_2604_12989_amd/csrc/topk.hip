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

// Ranks the m distinct composites in list[] (descending; m <= kCandCap) and calls
// emit(rank, composite) once per element: all-pairs counting, used on the rare tie-heavy path.
template <int NT, class Emit>
__device__ void block_rank_emit(const uint64_t *list, int m, Emit emit)
{
    for (int e = threadIdx.x; e < m; e += NT) {
        const uint64_t c = list[e];
        int g = 0;
        for (int j = 0; j < m; ++j) g += list[j] > c ? 1 : 0;
        emit(g, c);
    }
}

// Sum over the wave's lanes in a fixed butterfly order.
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

constexpr int kCandCap = 2048;  // elements placed in LDS for exact ranking
constexpr int kBuckets = 1024;

struct BucketScratch {
    uint32_t *cnt;     // [kBuckets]
    int *start;        // [kBuckets]
    uint64_t *sorted;  // [kCandCap]
    int *s_wave;       // [NT/64 + 1]
    int *s_misc;       // [8]
};

// Exact descending ranks, for ranks < want, of the workgroup's composites with key in
// [lo_key, hi_key]; each thread brings NS composites in registers (0 = empty slot, and slots
// with key < lo_key are ignored).  The key range is cut into kBuckets equal buckets, bucket 0
// the highest: an element's rank is the population of the buckets above its own plus the number
// of larger elements inside its bucket, which is found by placing the buckets that can reach
// rank < want side by side in LDS.  Returns false, having emitted nothing, if those buckets
// hold more than kCandCap elements (heavy ties); *total_out = number of elements considered.
template <int NT, int NS, class Emit>
__device__ bool block_bucket_rank(const uint64_t (&c)[NS], uint32_t lo_key, uint32_t hi_key, int want,
                                  BucketScratch s, int *total_out, Emit emit)
{
    static_assert(NT == kBuckets, "one bucket per thread");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    s.cnt[tid] = 0;
    if (tid == 0) {
        s.s_misc[0] = -1;
        s.s_misc[1] = kBuckets - 1;
    }
    __syncthreads();
    const float inv = (float)kBuckets / ((float)(hi_key - lo_key) + 1.0f);
    auto bucket_of = [&](uint32_t key) {
        const int b = (int)((float)(key - lo_key) * inv);
        return kBuckets - 1 - min(b, kBuckets - 1);
    };
    // bucket of every slot first, then the counting atomics back to back: their returned
    // positions are not needed before the scan below
    int bkt[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const uint32_t key = (uint32_t)(c[i] >> 32);
        bkt[i] = (c[i] != 0ull && key >= lo_key) ? bucket_of(key) : -1;
    }
    uint32_t pos[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        pos[i] = 0;
        if (bkt[i] >= 0) pos[i] = atomicAdd(&s.cnt[bkt[i]], 1u);
    }
    __syncthreads();
    // exclusive scan of the bucket populations, bucket 0 (highest keys) first
    const int mine = (int)s.cnt[tid];
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    if (lane == 63) s.s_wave[wave] = incl;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const int v = s.s_wave[w];
        base += w < wave ? v : 0;
        total += v;
    }
    const int start = base + incl - mine;
    s.start[tid] = start;
    if (start < want && start + mine >= want) {  // the last bucket that can hold a rank < want
        s.s_misc[0] = start + mine;
        s.s_misc[1] = tid;
    }
    __syncthreads();
    const int placed = s.s_misc[0] < 0 ? total : s.s_misc[0];
    const int b_last = s.s_misc[1];
    *total_out = total;
    if (placed > kCandCap) return false;
    // place the elements of buckets 0..b_last side by side, bucket by bucket
    int st[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) st[i] = s.start[bkt[i] >= 0 ? bkt[i] : 0];
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if (bkt[i] >= 0 && bkt[i] <= b_last) s.sorted[st[i] + (int)pos[i]] = c[i];
    __syncthreads();
    // one thread per placed element: count the larger members of its bucket
    for (int e = tid; e < placed; e += NT) {
        const uint64_t ce = s.sorted[e];
        const int b = bucket_of((uint32_t)(ce >> 32));
        const int bs = s.start[b], nb = (int)s.cnt[b];
        int g = 0;
        for (int j = 0; j < nb; ++j) g += s.sorted[bs + j] > ce ? 1 : 0;
        if (bs + g < want) emit(bs + g, ce);
    }
    return true;
}

// ------------------------------------------------------------------------------------------
// Chunk kernel
// ------------------------------------------------------------------------------------------
constexpr int kChunkThreads = 1024;
constexpr int kChunkWaves = kChunkThreads / 64;
constexpr int kVecPerThread = kTopkChunkMax / 4 / kChunkThreads;
constexpr int kSlots = 4 * kVecPerThread + 2;  // float4 body + one head and one tail element
static_assert(kVecPerThread * 4 * kChunkThreads == kTopkChunkMax, "chunk must tile the workgroup");

// The chunk stays in registers (at most 14 elements per thread).  A lower bound t on the
// chunk's kc-th largest key comes almost free: cut every wave into g >= kc / waves groups of
// adjacent lanes, take each group's largest key, and let t be the smallest of all group
// maxima; the waves * g >= kc maxima are distinct elements that reach t.  Elements with
// key >= t (about one in seven for kc = 256) are ranked exactly by block_bucket_rank and the top
// kc written in descending order.  Chunks it cannot handle (heavy ties, or kc so large that
// the bound passes most of the chunk) take the radix select over keys staged in LDS.
__global__ __launch_bounds__(kChunkThreads) void topk_chunk_kernel(
    const float *__restrict__ logits, int V, int chunk_len, int kc, int chunks,
    uint64_t *__restrict__ cand, double *__restrict__ stat)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *s_key = reinterpret_cast<uint32_t *>(smem);  // [chunk_len], fallback only
    uint32_t *hist = s_key + chunk_len;                    // [kHistBins], fallback only
    __shared__ __align__(16) uint64_t s_list[kCandCap];
    __shared__ uint32_t s_cnt[kBuckets];
    __shared__ int s_start[kBuckets];
    __shared__ int s_wave[kChunkWaves + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ float s_fmax[kChunkWaves];
    __shared__ uint32_t s_bound[kChunkWaves];
    __shared__ double s_dsum[kChunkWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = blockIdx.x;
    const size_t row = (size_t)blockIdx.z * gridDim.y + blockIdx.y;
    const int start = c * chunk_len;
    const int n = min(chunk_len, V - start);
    const float *p = logits + row * (size_t)V + start;

    // ---- load: scalar head up to 16-byte alignment, float4 body, scalar tail; all of a
    //      thread's loads are in flight together ----
    int head = (int)((4 - ((reinterpret_cast<uintptr_t>(p) >> 2) & 3)) & 3);
    if (head > n) head = n;
    const int nvec = (n - head) >> 2;
    const int tail0 = head + 4 * nvec;
    const float4 *pv = reinterpret_cast<const float4 *>(p + head);
    float x[kSlots];
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
        const int j = tid + u * kChunkThreads;
        const float4 v = j < nvec ? pv[j] : make_float4(0.f, 0.f, 0.f, 0.f);
        x[4 * u + 0] = v.x;
        x[4 * u + 1] = v.y;
        x[4 * u + 2] = v.z;
        x[4 * u + 3] = v.w;
    }
    x[kSlots - 2] = tid < head ? p[tid] : 0.f;
    x[kSlots - 1] = tid < n - tail0 ? p[tail0 + tid] : 0.f;
    // element index of slot s within the chunk, -1 if the slot is empty
    auto slot_index = [&](int s) -> int {
        if (s < 4 * kVecPerThread) {
            const int j = tid + (s >> 2) * kChunkThreads;
            return j < nvec ? head + 4 * j + (s & 3) : -1;
        }
        if (s == kSlots - 2) return tid < head ? tid : -1;
        return tid < n - tail0 ? tail0 + tid : -1;
    };

    // ---- chunk max, and the bound t (for n <= kCandCap every element is ranked: t = the
    //      smallest key) ----
    const bool take_all = n <= kCandCap;
    float tmax = -INFINITY, tmin = INFINITY;
    bool any = false;
#pragma unroll
    for (int s = 0; s < kSlots; ++s)
        if (slot_index(s) >= 0) {
            tmax = fmaxf(tmax, x[s]);
            tmin = fminf(tmin, x[s]);
            any = true;
        }
    float wmax = tmax;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) wmax = fmaxf(wmax, __shfl_xor(wmax, d, 64));
    int group = 64;  // lanes per group: the largest power of two with waves * (64 / group) >= kc
    while (group > 1 && kChunkWaves * (64 / group) < kc) group >>= 1;
    uint32_t bound = take_all ? (any ? float_key(tmin) : ~0u) : (any ? float_key(tmax) : 0u);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)bound, d, 64);
        bound = (d < group && !take_all) ? max(bound, o) : min(bound, o);
    }
    if (lane == 0) {
        s_fmax[wave] = wmax;
        s_bound[wave] = bound;
    }
    __syncthreads();
    float cmax = s_fmax[0];
    uint32_t t = s_bound[0];
#pragma unroll
    for (int w = 1; w < kChunkWaves; ++w) {
        cmax = fmaxf(cmax, s_fmax[w]);
        t = min(t, s_bound[w]);
    }

    // ---- sum of exp(x - cmax) in fp64, fixed reduction order ----
    double acc = 0.0;
#pragma unroll
    for (int s = 0; s < kSlots; ++s)
        if (slot_index(s) >= 0) acc += exp((double)x[s] - (double)cmax);
    acc = wave_sum_f64(acc);
    if (lane == 0) s_dsum[wave] = acc;

    // ---- rank the elements that reach t ----
    const uint32_t base_id = (uint32_t)start;
    auto composite = [&](uint32_t key, int i) -> uint64_t {
        return ((uint64_t)key << 32) | (uint64_t)(uint32_t)(~(base_id + (uint32_t)i));
    };
    uint64_t comp[kSlots];
#pragma unroll
    for (int s = 0; s < kSlots; ++s) {
        const int i = slot_index(s);
        comp[s] = i >= 0 ? composite(float_key(x[s]), i) : 0ull;
    }
    uint64_t *out = cand + (row * chunks + c) * (size_t)kc;
    auto emit = [&](int rank, uint64_t cc) { out[rank] = cc; };
    BucketScratch bs{s_cnt, s_start, s_list, s_wave, s_misc};
    int m;
    const bool done = block_bucket_rank<kChunkThreads, kSlots>(comp, t, float_key(cmax), kc, bs, &m, emit);
    if (tid == 0) {  // s_dsum is complete: block_bucket_rank synchronised the workgroup
        double S = s_dsum[0];
        for (int w = 1; w < kChunkWaves; ++w) S += s_dsum[w];
        double *st = stat + (row * chunks + c) * 2;
        st[0] = (double)cmax;
        st[1] = S;
    }
    if (!done) {
        // exact radix select over the whole chunk, then all-pairs ranking of the kc selected
#pragma unroll
        for (int s = 0; s < kSlots; ++s) {
            const int i = slot_index(s);
            if (i >= 0) s_key[i] = float_key(x[s]);
        }
        if (tid == 0) s_misc[7] = 0;
        __syncthreads();
        auto get = [&](int i) -> uint64_t { return composite(s_key[i], i); };
        SelectScratch sc{hist, s_list, s_wave, s_misc, &s_thr};
        const uint64_t thr = block_select_threshold<kChunkThreads>(get, n, kc, sc);  // n > kc here
        for (int i = tid; i < n; i += kChunkThreads) {
            const uint64_t cc = get(i);
            if (cc >= thr) s_list[atomicAdd(&s_misc[7], 1)] = cc;  // exactly kc <= kCandCap
        }
        __syncthreads();
        block_rank_emit<kChunkThreads>(s_list, kc, emit);
        m = kc;
    }
    for (int i = m + tid; i < kc; i += kChunkThreads) out[i] = 0ull;  // chunk shorter than kc
}

// ------------------------------------------------------------------------------------------
// Merge kernel
// ------------------------------------------------------------------------------------------
constexpr int kMergeThreads = 1024;
constexpr int kMergeWaves = kMergeThreads / 64;
constexpr int kMergeLoads = (kTopkMergeMaxCand + kMergeThreads - 1) / kMergeThreads;

// Every chunk's list arrives sorted, so the q-th entry of each (q = ceil(K / chunks)) bounds
// the row's K-th largest from below: T = the smallest of them is reached by at least
// chunks * q >= K candidates.  Only candidates >= T (a little more than K) are ranked.
__global__ __launch_bounds__(kMergeThreads) void topk_merge_kernel(
    const uint64_t *__restrict__ cand, const double *__restrict__ stat, int K, int kc, int chunks,
    int32_t *__restrict__ topk_tok, float *__restrict__ topk_lp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int n = chunks * kc;
    uint64_t *s_cand = reinterpret_cast<uint64_t *>(smem);        // [n], fallback only
    uint32_t *hist = reinterpret_cast<uint32_t *>(s_cand + n);    // [kHistBins], fallback only
    __shared__ __align__(16) uint64_t s_list[kCandCap];
    __shared__ uint32_t s_cnt[kBuckets];
    __shared__ int s_start[kBuckets];
    __shared__ int s_wave[kMergeWaves + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ unsigned long long s_T, s_top;
    __shared__ uint32_t s_mkey;
    __shared__ double s_part[kMergeWaves];
    __shared__ double s_lse;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t *in = cand + row * (size_t)n;
    const double *st = stat + row * (size_t)chunks * 2;
    if (tid == 0) {
        s_T = ~0ull;
        s_top = 0ull;
        s_mkey = 0u;
        s_misc[7] = 0;
    }
    // candidates of the row (at most kTopkMergeMaxCand): loads issued back to back
    uint64_t cv[kMergeLoads];
#pragma unroll
    for (int u = 0; u < kMergeLoads; ++u) {
        const int i = tid + u * kMergeThreads;
        cv[u] = i < n ? in[i] : 0ull;
    }
    // per-chunk entries: statistics, first (largest) and q-th candidate
    const int q = (K + chunks - 1) / chunks;
    uint64_t c_q = ~0ull, c_top = 0ull;
    double c_max = 0.0, c_sum = 0.0;
    if (tid < chunks) {
        c_q = in[(size_t)tid * kc + q - 1];
        c_top = in[(size_t)tid * kc];
        c_max = st[2 * tid];
        c_sum = st[2 * tid + 1];
    }
    __syncthreads();
    if (tid < chunks) {
        atomicMax(&s_mkey, float_key((float)c_max));
        atomicMin(&s_T, (unsigned long long)c_q);
        atomicMax(&s_top, (unsigned long long)c_top);
    }
    for (int c = tid + kMergeThreads; c < chunks; c += kMergeThreads) {
        atomicMax(&s_mkey, float_key((float)st[2 * c]));
        atomicMin(&s_T, (unsigned long long)in[(size_t)c * kc + q - 1]);
        atomicMax(&s_top, (unsigned long long)in[(size_t)c * kc]);
    }
    __syncthreads();
    // ---- log-sum-exp of the row from the chunk statistics (fp64, fixed order) ----
    const double mx = (double)key_float(s_mkey);
    double part = tid < chunks ? c_sum * exp(c_max - mx) : 0.0;
    for (int c = tid + kMergeThreads; c < chunks; c += kMergeThreads)
        part += st[2 * c + 1] * exp(st[2 * c] - mx);
    part = wave_sum_f64(part);
    if (lane == 0) s_part[wave] = part;
    const uint32_t lo_key = (uint32_t)(s_T >> 32), hi_key = (uint32_t)(s_top >> 32);
    __syncthreads();
    if (tid == kMergeThreads - 1) {  // read by emit() only after further barriers
        double S = s_part[0];
        for (int w = 1; w < kMergeWaves; ++w) S += s_part[w];
        s_lse = mx + log(S);
    }
    // ---- rank the candidates that reach T ----
    // T == 0 (a chunk shorter than q): every candidate counts, down to key 0
    auto emit = [&](int rank, uint64_t cc) {
        topk_tok[row * (size_t)K + rank] = (int32_t)(~(uint32_t)cc);
        topk_lp[row * (size_t)K + rank] = (float)((double)key_float((uint32_t)(cc >> 32)) - s_lse);
    };
    BucketScratch bs{s_cnt, s_start, s_list, s_wave, s_misc};
    int m;
    if (block_bucket_rank<kMergeThreads, kMergeLoads>(cv, lo_key, hi_key, K, bs, &m, emit)) return;
    // heavy ties: exact radix select over all candidates staged in LDS
#pragma unroll
    for (int u = 0; u < kMergeLoads; ++u) {
        const int i = tid + u * kMergeThreads;
        if (i < n) s_cand[i] = cv[u];
    }
    __syncthreads();
    auto get = [&](int i) -> uint64_t { return s_cand[i]; };
    SelectScratch sc{hist, s_list, s_wave, s_misc, &s_thr};
    // zero padding entries are smaller than every candidate, and K <= the number of real ones
    const uint64_t thr = n > K ? block_select_threshold<kMergeThreads>(get, n, K, sc) : 1ull;
    for (int i = tid; i < n; i += kMergeThreads) {
        const uint64_t cc = s_cand[i];
        if (cc >= thr && cc != 0ull) s_list[atomicAdd(&s_misc[7], 1)] = cc;  // exactly K
    }
    __syncthreads();
    block_rank_emit<kMergeThreads>(s_list, K, emit);
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
    const size_t lds_chunk = (size_t)p.chunk_len * 4 + kHistBins * 4;
    const size_t lds_merge = (size_t)p.chunks * p.kc * 8 + kHistBins * 4;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(topk_chunk_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kTopkChunkMax * 4 + kHistBins * 4) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(topk_merge_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kTopkMergeMaxCand * 8 + kHistBins * 4) != hipSuccess)
            return DDTREE_ERR_HIP;
        attr_set = true;
    }
    hipStream_t st = as_stream(stream);
    DDT_LAUNCH(DDTREE_KERNEL_TOPK_CHUNK, st, topk_chunk_kernel, dim3(p.chunks, B, batch), dim3(kChunkThreads), lds_chunk, st,
                       logits, V, p.chunk_len, p.kc, p.chunks, cand, stat);
    DDT_LAUNCH(DDTREE_KERNEL_TOPK_MERGE, st, topk_merge_kernel, dim3(B, batch), dim3(kMergeThreads), lds_merge, st, cand,
                       stat, K, p.kc, p.chunks, topk_tok, topk_lp);
    return launch_status();
}
