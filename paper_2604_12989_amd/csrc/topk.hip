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
#include <type_traits>

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
    if (rows >= kTopkRowKernelMinRows) {  // one workgroup per row, no scratch
        p.row_kernel = true;
        p.chunks = 1;
        p.chunk_len = V;
        p.kc = K;
        p.cand_off = p.stat_off = 0;
        p.bytes = 256;
        p.ok = true;
        return p;
    }
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

constexpr int kCandCap = 2048;  // elements placed in LDS for exact ranking
constexpr int kBuckets = 1024;

struct BucketScratch {
    uint32_t *cnt;     // [kBuckets]
    int *start;        // [kBuckets + 1]
    uint64_t *sorted;  // [kCandCap]
    int *s_wave;       // [NT/64]
    int *s_misc;       // [8]
};

// Exact descending ranks, for ranks < want, of the workgroup's elements whose value lies in
// [lo, hi].  Each thread brings NS values in registers (-inf = empty slot; values below lo are
// ignored) and comp(i), the composite of slot i, evaluated only for the few elements that are
// placed.  Bit i of `active` (uniform over the wave) tells whether slot i can be non-empty
// anywhere in the wave, so that a wave skips the code of slots it does not use.
// The value range is cut into kBuckets equal buckets, bucket 0 the highest: an element's rank
// is the population of the buckets above its own plus the number of larger elements inside its
// bucket, which is found by placing the buckets that can reach rank < want side by side in LDS.
// Returns false, having emitted nothing, if those buckets hold more than kCandCap elements
// (heavy ties); *total_out = number of elements considered.
template <int NT, int NS, class Comp, class Emit>
__device__ bool block_bucket_rank(const float (&x)[NS], Comp comp, uint32_t active, float lo, float hi,
                                  int want, BucketScratch s, int *total_out, Emit emit)
{
    static_assert(NT == kBuckets, "one bucket per thread");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    s.cnt[tid] = 0;
    if (tid == 0) {
        s.s_misc[0] = -1;
        s.s_misc[1] = kBuckets - 1;
        s.start[kBuckets] = 0;  // read (and ignored) by slots that hold no element
    }
    __syncthreads();
    const float inv = (float)kBuckets / fmaxf(hi - lo, 1e-30f);
    // monotone in the value: float subtraction, scaling and truncation all preserve order
    auto bucket_of = [&](float v) { return min((int)((hi - v) * inv), kBuckets - 1); };
    // the counting atomics go out back to back: the positions they return are not needed
    // before the scan below
    int bkt[NS];
    uint32_t pos[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        bkt[i] = kBuckets;
        pos[i] = 0;
        if ((active >> i) & 1u) {
            if (x[i] >= lo) {
                bkt[i] = bucket_of(x[i]);
                pos[i] = atomicAdd(&s.cnt[bkt[i]], 1u);
            }
        }
    }
    __syncthreads();
    // exclusive scan of the bucket populations, bucket 0 (highest values) first
    const int mine = (int)s.cnt[tid];
    const int incl = wave_scan_inclusive_i32(mine);
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
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if ((active >> i) & 1u) {
            const int st = s.start[bkt[i]];
            if (bkt[i] <= b_last) s.sorted[st + (int)pos[i]] = comp(i);
        }
    __syncthreads();
    // one thread per placed element: count the larger members of its bucket
    for (int e = tid; e < placed; e += NT) {
        const uint64_t ce = s.sorted[e];
        const int b = bucket_of(key_float((uint32_t)(ce >> 32)));
        const int bs = s.start[b], nb = (int)s.cnt[b];
        int g = 0;
        for (int j = 0; j < nb; ++j) g += s.sorted[bs + j] > ce ? 1 : 0;
        if (bs + g < want) emit(bs + g, ce);
    }
    return true;
}

// exp(y) for y <= 0 in fp64 to a relative error below 4e-11: y = (64 n + j) ln2/64 + r with
// |r| <= ln2/128, so exp(y) = 2^n * 2^(j/64) * exp(r); 2^(j/64) comes from a 64-entry table and
// exp(r) from its Taylor polynomial of degree 3 (remainder r^4/24 < 3.6e-11; the reduction by one
// fp64 multiple of ln2/64 is off by less than 6e-14).  The row's log-sum-exp needs its sum to some
// 1e-8 for a log-probability that is right to the last fp32 bit; every fp64 instruction here is
// paid 9.7 million times a step.  Returns 0 below the fp64 range.
__device__ const double kExp2Table[64] = {
    0x1.0000000000000p+0, 0x1.02c9a3e778061p+0, 0x1.059b0d3158574p+0, 0x1.0874518759bc8p+0,
    0x1.0b5586cf9890fp+0, 0x1.0e3ec32d3d1a2p+0, 0x1.11301d0125b51p+0, 0x1.1429aaea92de0p+0,
    0x1.172b83c7d517bp+0, 0x1.1a35beb6fcb75p+0, 0x1.1d4873168b9aap+0, 0x1.2063b88628cd6p+0,
    0x1.2387a6e756238p+0, 0x1.26b4565e27cddp+0, 0x1.29e9df51fdee1p+0, 0x1.2d285a6e4030bp+0,
    0x1.306fe0a31b715p+0, 0x1.33c08b26416ffp+0, 0x1.371a7373aa9cbp+0, 0x1.3a7db34e59ff7p+0,
    0x1.3dea64c123422p+0, 0x1.4160a21f72e2ap+0, 0x1.44e086061892dp+0, 0x1.486a2b5c13cd0p+0,
    0x1.4bfdad5362a27p+0, 0x1.4f9b2769d2ca7p+0, 0x1.5342b569d4f82p+0, 0x1.56f4736b527dap+0,
    0x1.5ab07dd485429p+0, 0x1.5e76f15ad2148p+0, 0x1.6247eb03a5585p+0, 0x1.6623882552225p+0,
    0x1.6a09e667f3bcdp+0, 0x1.6dfb23c651a2fp+0, 0x1.71f75e8ec5f74p+0, 0x1.75feb564267c9p+0,
    0x1.7a11473eb0187p+0, 0x1.7e2f336cf4e62p+0, 0x1.82589994cce13p+0, 0x1.868d99b4492edp+0,
    0x1.8ace5422aa0dbp+0, 0x1.8f1ae99157736p+0, 0x1.93737b0cdc5e5p+0, 0x1.97d829fde4e50p+0,
    0x1.9c49182a3f090p+0, 0x1.a0c667b5de565p+0, 0x1.a5503b23e255dp+0, 0x1.a9e6b5579fdbfp+0,
    0x1.ae89f995ad3adp+0, 0x1.b33a2b84f15fbp+0, 0x1.b7f76f2fb5e47p+0, 0x1.bcc1e904bc1d2p+0,
    0x1.c199bdd85529cp+0, 0x1.c67f12e57d14bp+0, 0x1.cb720dcef9069p+0, 0x1.d072d4a07897cp+0,
    0x1.d5818dcfba487p+0, 0x1.da9e603db3285p+0, 0x1.dfc97337b9b5fp+0, 0x1.e502ee78b3ff6p+0,
    0x1.ea4afa2a490dap+0, 0x1.efa1bee615a27p+0, 0x1.f50765b6e4540p+0, 0x1.fa7c1819e90d8p+0};
__device__ __forceinline__ double exp_nonpositive(double y, const double *s_tab)
{
    const double k = rint(y * 92.33248261689366);              // 64 / ln 2
    const double r = fma(k, -0x1.62e42fefa39efp-7, y);         // ln2/64
    const int ki = (int)k;
    double p = fma(r, 1.0 / 6.0, 0.5);
    p = fma(r, p, 1.0);
    p = fma(r, p, 1.0);
    const double v = ldexp(s_tab[ki & 63] * p, ki >> 6);
    return y > -708.0 ? v : 0.0;
}

// ------------------------------------------------------------------------------------------
// Chunk kernel
// ------------------------------------------------------------------------------------------
constexpr int kChunkThreads = 1024;
constexpr int kChunkWaves = kChunkThreads / 64;
constexpr int kVecPerThread = kTopkChunkMax / 4 / kChunkThreads;
constexpr int kSlots = 4 * kVecPerThread + 2;  // float4 body + one head and one tail element
static_assert(kVecPerThread * 4 * kChunkThreads == kTopkChunkMax, "chunk must tile the workgroup");

// Largest value of each group of `group` adjacent lanes (a power of two), then the smallest of
// the wave's group maxima.  Valid in lane 63.
__device__ __forceinline__ uint32_t wave_min_of_group_max(uint32_t v, int group)
{
    auto step = [&](uint32_t o, int d) { v = d < group ? max(v, o) : min(v, o); };
    step(dpp_u<0xB1>(v), 1);
    step(dpp_u<0x4E>(v), 2);
    step(dpp_u<0x141>(v), 4);
    step(dpp_u<0x140>(v), 8);
    step(dpp_u<0x142, 0xA>(v), 16);
    step(dpp_u<0x143, 0xC>(v), 32);
    return v;
}

// The chunk stays in registers (at most 14 elements per thread).  A lower bound t on the
// chunk's kc-th largest value comes almost free: cut every wave into g >= kc / waves groups of
// adjacent lanes, take each group's largest value, and let t be the smallest of all group
// maxima; the waves * g >= kc maxima are distinct elements that reach t.  Elements >= t (about
// one in seven for kc = 256) are ranked exactly by block_bucket_rank and the top kc written in
// descending order.  Chunks it cannot handle (heavy ties, or kc so large that the bound passes
// most of the chunk) take the radix select over keys staged in LDS.
__global__ __launch_bounds__(kChunkThreads) void topk_chunk_kernel(
    const float *__restrict__ logits, int V, int chunk_len, int kc, int chunks,
    uint64_t *__restrict__ cand, double *__restrict__ stat)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *s_key = reinterpret_cast<uint32_t *>(smem);  // [chunk_len], fallback only
    uint32_t *hist = s_key + chunk_len;                    // [kHistBins], fallback only
    __shared__ __align__(16) uint64_t s_list[kCandCap];
    __shared__ uint32_t s_cnt[kBuckets];
    __shared__ int s_start[kBuckets + 1];
    __shared__ int s_wave[kChunkWaves + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ float s_fmax[kChunkWaves];
    __shared__ uint32_t s_bound[kChunkWaves];
    __shared__ float s_fmin[kChunkWaves];
    __shared__ double s_dsum[kChunkWaves];
    __shared__ int s_neq[kChunkWaves];
    __shared__ double s_exp2[64];

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
    // empty slots hold -inf: no effect on the max, an exp term of 0, and below every bound lo
    // that block_bucket_rank is given (chunks with real -inf elements take the radix select)
    const float kEmpty = -INFINITY;
    float x[kSlots];
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
        const int j = tid + u * kChunkThreads;
        const float4 v = j < nvec ? pv[j] : make_float4(kEmpty, kEmpty, kEmpty, kEmpty);
        x[4 * u + 0] = v.x;
        x[4 * u + 1] = v.y;
        x[4 * u + 2] = v.z;
        x[4 * u + 3] = v.w;
    }
    x[kSlots - 2] = tid < head ? p[tid] : kEmpty;
    x[kSlots - 1] = tid < n - tail0 ? p[tail0 + tid] : kEmpty;
    if (tid < 64) s_exp2[tid] = kExp2Table[tid];
    // element index of slot s within the chunk, -1 if the slot is empty
    auto slot_index = [&](int s) -> int {
        if (s < 4 * kVecPerThread) {
            const int j = tid + (s >> 2) * kChunkThreads;
            return j < nvec ? head + 4 * j + (s & 3) : -1;
        }
        if (s == kSlots - 2) return tid < head ? tid : -1;
        return tid < n - tail0 ? tail0 + tid : -1;
    };
    // slots that hold an element in at least one lane of this wave (uniform)
    const int wave_base = __builtin_amdgcn_readfirstlane(tid & ~63);
    uint32_t active = 0;
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u)
        if (wave_base + u * kChunkThreads < nvec) active |= 0xFu << (4 * u);
    if (wave_base < head) active |= 1u << (kSlots - 2);
    if (wave_base < n - tail0) active |= 1u << (kSlots - 1);

    // ---- chunk max, chunk min and the bound t.  Every element is ranked (t = chunk min) when
    //      the chunk is small, or when a group has no element at all and the bound is void ----
    const bool take_all = n <= kCandCap;
    const bool void_bound = nvec < kChunkThreads;  // some thread holds no element
    float tmax = -INFINITY, tmin = INFINITY;
#pragma unroll
    for (int s = 0; s < kSlots; ++s)
        if ((active >> s) & 1u) tmax = fmaxf(tmax, x[s]);
    if (take_all || void_bound) {
#pragma unroll
        for (int s = 0; s < kSlots; ++s)
            if (((active >> s) & 1u) && slot_index(s) >= 0) tmin = fminf(tmin, x[s]);
    }
    const bool any = tid < nvec || tid < head || tid < n - tail0;
    const float wmax = wave_max_f32(tmax);
    int group = 64;  // lanes per group: the largest power of two with waves * (64 / group) >= kc
    while (group > 1 && kChunkWaves * (64 / group) < kc) group >>= 1;
    const uint32_t bound = wave_min_of_group_max(any ? float_key(tmax) : 0u, group);
    const float wmin = -wave_max_f32(-tmin);
    if (lane == 63) {
        s_fmax[wave] = wmax;
        s_fmin[wave] = wmin;
        s_bound[wave] = bound;
    }
    __syncthreads();
    float cmax = s_fmax[0], cmin = s_fmin[0];
    uint32_t t = s_bound[0];
#pragma unroll
    for (int w = 1; w < kChunkWaves; ++w) {
        cmax = fmaxf(cmax, s_fmax[w]);
        cmin = fminf(cmin, s_fmin[w]);
        t = min(t, s_bound[w]);
    }
    const float lo = (take_all || void_bound) ? cmin : key_float(t);

    // ---- sum of exp(x - cmax) in fp64, fixed reduction order, one instance of the maximum left
    //      out: the row's log-sum-exp is formed as max + log1p(sum over everything else), which
    //      stays accurate when one token holds nearly all the probability (its log-probability
    //      is -log1p(tiny), and a sum that starts at 1 would have rounded the tiny part away).
    //      Elements equal to the maximum are counted, not added.
    //      (The four elements of a 16-byte load go through the exponential side by side, in one
    //      basic block: taken one slot at a time behind a test of its own, each exponential is a
    //      chain of dependent fp64 instructions and an LDS read with nothing to overlap it.)
    double acc = 0.0;
    int neq = 0;
    static_assert(kVecPerThread == 3, "the grouping below is written for three loads per thread");
    auto exp_slots = [&](auto First, auto Count) {
        constexpr int s0 = decltype(First)::value, cnt = decltype(Count)::value;
        double e[cnt];
#pragma unroll
        for (int j = 0; j < cnt; ++j) e[j] = exp_nonpositive((double)x[s0 + j] - (double)cmax, s_exp2);
#pragma unroll
        for (int j = 0; j < cnt; ++j) {
            const bool eq = x[s0 + j] == cmax;
            neq += eq ? 1 : 0;
            acc += eq ? 0.0 : e[j];
        }
    };
    // (the four slots of a load are active together; the first two loads of a wave mostly both are)
    if ((active & 0xFFu) == 0xFFu) {
        exp_slots(std::integral_constant<int, 0>{}, std::integral_constant<int, 8>{});
    } else {
        if (active & 0x1u) exp_slots(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
        if (active & 0x10u) exp_slots(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
    }
    if (active & 0x100u) exp_slots(std::integral_constant<int, 8>{}, std::integral_constant<int, 4>{});
#pragma unroll
    for (int s = 4 * kVecPerThread; s < kSlots; ++s)
        if ((active >> s) & 1u) {
            const bool eq = x[s] == cmax;
            neq += eq ? 1 : 0;
            const double e = exp_nonpositive((double)x[s] - (double)cmax, s_exp2);
            acc += eq ? 0.0 : e;
        }
    acc = wave_sum_f64_lane63(acc);
    neq = wave_scan_inclusive_i32(neq);
    if (lane == 63) {
        s_dsum[wave] = acc;
        s_neq[wave] = neq;
    }

    // ---- rank the elements that reach t ----
    const uint32_t base_id = (uint32_t)start;
    auto composite = [&](uint32_t key, int i) -> uint64_t {
        return ((uint64_t)key << 32) | (uint64_t)(uint32_t)(~(base_id + (uint32_t)i));
    };
    auto comp = [&](int s) { return composite(float_key(x[s]), slot_index(s)); };
    uint64_t *out = cand + (row * chunks + c) * (size_t)kc;
    auto emit = [&](int rank, uint64_t cc) { out[rank] = cc; };
    BucketScratch bs{s_cnt, s_start, s_list, s_wave, s_misc};
    int m = 0;
    const bool done = lo > -INFINITY &&
                      block_bucket_rank<kChunkThreads, kSlots>(x, comp, active, lo, cmax, kc, bs, &m, emit);
    __syncthreads();
    if (tid == 0) {
        double S = s_dsum[0];
        int n_max = s_neq[0];
        for (int w = 1; w < kChunkWaves; ++w) {
            S += s_dsum[w];
            n_max += s_neq[w];
        }
        double *st = stat + (row * chunks + c) * 2;
        st[0] = (double)cmax;
        st[1] = S + (double)(n_max - 1);  // everything but one instance of the chunk maximum
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
        if (n <= kc) {
            // a ragged last chunk no longer than kc (it holds real -inf entries, or it would have
            // been ranked above): every element is a candidate; n <= kc <= kCandCap
            for (int i = tid; i < n; i += kChunkThreads) s_list[i] = get(i);
            __syncthreads();
            block_rank_emit<kChunkThreads>(s_list, n, emit);
            m = n;
        } else {
            SelectScratch sc{hist, s_list, s_wave, s_misc, &s_thr};
            const uint64_t thr = block_select_threshold<kChunkThreads>(get, n, kc, sc);
            for (int i = tid; i < n; i += kChunkThreads) {
                const uint64_t cc = get(i);
                if (cc >= thr) s_list[atomicAdd(&s_misc[7], 1)] = cc;  // exactly kc <= kCandCap
            }
            __syncthreads();
            block_rank_emit<kChunkThreads>(s_list, kc, emit);
            m = kc;
        }
    }
    for (int i = m + tid; i < kc; i += kChunkThreads) out[i] = 0ull;  // chunk shorter than kc
}

// ------------------------------------------------------------------------------------------
// Merge kernel
// ------------------------------------------------------------------------------------------
constexpr int kMergeThreads = 1024;
constexpr int kMergeWaves = kMergeThreads / 64;
constexpr int kMergeLoads = (kTopkMergeMaxCand + kMergeThreads - 1) / kMergeThreads;
// The kernel is built for 4, 8 and kMergeLoads candidates per thread and the host takes the
// smallest that holds the row's chunks * kc candidates (config 3: 4096 = 4 per thread): the
// per-slot code of the ranking is issued by all sixteen waves whether a slot holds anything or not.

// Every chunk's list arrives sorted, so the q-th entry of each (q = ceil(K / chunks)) bounds
// the row's K-th largest from below: T = the smallest of them is reached by at least
// chunks * q >= K candidates.  Only candidates >= T (a little more than K) are ranked.
template <int NS>
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
    __shared__ int s_start[kBuckets + 1];
    __shared__ int s_wave[kMergeWaves + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ unsigned long long s_T, s_top;
    __shared__ uint32_t s_mkey;
    __shared__ double s_part[kMergeWaves];
    __shared__ double s_lse;  // log1p(sum over everything but the first maximum): lse - max

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
    const int wave_base = __builtin_amdgcn_readfirstlane(tid & ~63);
    uint32_t active = 0;
    uint64_t cv[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const int i = tid + u * kMergeThreads;
        cv[u] = i < n ? in[i] : 0ull;
        if (wave_base + u * kMergeThreads < n) active |= 1u << u;
    }
    float xv[NS];  // candidate values, -inf where there is none
#pragma unroll
    for (int u = 0; u < NS; ++u)
        xv[u] = cv[u] != 0ull ? key_float((uint32_t)(cv[u] >> 32)) : -INFINITY;
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
    // The chunk sums leave one instance of their own maximum out; the chunk that holds the row's
    // first maximum (its top candidate is the row's top candidate) stays that way, every other
    // chunk gets its instance back: the total is the sum over everything but the row's first
    // maximum, and the log-sum-exp is mx + log1p(total).
    const double mx = (double)key_float(s_mkey);
    double part = tid < chunks ? (c_sum + (c_top == s_top ? 0.0 : 1.0)) * exp(c_max - mx) : 0.0;
    for (int c = tid + kMergeThreads; c < chunks; c += kMergeThreads)
        part += (st[2 * c + 1] + (in[(size_t)c * kc] == s_top ? 0.0 : 1.0)) * exp(st[2 * c] - mx);
    part = wave_sum_f64_lane63(part);
    // T == 0 (a chunk shorter than q): every candidate counts, which the radix select handles
    const float lo = s_T >> 32 ? key_float((uint32_t)(s_T >> 32)) : -INFINITY;
    const float hi = key_float((uint32_t)(s_top >> 32));
    // s_lse is read by emit() only after the barriers of the ranking
    if (chunks <= 64) {
        if (tid == 63) s_lse = log1p(part);
    } else {
        if (lane == 63) s_part[wave] = part;
        __syncthreads();
        if (tid == kMergeThreads - 1) {
            double S = s_part[0];
            for (int w = 1; w < kMergeWaves; ++w) S += s_part[w];
            s_lse = log1p(S);
        }
    }
    // ---- rank the candidates that reach T ----
    auto emit = [&](int rank, uint64_t cc) {
        topk_tok[row * (size_t)K + rank] = (int32_t)(~(uint32_t)cc);
        topk_lp[row * (size_t)K + rank] = (float)(((double)key_float((uint32_t)(cc >> 32)) - mx) - s_lse);
    };
    BucketScratch bs{s_cnt, s_start, s_list, s_wave, s_misc};
    int m;
    if (lo > -INFINITY && block_bucket_rank<kMergeThreads, NS>(
                              xv, [&](int u) { return cv[u]; }, active, lo, hi, K, bs, &m, emit))
        return;
    __syncthreads();  // s_lse is complete
    // heavy ties: exact radix select over all candidates staged in LDS
#pragma unroll
    for (int u = 0; u < NS; ++u) {
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


// ------------------------------------------------------------------------------------------
// Row kernel: with a row for every compute unit (many sequences per call) one workgroup scans a
// whole row, the chunk / merge pair and its scratch are not needed, and the scan is bound by HBM
// and the fp64 exponentials instead of by the latency chain of a single chunk.
//   pass 1  every thread streams its share of the row keeping a running maximum, the fp64 sum of
//           exp(x - maximum) over the entries that differ from it and the count of those equal to
//           it (a new maximum rescales sum + count); the workgroup merges these into the row
//           maximum and the sum over everything but one instance of it.  The smallest of the
//           maxima of groups of adjacent threads bounds the K-th largest entry from below.
//   pass 2  the row is read again (it is still in the last-level cache), entries that reach the
//           bound go to a list in LDS, a radix select over the list finds the K-th largest, and
//           the K selected are ranked all-pairs.
// A list that overflows (heavy ties, a void bound) falls back to the radix select over the row.
// ------------------------------------------------------------------------------------------
constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kRowCap = 8192;  // candidates held in LDS
constexpr int kRowBatch = 4;   // 16-byte loads in flight per thread
constexpr size_t kRowLdsBytes = (size_t)kRowCap * 8 + (size_t)kListCap * 8 + (size_t)kHistBins * 4;

template <int N>
__device__ __forceinline__ void row_absorb(const float (&x)[N], float &tmax, double &S, int &neq,
                                           const double *s_exp2)
{
    float bmax = x[0];
#pragma unroll
    for (int i = 1; i < N; ++i) bmax = fmaxf(bmax, x[i]);
    if (bmax > tmax) {
        // what was summed against the old maximum, its own instances included, moves to the new one
        S = tmax > -INFINITY ? (S + (double)neq) * exp_nonpositive((double)tmax - (double)bmax, s_exp2) : 0.0;
        neq = 0;
        tmax = bmax;
    }
    if (tmax > -INFINITY) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const bool eq = x[i] == tmax;
            const double e = exp_nonpositive((double)x[i] - (double)tmax, s_exp2);
            neq += eq ? 1 : 0;
            S += eq ? 0.0 : e;
        }
    }
}

__global__ __launch_bounds__(kRowThreads) void topk_row_kernel(const float *__restrict__ logits, int V, int K,
                                                               int32_t *__restrict__ topk_tok,
                                                               float *__restrict__ topk_lp)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t *s_list = reinterpret_cast<uint64_t *>(smem);       // [kRowCap]
    uint64_t *s_sel = s_list + kRowCap;                          // [kListCap] >= K
    uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_sel + kListCap);  // [kHistBins]
    __shared__ int s_wave[kRowWaves + 1];
    __shared__ int s_misc[8];
    __shared__ uint64_t s_thr;
    __shared__ float s_fmax[kRowWaves];
    __shared__ uint32_t s_bound[kRowWaves];
    __shared__ double s_dsum[kRowWaves];
    __shared__ double s_exp2[64];
    __shared__ double s_exc;
    __shared__ int s_owner, s_cnt;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = blockIdx.x;
    const float *p = logits + row * (size_t)V;
    int head = (int)((4 - ((reinterpret_cast<uintptr_t>(p) >> 2) & 3)) & 3);
    if (head > V) head = V;
    const int nvec = (V - head) >> 2;
    const int tail0 = head + 4 * nvec;
    const float4 *pv = reinterpret_cast<const float4 *>(p + head);
    const bool edge = tid < head || tid < V - tail0;  // this thread holds a head or tail element
    if (tid < 64) s_exp2[tid] = kExp2Table[tid];
    if (tid == 0) {
        s_owner = kRowThreads;
        s_cnt = 0;
    }
    __syncthreads();

    const bool any = tid < nvec || edge;
    const bool take_all = V <= kRowCap || nvec < kRowThreads;  // some thread may hold no element
    int group = 64;  // lanes per group: the largest power of two with waves * (64 / group) >= K
    while (group > 1 && kRowWaves * (64 / group) < K) group >>= 1;
    // Lower bound on the row's K-th largest entry from what the threads have seen so far: the
    // smallest of the maxima of groups of adjacent threads (waves * 64 / group >= K distinct
    // entries reach it).  It only grows as the scan proceeds.
    float tmax = -INFINITY;
    auto bound_now = [&]() -> float {
        const uint32_t bound = wave_min_of_group_max(any ? float_key(tmax) : 0u, group);
        if (lane == 63) s_bound[wave] = bound;
        __syncthreads();
        uint32_t t = s_bound[0];
#pragma unroll
        for (int w = 1; w < kRowWaves; ++w) t = min(t, s_bound[w]);
        __syncthreads();
        return key_float(t);
    };
    float lo = -INFINITY;  // entries >= lo go to the list
    auto composite = [&](float x, int i) -> uint64_t {
        return ((uint64_t)float_key(x) << 32) | (uint64_t)(uint32_t)(~(uint32_t)i);
    };
    auto push = [&](bool on, float x, int i) {
        const bool take = on && x >= lo;
        const uint64_t bal = __ballot(take);
        if (bal == 0) return;  // uniform over the wave
        const int n_take = __popcll(bal);
        int base = 0;
        if (lane == __builtin_ctzll(bal)) base = atomicAdd(&s_cnt, n_take);
        base = __shfl(base, __builtin_ctzll(bal), 64);
        const int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
        if (take && pos < kRowCap) s_list[pos] = composite(x, i);
    };
    // the same for the sixteen entries of a batch with one list reservation per wave
    auto push_batch = [&](const float (&x)[4 * kRowBatch], int base) {
        int n = 0;
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u) {
            const bool on = base + u * kRowThreads + tid < nvec;
#pragma unroll
            for (int e = 0; e < 4; ++e) n += (on && x[4 * u + e] >= lo) ? 1 : 0;
        }
        const int incl = wave_scan_inclusive_i32(n);
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (total == 0) return;  // uniform over the wave
        int first = 0;
        if (lane == 63) first = atomicAdd(&s_cnt, total);
        int pos = __builtin_amdgcn_readlane(first, 63) + incl - n;
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u) {
            const int j = base + u * kRowThreads + tid;
            const bool on = j < nvec;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (on && x[4 * u + e] >= lo) {
                    if (pos < kRowCap) s_list[pos] = composite(x[4 * u + e], head + 4 * j + e);
                    ++pos;
                }
        }
    };
    auto push_edges = [&]() {  // head and tail elements live in the first lanes of wave 0
        if (wave == 0) {
            push(tid < head, tid < head ? p[tid] : 0.0f, tid);
            push(tid < V - tail0, tid < V - tail0 ? p[tail0 + tid] : 0.0f, tail0 + tid);
        }
    };

    // ---- the scan: running maximum, sum and count per thread; entries that reach the bound of
    //      the moment (refreshed after 1, 2 and 4 batches) are appended to the list, a superset
    //      of what the final bound admits ----
    double S = 0.0;
    int neq = 0;
    int batch_no = 0;
    // the loads of the next batch are requested before the exponentials of this one
    auto load_batch = [&](int base, float4 (&v)[kRowBatch]) {
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u) {
            const int j = base + u * kRowThreads + tid;
            v[u] = j < nvec ? pv[j] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
    };
    float4 nxt[kRowBatch];
    load_batch(0, nxt);
    for (int base = 0; base < nvec; base += kRowBatch * kRowThreads, ++batch_no) {
        float x[4 * kRowBatch];
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u) {
            x[4 * u + 0] = nxt[u].x;
            x[4 * u + 1] = nxt[u].y;
            x[4 * u + 2] = nxt[u].z;
            x[4 * u + 3] = nxt[u].w;
        }
        load_batch(base + kRowBatch * kRowThreads, nxt);  // past the end: nothing is read
        row_absorb(x, tmax, S, neq, s_exp2);
        if (!take_all && (batch_no == 0 || batch_no == 1 || batch_no == 3)) lo = bound_now();
        push_batch(x, base);
    }
    if (edge) {
        const float x[2] = {tid < head ? p[tid] : -INFINITY, tid < V - tail0 ? p[tail0 + tid] : -INFINITY};
        row_absorb(x, tmax, S, neq, s_exp2);
    }
    push_edges();

    // ---- row maximum and the sum over everything but one instance of it ----
    const float wmax = wave_max_f32(tmax);
    if (lane == 63) s_fmax[wave] = wmax;
    __syncthreads();
    float m = s_fmax[0];
#pragma unroll
    for (int w = 1; w < kRowWaves; ++w) m = fmaxf(m, s_fmax[w]);
    if (any && tmax == m) atomicMin(&s_owner, tid);  // one thread gives up one instance of the maximum
    __syncthreads();
    double c = 0.0;
    if (tmax > -INFINITY)
        c = (S + (double)(neq - (tid == s_owner ? 1 : 0))) * exp_nonpositive((double)tmax - (double)m, s_exp2);
    c = wave_sum_f64_lane63(c);
    if (lane == 63) s_dsum[wave] = c;
    __syncthreads();
    if (tid == 0) {
        double S1 = s_dsum[0];
        for (int w = 1; w < kRowWaves; ++w) S1 += s_dsum[w];
        s_exc = log1p(S1);  // read by emit() after later barriers
    }

    // ---- a list that overflowed is filled again with the final bound, from the row in cache ----
    if (s_cnt > kRowCap && !take_all) {
        lo = bound_now();  // also orders the reads of s_cnt above before its reset
        if (tid == 0) s_cnt = 0;
        __syncthreads();
        for (int base = 0; base < nvec; base += kRowBatch * kRowThreads) {
            float4 v[kRowBatch];
            load_batch(base, v);
            float x[4 * kRowBatch];
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                x[4 * u + 0] = v[u].x;
                x[4 * u + 1] = v[u].y;
                x[4 * u + 2] = v[u].z;
                x[4 * u + 3] = v[u].w;
            }
            push_batch(x, base);
        }
        push_edges();
    }
    if (tid == 0) s_misc[7] = 0;
    __syncthreads();
    const int cnt = s_cnt;  // at least K: the bound is reached by K entries, or everything was taken

    // ---- the K largest of the list (or, on overflow, of the row), then their exact order ----
    SelectScratch sc{s_hist, s_sel, s_wave, s_misc, &s_thr};
    if (cnt <= kRowCap) {
        auto get = [&](int i) -> uint64_t { return s_list[i]; };
        const uint64_t thr = cnt > K ? block_select_threshold<kRowThreads>(get, cnt, K, sc) : 0ull;
        for (int i = tid; i < cnt; i += kRowThreads) {
            const uint64_t cc = s_list[i];
            if (cc >= thr) {
                const int pos = atomicAdd(&s_misc[7], 1);
                if (pos < kListCap) s_sel[pos] = cc;  // exactly K
            }
        }
    } else {
        auto get = [&](int i) -> uint64_t { return composite(p[i], i); };
        const uint64_t thr = block_select_threshold<kRowThreads>(get, V, K, sc);
        for (int i = tid; i < V; i += kRowThreads) {
            const uint64_t cc = get(i);
            if (cc >= thr) {
                const int pos = atomicAdd(&s_misc[7], 1);
                if (pos < kListCap) s_sel[pos] = cc;  // exactly K
            }
        }
    }
    __syncthreads();
    auto emit = [&](int rank, uint64_t cc) {
        topk_tok[row * (size_t)K + rank] = (int32_t)(~(uint32_t)cc);
        topk_lp[row * (size_t)K + rank] =
            (float)(((double)key_float((uint32_t)(cc >> 32)) - (double)m) - s_exc);
    };
    block_rank_emit<kRowThreads>(s_sel, K, emit);
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

    hipStream_t st = as_stream(stream);
    if (p.row_kernel) {
        static std::atomic<bool> row_lds_allowed{false};
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(topk_row_kernel), kRowLdsBytes, row_lds_allowed))
            return DDTREE_ERR_HIP;
        DDT_LAUNCH(DDTREE_KERNEL_TOPK_CHUNK, st, topk_row_kernel, dim3(batch * B), dim3(kRowThreads), kRowLdsBytes,
                   st, logits, V, K, topk_tok, topk_lp);
        return launch_status();
    }
    static std::atomic<bool> chunk_lds_allowed{false}, merge_lds_allowed[3] = {{false}, {false}, {false}};
    const size_t lds_chunk = (size_t)p.chunk_len * 4 + kHistBins * 4;
    const size_t lds_merge = (size_t)p.chunks * p.kc * 8 + kHistBins * 4;
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(topk_chunk_kernel), kTopkChunkMax * 4 + kHistBins * 4,
                           chunk_lds_allowed) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(topk_merge_kernel<4>), kTopkMergeMaxCand * 8 + kHistBins * 4,
                           merge_lds_allowed[0]) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(topk_merge_kernel<8>), kTopkMergeMaxCand * 8 + kHistBins * 4,
                           merge_lds_allowed[1]) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(topk_merge_kernel<kMergeLoads>),
                           kTopkMergeMaxCand * 8 + kHistBins * 4, merge_lds_allowed[2]))
        return DDTREE_ERR_HIP;
    DDT_LAUNCH(DDTREE_KERNEL_TOPK_CHUNK, st, topk_chunk_kernel, dim3(p.chunks, B, batch), dim3(kChunkThreads), lds_chunk, st,
                       logits, V, p.chunk_len, p.kc, p.chunks, cand, stat);
    const long long per_thread = ((long long)p.chunks * p.kc + kMergeThreads - 1) / kMergeThreads;
    if (per_thread <= 4)
        DDT_LAUNCH(DDTREE_KERNEL_TOPK_MERGE, st, topk_merge_kernel<4>, dim3(B, batch), dim3(kMergeThreads), lds_merge,
                   st, cand, stat, K, p.kc, p.chunks, topk_tok, topk_lp);
    else if (per_thread <= 8)
        DDT_LAUNCH(DDTREE_KERNEL_TOPK_MERGE, st, topk_merge_kernel<8>, dim3(B, batch), dim3(kMergeThreads), lds_merge,
                   st, cand, stat, K, p.kc, p.chunks, topk_tok, topk_lp);
    else
        DDT_LAUNCH(DDTREE_KERNEL_TOPK_MERGE, st, topk_merge_kernel<kMergeLoads>, dim3(B, batch), dim3(kMergeThreads),
                   lds_merge, st, cand, stat, K, p.kc, p.chunks, topk_tok, topk_lp);
    return launch_status();
}
