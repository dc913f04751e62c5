// Greedy verifier walk (paper Section 4.4, second paragraph, and Figure 1b) and cache compaction
// (Section 4.4, last sentence).
//
//   argmax kernel  HBM-bound scan of the target logits: one workgroup per (row, segment),
//                  coalesced 16-byte loads, first-maximum semantics (lowest id among equal
//                  maxima), one (value, index) partial per segment.
//   walk kernel    one workgroup per sequence: folds the partials into the posterior token of
//                  every node, then decides acceptance for all nodes at once: node i is accepted
//                  iff every node on its root path carries the token its parent's posterior
//                  chose.  The accepted nodes form the single path the sequential walk of the
//                  paper visits, and the deepest one yields the bonus token.
//   compact kernel copies the accepted tree rows of K and V behind the cache.
#include "common.hpp"

namespace ddt {

constexpr int kArgmaxThreads = 256;
constexpr int kWalkThreads = 256;

AcceptPlan accept_plan(int batch, int T, int V, bool sampled)
{
    AcceptPlan p{};
    long long rows = (long long)batch * T;
    // about 3000 workgroups stream closest to the HBM rate; the sampled scan prunes key evaluations
    // against the best key a wave has found so far, which longer segments serve better
    const int target = sampled ? 1024 : 3072;
    int S = (int)((target + rows - 1) / rows);
    int s_cap = V / 8192 > 0 ? V / 8192 : 1;  // keep segments at least 8192 long
    if (S > s_cap) S = s_cap;
    if (S < 1) S = 1;
    int len = (V + S - 1) / S;
    len = (len + 3) / 4 * 4;
    p.seg_len = len;
    p.splits = (V + len - 1) / len;
    p.part_off = 0;
    p.bytes = align_up((size_t)rows * p.splits * 8, 256);
    return p;
}

struct ArgPart {
    float val;
    int32_t idx;
};

__device__ __forceinline__ void arg_update(float &bv, int &bi, float v, int i)
{
    if (v > bv || (v == bv && i < bi)) {
        bv = v;
        bi = i;
    }
}

// Temperature sampling (Section 4.4: verification follows the target's decoding rule, greedy or
// temperature-based sampling).  The token selected at a node is argmax_v (logit[v] / tau + g[v])
// with Gumbel noise g = -log(-log(u)), which is a sample from softmax(logit / tau); u in (0,1)
// comes from a counter-based generator keyed by (seed, row, v), so the draw does not depend on
// how the scan is split over threads:
//     mix(x):  x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16
//     h = mix(mix(v ^ seed_lo) + 0x9E3779B9 * row + seed_hi),   u = ((h >> 8) + 0.5) / 2^24
struct SampleArgs {
    float inv_tau;       // 0 selects the greedy rule
    uint32_t seed_lo, seed_hi;
};
__device__ __forceinline__ uint32_t sample_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}
template <bool SAMPLE>
__device__ __forceinline__ float select_key(float logit, uint32_t id, uint32_t row_term, const SampleArgs &sa)
{
    if (!SAMPLE) return logit;
    const uint32_t h = sample_mix(sample_mix(id ^ sa.seed_lo) + row_term);
    // -ln u in fp32 without losing the draws that matter most (u close to 1 gives the largest
    // noise): for k < 2^23, u = (k + 0.5) / 2^24 is exact in fp32; otherwise w = 1 - u =
    // (2^24 - 1 - k + 0.5) / 2^24 is, and -ln(1 - w) is taken from its series when w is small
    const uint32_t k = h >> 8;
    const bool low = k < (1u << 23);
    const float frac = ((float)(low ? k : 16777215u - k) + 0.5f) * (1.0f / 16777216.0f);  // u or w
    const float la = -0.69314718056f * __builtin_amdgcn_logf(low ? frac : 1.0f - frac);
    const float series = frac * (1.0f + frac * (0.5f + frac * (0.333333343f + frac * 0.25f)));
    const float nl = (!low && frac < 0.015625f) ? series : la;
    const float g = -0.69314718056f * __builtin_amdgcn_logf(nl);  // g = -ln(-ln u)
    return fmaf(logit, sa.inv_tau, g);
}

template <bool SAMPLE>
__global__ __launch_bounds__(kArgmaxThreads) void accept_argmax_kernel(
    const float *__restrict__ logits, int T, int V, int seg_len, int splits,
    const int32_t *__restrict__ n_nodes, ArgPart *__restrict__ part, SampleArgs sa)
{
    __shared__ float s_v[kArgmaxThreads / 64];
    __shared__ int s_i[kArgmaxThreads / 64];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x, i = blockIdx.y, seq = blockIdx.z;
    if (i > n_nodes[seq]) return;  // padding row: never read, the walk ignores its partial
    const size_t rowi = (size_t)seq * T + i;
    const uint32_t row_term = 0x9E3779B9u * (uint32_t)rowi + sa.seed_hi;
    const int start = seg * seg_len;
    const int n = min(seg_len, V - start);
    const float *p = logits + rowi * (size_t)V + start;

    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
    int head = (int)((4 - ((reinterpret_cast<uintptr_t>(p) >> 2) & 3)) & 3);
    if (head > n) head = n;
    if (tid < head) {
        bv = select_key<SAMPLE>(p[tid], (uint32_t)(start + tid), row_term, sa);
        bi = start + tid;
    }
    const int nvec = (n - head) >> 2;
    const float4 *pv = reinterpret_cast<const float4 *>(p + head);
    // eight independent 16-byte loads in flight per thread and iteration: about 128 KB per compute
    // unit, what it takes to cover the HBM latency at full bandwidth; the logits are read once,
    // so the loads are marked non-temporal
    constexpr int kInFlight = 8;
    // Sampling: most elements are settled without their logarithms.  The noise is bounded from the
    // hash alone, g = -ln(-ln u) <= -ln(1 - u) = ln(2^25 / w) with the odd integer
    // w = 2^25 - 2k - 1, hence g <= ln2 * (clz(w) - 6); an element whose bound stays below a key
    // this wave has already found (wb) cannot be the row's maximum, nor tie with it.
    // The loop bound is uniform over the wave (its lanes leave the loop together): the wave
    // maximum below reads lane 63, which must have taken part in every round.
    float wb = -INFINITY;
    for (int jb = tid & ~63; jb < nvec; jb += kInFlight * kArgmaxThreads) {
        const int j0 = jb + (tid & 63);
        float4 x[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int j = j0 + u * kArgmaxThreads;
            if (j < nvec) {
                const float *q = reinterpret_cast<const float *>(pv + j);
                x[u].x = __builtin_nontemporal_load(q);
                x[u].y = __builtin_nontemporal_load(q + 1);
                x[u].z = __builtin_nontemporal_load(q + 2);
                x[u].w = __builtin_nontemporal_load(q + 3);
            } else {
                x[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            }
        }
        if (SAMPLE) wb = wave_max_f32(bv);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int ia = start + head + 4 * (j0 + u * kArgmaxThreads);
            if (SAMPLE) {
                if (j0 + u * kArgmaxThreads >= nvec) continue;  // padding lanes draw no noise
                const float xe[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
                bool need[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t h = sample_mix(sample_mix((uint32_t)(ia + e) ^ sa.seed_lo) + row_term);
                    const uint32_t w = 0x1FFFFFFu - ((h >> 8) << 1);
                    const float g_max = 0.6931472f * (float)(__builtin_clz(w) - 6);
                    // (the margin covers the rounding of the exact key, about 2e-6)
                    need[e] = fmaf(xe[e], sa.inv_tau, g_max) + 2e-3f >= wb;
                }
                if (__ballot(need[0] || need[1] || need[2] || need[3]) != 0ull) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (need[e]) {
                            const float ke = select_key<true>(xe[e], (uint32_t)(ia + e), row_term, sa);
                            if (ke > bv) {
                                bv = ke;
                                bi = ia + e;
                            }
                        }
                }
                continue;
            }
            const float k0 = select_key<SAMPLE>(x[u].x, (uint32_t)ia, row_term, sa);
            const float k1 = select_key<SAMPLE>(x[u].y, (uint32_t)ia + 1u, row_term, sa);
            const float k2 = select_key<SAMPLE>(x[u].z, (uint32_t)ia + 2u, row_term, sa);
            const float k3 = select_key<SAMPLE>(x[u].w, (uint32_t)ia + 3u, row_term, sa);
            if (k0 > bv) { bv = k0; bi = ia; }
            if (k1 > bv) { bv = k1; bi = ia + 1; }
            if (k2 > bv) { bv = k2; bi = ia + 2; }
            if (k3 > bv) { bv = k3; bi = ia + 3; }
        }
    }
    const int tail0 = head + 4 * nvec;
    if (tid < n - tail0) {
        const float x = select_key<SAMPLE>(p[tail0 + tid], (uint32_t)(start + tail0 + tid), row_term, sa);
        if (x > bv) { bv = x; bi = start + tail0 + tid; }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float ov = __shfl_xor(bv, d, 64);
        const int oi = __shfl_xor(bi, d, 64);
        arg_update(bv, bi, ov, oi);
    }
    if ((tid & 63) == 0) {
        s_v[tid >> 6] = bv;
        s_i[tid >> 6] = bi;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kArgmaxThreads / 64; ++w) arg_update(bv, bi, s_v[w], s_i[w]);
        ArgPart r;
        r.val = bv;
        r.idx = bi;
        part[rowi * splits + seg] = r;
    }
}

__global__ __launch_bounds__(kWalkThreads) void accept_walk_kernel(
    const ArgPart *__restrict__ part, int T, int splits, int B, const int32_t *__restrict__ tokens,
    const int32_t *__restrict__ parent, const int32_t *__restrict__ depth,
    const int32_t *__restrict__ n_nodes, int32_t *__restrict__ path,
    int32_t *__restrict__ n_accepted, int32_t *__restrict__ bonus_token,
    int32_t *__restrict__ posterior)
{
    __shared__ int s_post[DDTREE_MAX_N + 1];
    __shared__ int s_tok[DDTREE_MAX_N + 1];
    __shared__ int s_par[DDTREE_MAX_N + 1];
    __shared__ int s_dep[DDTREE_MAX_N + 1];
    __shared__ int s_path[DDTREE_MAX_B + 1];
    __shared__ int s_len;
    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const int n = n_nodes[seq];
    const size_t base = (size_t)seq * T;
    for (int i = tid; i < T; i += kWalkThreads) {
        // Everything a row needs is requested before the node count is looked at, so that its
        // arrival and theirs overlap: the first eight partial results of the row (padding rows
        // have none written: what is read there is never used), its token, parent and depth.
        const ArgPart *pp = part + (base + i) * splits;
        ArgPart a[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = u < splits ? pp[u] : ArgPart{-INFINITY, -1};
        const int tk = tokens[base + i], pr = parent[base + i], dp = depth[base + i];
        const bool in_tree = i <= n;
        int post = -1;
        float bv = -INFINITY;
        for (int s0 = 0; s0 < splits; s0 += 8) {
            if (s0 > 0) {
#pragma unroll
                for (int u = 0; u < 8; ++u) a[u] = s0 + u < splits ? pp[s0 + u] : ArgPart{-INFINITY, -1};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < splits && (post < 0 || a[u].val > bv)) {
                    // later segments hold higher ids: strict > keeps the first maximum
                    bv = a[u].val;
                    post = a[u].idx;
                }
        }
        if (!in_tree) post = -1;
        s_post[i] = post;
        s_tok[i] = in_tree ? tk : -1;
        s_par[i] = in_tree ? pr : -1;
        s_dep[i] = dp;
        if (posterior) posterior[base + i] = post;
    }
    if (tid <= B) s_path[tid] = tid == 0 ? 0 : -1;
    if (tid == 0) s_len = 0;
    __syncthreads();
    for (int i = 1 + tid; i <= n; i += kWalkThreads) {
        bool ok = true;
        int j = i;
        while (j > 0 && ok) {
            const int pj = s_par[j];
            ok = s_tok[j] == s_post[pj];
            j = pj;
        }
        if (ok) {
            const int d = s_dep[i];
            if (d >= 1 && d <= B) {
                s_path[d] = i;
                atomicMax(&s_len, d);
            }
        }
    }
    __syncthreads();
    if (tid <= B) path[(size_t)seq * (B + 1) + tid] = s_path[tid];
    if (tid == 0) {
        const int len = s_len;
        n_accepted[seq] = len;
        bonus_token[seq] = s_post[s_path[len]];
    }
}

struct CompactArgs {
    int32_t dst_row[DDTREE_MAX_BATCH];
};

__global__ __launch_bounds__(256) void compact_kernel(
    const uint32_t *__restrict__ k_tree, const uint32_t *__restrict__ v_tree,
    const int32_t *__restrict__ path, const int32_t *__restrict__ n_accepted, CompactArgs args,
    int T, int B, int row_words, uint32_t *__restrict__ k_cache, uint32_t *__restrict__ v_cache)
{
    const int j = blockIdx.x, seq = blockIdx.y;
    if (j > n_accepted[seq]) return;
    const int node = path[(size_t)seq * (B + 1) + j];
    if (node < 0 || node >= T) return;
    const size_t src = ((size_t)seq * T + node) * row_words;
    const size_t dst = ((size_t)args.dst_row[seq] + j) * row_words;
    for (int w = threadIdx.x; w < row_words; w += blockDim.x) {
        k_cache[dst + w] = k_tree[src + w];
        v_cache[dst + w] = v_tree[src + w];
    }
}

}  // namespace ddt

// Scratch of ddtree_accept_noalloc: the partial argmaxes live in this array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device address it returns
// (one per device) is what the kernels are given.
namespace ddt {
constexpr size_t kNoAllocScratchBytes = DDTREE_NOALLOC_SCRATCH_BYTES;  // 32768 (value, index) partials
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kNoAllocMaxDevices = 64;
}  // namespace ddt

// Device address of the scratch array on the current device, looked up once per device.
static int noalloc_scratch(void **out)
{
    static std::atomic<void *> ptrs[ddt::kNoAllocMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= ddt::kNoAllocMaxDevices) return DDTREE_ERR_HIP;
    void *p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(ddt::scratch)) != hipSuccess || !p) return DDTREE_ERR_HIP;
        ptrs[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return DDTREE_OK;
}

static int accept_impl(const float *target_logits, int batch, int T, int V, const int32_t *tokens,
                       const int32_t *parent, const int32_t *depth, const int32_t *n_nodes,
                       int32_t *path, int32_t *n_accepted, int32_t *bonus_token, int32_t *posterior,
                       int B, void *workspace, size_t workspace_bytes, void *stream, bool sample,
                       ddt::SampleArgs sa)
{
    using namespace ddt;
    if (!target_logits || !tokens || !parent || !depth || !n_nodes || !path || !n_accepted ||
        !bonus_token)
        return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 2 || T > DDTREE_MAX_N + 1 || V < 1 || B < 1 ||
        B > DDTREE_MAX_B)
        return DDTREE_ERR_ARG;
    AcceptPlan p = accept_plan(batch, T, V, sample);
    if (!ws_ok(workspace, workspace_bytes, p.bytes)) return DDTREE_ERR_WORKSPACE;
    ArgPart *part = reinterpret_cast<ArgPart *>(static_cast<char *>(workspace) + p.part_off);
    hipStream_t st = as_stream(stream);
    if (sample)
        DDT_LAUNCH(DDTREE_KERNEL_ACCEPT_ARGMAX, st, accept_argmax_kernel<true>, dim3(p.splits, T, batch),
                   dim3(kArgmaxThreads), 0, st, target_logits, T, V, p.seg_len, p.splits, n_nodes, part, sa);
    else
        DDT_LAUNCH(DDTREE_KERNEL_ACCEPT_ARGMAX, st, accept_argmax_kernel<false>, dim3(p.splits, T, batch),
                   dim3(kArgmaxThreads), 0, st, target_logits, T, V, p.seg_len, p.splits, n_nodes, part, sa);
    DDT_LAUNCH(DDTREE_KERNEL_ACCEPT_WALK, st, accept_walk_kernel, dim3(batch), dim3(kWalkThreads), 0, st, part, T, p.splits,
                       B, tokens, parent, depth, n_nodes, path, n_accepted, bonus_token, posterior);
    return launch_status();
}

extern "C" int ddtree_accept(const float *target_logits, int batch, int T, int V,
                             const int32_t *tokens, const int32_t *parent, const int32_t *depth,
                             const int32_t *n_nodes, int32_t *path, int32_t *n_accepted,
                             int32_t *bonus_token, int32_t *posterior, int B, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    return accept_impl(target_logits, batch, T, V, tokens, parent, depth, n_nodes, path, n_accepted,
                       bonus_token, posterior, B, workspace, workspace_bytes, stream, false,
                       ddt::SampleArgs{0.0f, 0u, 0u});
}

extern "C" int ddtree_accept_noalloc(const float *target_logits, int batch, int T, int V,
                                     const int32_t *tokens, const int32_t *parent, const int32_t *depth,
                                     const int32_t *n_nodes, int32_t *path, int32_t *n_accepted,
                                     int32_t *bonus_token, int32_t *posterior, int B, void *stream)
{
    using namespace ddt;
    if (!target_logits || !tokens || !parent || !depth || !n_nodes || !path || !n_accepted || !bonus_token)
        return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 2 || T > DDTREE_MAX_N + 1 || V < 1 || B < 1 ||
        B > DDTREE_MAX_B)
        return DDTREE_ERR_ARG;
    // the partials of this shape must fit the static array (nothing here can grow it)
    if (accept_plan(batch, T, V, false).bytes > kNoAllocScratchBytes) return DDTREE_ERR_WORKSPACE;
    void *ws = nullptr;
    const int rc = noalloc_scratch(&ws);
    if (rc != DDTREE_OK) return rc;
    // Every partial the walk reads is written by the scan of the same call (rows up to n_nodes,
    // all segments), so nothing in the array has to start at zero.
    return accept_impl(target_logits, batch, T, V, tokens, parent, depth, n_nodes, path, n_accepted,
                       bonus_token, posterior, B, ws, kNoAllocScratchBytes, stream, false,
                       ddt::SampleArgs{0.0f, 0u, 0u});
}

extern "C" int ddtree_accept_sampled(const float *target_logits, int batch, int T, int V,
                                     const int32_t *tokens, const int32_t *parent,
                                     const int32_t *depth, const int32_t *n_nodes, float temperature,
                                     uint64_t seed, int32_t *path, int32_t *n_accepted,
                                     int32_t *bonus_token, int32_t *posterior, int B,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!(temperature > 0.0f) || !(temperature < 1e30f)) return DDTREE_ERR_ARG;
    return accept_impl(target_logits, batch, T, V, tokens, parent, depth, n_nodes, path, n_accepted,
                       bonus_token, posterior, B, workspace, workspace_bytes, stream, true,
                       ddt::SampleArgs{1.0f / temperature, (uint32_t)seed, (uint32_t)(seed >> 32)});
}

extern "C" int ddtree_compact(const void *k_tree, const void *v_tree, const int32_t *path,
                              const int32_t *n_accepted, const int32_t *dst_row, int batch, int T,
                              int B, int Hkv, int D, int elem_bytes, void *k_cache, void *v_cache,
                              void *stream)
{
    using namespace ddt;
    if (!k_tree || !v_tree || !path || !n_accepted || !dst_row || !k_cache || !v_cache)
        return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || T < 2 || B < 1 || B > DDTREE_MAX_B || Hkv < 1 ||
        D < 1 || (elem_bytes != 2 && elem_bytes != 4))
        return DDTREE_ERR_ARG;
    const long long row_bytes = (long long)Hkv * D * elem_bytes;
    if (row_bytes % 4 != 0) return DDTREE_ERR_ARG;
    for (const void *t : {k_tree, v_tree, static_cast<const void *>(k_cache), static_cast<const void *>(v_cache)})
        if (reinterpret_cast<uintptr_t>(t) & 3u) return DDTREE_ERR_ARG;  // rows are copied in 4-byte words
    CompactArgs args;
    for (int s = 0; s < batch; ++s) {
        if (dst_row[s] < 0) return DDTREE_ERR_ARG;
        args.dst_row[s] = dst_row[s];
    }
    hipLaunchKernelGGL(compact_kernel, dim3(B + 1, batch), dim3(256), 0, as_stream(stream),
                       static_cast<const uint32_t *>(k_tree), static_cast<const uint32_t *>(v_tree),
                       path, n_accepted, args, T, B, (int)(row_bytes / 4),
                       static_cast<uint32_t *>(k_cache), static_cast<uint32_t *>(v_cache));
    return launch_status();
}
