// Best-first draft-tree construction (paper Algorithm 1) and the tensors compiled from the
// tree for the verifier (Section 4.4: token ids, depth as position id, ancestor-only mask).
//
// One workgroup per sequence; the pops are inherently serial (pop i+1 depends on the pushes of
// pop i), so a single wavefront runs them and the other three wait at a barrier, then all
// 256 threads write the outputs and the ancestor bitmask.
//
// Frontier layout.  Algorithm 1's heap holds, at any time, exactly one candidate per node that
// is already in the tree (root included): that node's next unused child rank.  Popping the
// candidate of node p with rank c creates node n = (p, c); "push next sibling" is c -> c+1 in
// p's entry and "push first child" is a fresh entry for n.  So the frontier is an array indexed
// by node id, with no free list.  Entry e lives in lane e % 64, register slot e / 64, and stays
// in registers for the whole run; a pop is a lane-local max followed by a DPP wave max.
// The log-probability a popped entry needs next (rank c+1 of its row) is prefetched into the
// entry one pop ahead, so no LDS access sits on the pop-to-pop dependency chain.
//
// Runs of consecutive siblings (flat distributions pop many ranks of one parent in a row) are
// popped as one batch: 64 lanes evaluate the next 64 ranks at once against a bound that no other
// entry and no child created by the batch can exceed.
//
// Ties (equal fp32 scores) are resolved as the boundary specifies: the lexicographically
// smaller rank tuple first, a prefix before its extensions.  They are rare and take a slow
// path that walks parent links in LDS.
#include "common.hpp"

namespace ddt {

constexpr int kBuildThreads = 256;

__device__ __forceinline__ uint32_t pack_node(int parent, int rank, int depth)
{
    return (uint32_t)parent | ((uint32_t)rank << 11) | ((uint32_t)depth << 21);
}
__device__ __forceinline__ int node_parent(uint32_t x) { return (int)(x & 0x7FFu); }
__device__ __forceinline__ int node_rank(uint32_t x) { return (int)((x >> 11) & 0x3FFu); }
__device__ __forceinline__ int node_depth(uint32_t x) { return (int)(x >> 21); }

// Rank-tuple order of two frontier candidates (parent node, child rank); true if a goes first.
// s_node[j] describes tree node j (root: parent field unused, depth 0).
__device__ bool tuple_before(const uint32_t *s_node, int pa, int ra, int pb, int rb)
{
    int da = node_depth(s_node[pa]) + 1, db = node_depth(s_node[pb]) + 1;
    const int da0 = da, db0 = db;
    while (da > db) {
        ra = node_rank(s_node[pa]);
        pa = node_parent(s_node[pa]);
        --da;
    }
    while (db > da) {
        rb = node_rank(s_node[pb]);
        pb = node_parent(s_node[pb]);
        --db;
    }
    while (pa != pb) {
        ra = node_rank(s_node[pa]);
        pa = node_parent(s_node[pa]);
        rb = node_rank(s_node[pb]);
        pb = node_parent(s_node[pb]);
    }
    if (ra != rb) return ra < rb;
    return da0 < db0;
}

template <int NSLOT>
__global__ __launch_bounds__(kBuildThreads) void build_kernel(
    const int32_t *__restrict__ topk_tok, const float *__restrict__ topk_lp, int B, int K, int N,
    const int32_t *__restrict__ root_token, int32_t *__restrict__ tokens,
    int32_t *__restrict__ parent, int32_t *__restrict__ depth, int32_t *__restrict__ rank,
    float *__restrict__ node_score, uint64_t *__restrict__ ancestor_mask,
    int32_t *__restrict__ n_nodes)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int Kp = K + 3;
    const int T = N + 1;
    float *s_lp = reinterpret_cast<float *>(smem);                     // [B][Kp], -inf padded
    uint32_t *s_node = reinterpret_cast<uint32_t *>(s_lp + B * Kp);     // [T]
    float *s_score = reinterpret_cast<float *>(s_node + T);             // [T]
    uint16_t *s_chain = reinterpret_cast<uint16_t *>(s_score + T);      // [B+1][kBuildThreads]
    __shared__ int s_built;

    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const float *lp = topk_lp + (size_t)seq * B * K;
    const int32_t *tk = topk_tok + (size_t)seq * B * K;

    // log-probabilities into LDS, rows padded with -inf; four rows' loads in flight together
    for (int d0 = 0; d0 < B; d0 += 4)
        for (int k0 = 0; k0 < Kp; k0 += kBuildThreads) {
            const int k = k0 + tid;
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = (d0 + r < B && k < K) ? lp[(d0 + r) * K + k] : -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (d0 + r < B && k < Kp) s_lp[(d0 + r) * Kp + k] = v[r];
        }
    if (tid == 0) {
        s_node[0] = pack_node(0, 0, 0);
        s_score[0] = 0.0f;
    }
    __syncthreads();

    if (tid < kWave) {
        const int lane = tid;
        // lane d holds the first two log-probabilities of row d (children of a node at depth
        // d), -inf past the last row: what a fresh entry for a node at depth d needs
        const float lp0 = lane < B ? s_lp[lane * Kp + 0] : -INFINITY;
        const float lp1 = lane < B ? s_lp[lane * Kp + 1] : -INFINITY;
        // Scores are sums of log-probabilities, hence never positive: for such floats a larger
        // value has the smaller bit pattern, so "best candidate" is an unsigned minimum and
        // -inf (0xFF800000) marks an empty entry.
        constexpr uint32_t kEmpty = 0xFF800000u;
        uint32_t cand[NSLOT];   // candidate score bits of the entry (node) in this lane and slot
        float nsc[NSLOT];       // score of the entry's node
        float nlp1[NSLOT];      // lp[row][c+1], prefetched: the increment of the next sibling
        int meta[NSLOT];        // (c << 8) | row: current child rank and the children's row
#pragma unroll
        for (int s = 0; s < NSLOT; ++s) {
            cand[s] = kEmpty;
            nsc[s] = 0.0f;
            nlp1[s] = -INFINITY;
            meta[s] = 0;
        }
        if (lane == 0) {  // the root's entry: candidate = rank 0 of row 0
            cand[0] = __float_as_uint(lp0);
            nlp1[0] = lp1;
        }
        int n = 0;
        int prev_p = -1;  // entry popped by the previous iteration
        while (n < N) {
            // this lane's best entry and that entry's fields (selects, no branches)
            uint32_t lb = cand[0];
            int l_meta = meta[0], l_slot = 0;
            float l_nsc = nsc[0], l_nlp1 = nlp1[0];
#pragma unroll
            for (int s = 1; s < NSLOT; ++s) {
                const bool better = cand[s] < lb;
                lb = better ? cand[s] : lb;
                l_meta = better ? meta[s] : l_meta;
                l_nsc = better ? nsc[s] : l_nsc;
                l_nlp1 = better ? nlp1[s] : l_nlp1;
                l_slot = better ? s : l_slot;
            }
            const uint32_t wmb = wave_min_u32(lb);
            if (wmb == kEmpty) break;  // frontier empty: fewer than N prefixes exist
            // how many entries hold the best score: more than one takes the tie path
            int eqcnt = 0;
#pragma unroll
            for (int s = 0; s < NSLOT; ++s) eqcnt += cand[s] == wmb ? 1 : 0;
            const unsigned long long bal = __ballot(eqcnt > 0);
            const bool tie = __popcll(bal) > 1 || __ballot(eqcnt > 1) != 0ull;
            int wl = __ffsll((long long)bal) - 1;
            int ws, M;
            float NS, NL;
            if (!tie) {
                ws = __builtin_amdgcn_readlane(l_slot, wl);
                M = __builtin_amdgcn_readlane(l_meta, wl);
                NS = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l_nsc), wl));
                NL = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(l_nlp1), wl));
            } else {
                // slow path: several candidates share the best score; the rank-tuple order decides
                int bp = -1, bc = 0;
                ws = 0;
#pragma unroll 1
                for (int s = 0; s < NSLOT; ++s) {
                    unsigned long long mm = 0ull;
#pragma unroll
                    for (int s2 = 0; s2 < NSLOT; ++s2)
                        if (s2 == s) mm = __ballot(cand[s2] == wmb);
                    while (mm) {
                        const int l = __ffsll((long long)mm) - 1;
                        mm &= mm - 1;
                        const int p2 = s * 64 + l;
                        int ms = 0;
#pragma unroll
                        for (int s2 = 0; s2 < NSLOT; ++s2)
                            if (s2 == s) ms = __builtin_amdgcn_readlane(meta[s2], l);
                        const int c2 = ms >> 8;
                        if (bp < 0 || tuple_before(s_node, p2, c2, bp, bc)) {
                            bp = p2;
                            bc = c2;
                            ws = s;
                            wl = l;
                        }
                    }
                }
                M = 0;
                NS = 0.0f;
                NL = 0.0f;
#pragma unroll
                for (int s = 0; s < NSLOT; ++s)
                    if (ws == s) {
                        M = __builtin_amdgcn_readlane(meta[s], wl);
                        NS = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(nsc[s]), wl));
                        NL = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(nlp1[s]), wl));
                    }
            }
            const int p = ws * 64 + wl;
            const int c = M >> 8, row = M & 0xFF, d = row + 1;  // rank, children's row, depth of the new node
            const float wm = __uint_as_float(wmb);
            const float lp0d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lp0), d));
            const float lp1d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lp1), d));
            const bool me = lane == wl;

            // Sibling run.  When the same entry is popped twice in a row (flat distributions pop
            // long runs of consecutive ranks of one parent), pop a whole batch: ranks c .. c+J-1
            // go out in this order as long as each score is strictly above every other frontier
            // entry and above the best child the batch itself creates (the first one's).  Lane j
            // evaluates rank c+j; equal scores end the batch and are left to the tie logic.
            int J = 1;
            float myscore = wm;  // score of rank c + lane (lane 0: the popped candidate itself)
            if (p == prev_p && !tie) {
                uint32_t lb2 = kEmpty;  // best of this lane's entries, the popped one left out
#pragma unroll
                for (int s = 0; s < NSLOT; ++s) lb2 = min(lb2, (me && ws == s) ? kEmpty : cand[s]);
                const float others = __uint_as_float(wave_min_u32(lb2));
                const float bound = fmaxf(others, wm + lp0d);
                myscore = NS + s_lp[row * Kp + min(c + lane, Kp - 1)];  // -inf past rank K-1
                const unsigned long long okm = __ballot(lane == 0 || myscore > bound);
                J = ~okm == 0ull ? 64 : __ffsll((long long)~okm) - 1;
                J = min(J, N - n);
            }
            prev_p = p;
            // the popped entry moves on to rank c + J ("push next sibling"): its new candidate and
            // the log-probability after it
            const float p_inc = J == 1 ? NL : s_lp[row * Kp + min(c + J, Kp - 1)];  // -inf once c+J >= K
            const float p_nlp1 = s_lp[row * Kp + min(c + J + 1, Kp - 1)];
            // records of nodes n+1 .. n+J
            if (lane < J) {
                s_node[n + 1 + lane] = pack_node(p, c + lane, d);
                s_score[n + 1 + lane] = myscore;
            }
            // their frontier entries ("push first child"): entry e = n+1+j lives in lane e % 64,
            // slot e / 64; lane j's score travels there
            const int j_here = (lane - (n + 1)) & 63;
            const float sc_e = J == 1 ? wm : __shfl(myscore, j_here, 64);
            const int slot_e = j_here < J ? (n + 1 + j_here) >> 6 : -1;
            const uint32_t e_cand = __float_as_uint(sc_e + lp0d);  // -inf once d == B
            const uint32_t p_cand = __float_as_uint(NS + p_inc);
            const int p_meta = M + (J << 8);
#pragma unroll
            for (int s = 0; s < NSLOT; ++s) {
                const bool fresh = slot_e == s;
                const bool popped = me && ws == s;
                cand[s] = fresh ? e_cand : popped ? p_cand : cand[s];
                nsc[s] = fresh ? sc_e : nsc[s];
                nlp1[s] = fresh ? lp1d : popped ? p_nlp1 : nlp1[s];
                meta[s] = fresh ? d : popped ? p_meta : meta[s];  // fresh: rank 0, children read row d
            }
            n += J;
        }
        if (lane == 0) s_built = n;
    }
    __syncthreads();
    const int built = s_built;
    const int W = (T + 63) / 64;
    if (tid == 0) n_nodes[seq] = built;

    for (int i0 = 0; i0 < T; i0 += kBuildThreads) {
        const int i = i0 + tid;
        if (i >= T) break;
        const size_t o = (size_t)seq * T + i;
        uint64_t *mrow = ancestor_mask + o * W;
        if (i > built) {
            tokens[o] = -1;
            parent[o] = -1;
            depth[o] = -1;
            if (rank) rank[o] = -1;
            if (node_score) node_score[o] = 0.0f;
            for (int w = 0; w < W; ++w) mrow[w] = 0ull;
            continue;
        }
        const uint32_t nd = s_node[i];
        const int d = i == 0 ? 0 : node_depth(nd);
        if (i == 0) {
            tokens[o] = root_token[seq];
            parent[o] = -1;
            depth[o] = 0;
            if (rank) rank[o] = -1;
            if (node_score) node_score[o] = 0.0f;
        } else {
            tokens[o] = tk[(d - 1) * K + node_rank(nd)];
            parent[o] = node_parent(nd);
            depth[o] = d;
            if (rank) rank[o] = node_rank(nd);
            if (node_score) node_score[o] = s_score[i];
        }
        // ancestors of i (itself first, the root last): d + 1 ids, kept in this thread's
        // column of s_chain, then folded into the W mask words
        int j = i;
        for (int t = 0; t <= d; ++t) {
            s_chain[t * kBuildThreads + tid] = (uint16_t)j;
            j = node_parent(s_node[j]);
        }
        for (int w = 0; w < W; ++w) {
            uint64_t word = 0ull;
            for (int t = 0; t <= d; ++t) {
                const int a = s_chain[t * kBuildThreads + tid];
                if ((a >> 6) == w) word |= 1ull << (a & 63);
            }
            mrow[w] = word;
        }
    }
}

static size_t build_lds_bytes(int B, int K, int N)
{
    return (size_t)B * (K + 3) * 4 + (size_t)(N + 1) * 8 + (size_t)(B + 1) * kBuildThreads * 2;
}

template <int NSLOT>
static int launch_build(const int32_t *topk_tok, const float *topk_lp, int batch, int B, int K, int N,
                        const int32_t *root_token, int32_t *tokens, int32_t *parent, int32_t *depth,
                        int32_t *rank, float *node_score, uint64_t *ancestor_mask, int32_t *n_nodes,
                        hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(build_kernel<NSLOT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) != hipSuccess)
            return DDTREE_ERR_HIP;
        attr_set = true;
    }
    DDT_LAUNCH(DDTREE_KERNEL_BUILD, st, build_kernel<NSLOT>, dim3(batch), dim3(kBuildThreads), build_lds_bytes(B, K, N),
                       st, topk_tok, topk_lp, B, K, N, root_token, tokens, parent, depth, rank,
                       node_score, ancestor_mask, n_nodes);
    return launch_status();
}

}  // namespace ddt

extern "C" int ddtree_build(const int32_t *topk_tok, const float *topk_lp, int batch, int B, int K,
                            int N, const int32_t *root_token, int32_t *tokens, int32_t *parent,
                            int32_t *depth, int32_t *rank, float *node_score,
                            uint64_t *ancestor_mask, int32_t *n_nodes, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    using namespace ddt;
    (void)workspace;
    (void)workspace_bytes;
    if (!topk_tok || !topk_lp || !root_token || !tokens || !parent || !depth || !ancestor_mask ||
        !n_nodes)
        return DDTREE_ERR_ARG;
    if (batch < 1 || batch > DDTREE_MAX_BATCH || B < 1 || B > DDTREE_MAX_B || K < 1 ||
        K > DDTREE_MAX_N || N < 1 || N > DDTREE_MAX_N)
        return DDTREE_ERR_ARG;
    if (build_lds_bytes(B, K, N) > 150 * 1024) return DDTREE_ERR_ARG;
    hipStream_t st = as_stream(stream);
    const int slots = (N + 1 + 63) / 64;
#define DDT_BUILD(S)                                                                              \
    return launch_build<S>(topk_tok, topk_lp, batch, B, K, N, root_token, tokens, parent, depth, \
                           rank, node_score, ancestor_mask, n_nodes, st)
    if (slots <= 1) DDT_BUILD(1);
    if (slots <= 2) DDT_BUILD(2);
    if (slots <= 3) DDT_BUILD(3);
    if (slots <= 5) DDT_BUILD(5);
    if (slots <= 9) DDT_BUILD(9);
    DDT_BUILD(17);
#undef DDT_BUILD
}
