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
#include <atomic>

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

// ------------------------------------------------------------------------------------------
// Level-synchronous construction.
//
// The tree is the set of the N best prefixes (Proposition 2) under the total order "score
// descending, then rank tuple", and the pop order of Algorithm 1 is that order.  Instead of N
// dependent pops, the workgroup works depth by depth:
//   * "alive" is a score bucket cut: the score range [lp[0][N-1], lp[0][0]] is divided into 256
//     equal buckets (bucket 0 the best; one more bucket takes everything below the range), a
//     histogram of every prefix known so far is kept, and the cut b* is the first bucket at which
//     the cumulative count reaches N.  At least N prefixes lie at or above the cut, so a prefix
//     below it is not in the tree, nor is any descendant (scores only fall along a path).  b* only
//     moves up.  "Known" is more than "found": a prefix found with rank >= 1 brings its top-1
//     continuation with it (see count_continuation), which on peaked rows, where most nodes are
//     rank-0 children, puts the cut near its final place after the first level.
//   * level d: every alive depth-(d-1) member finds, by bisection over its (sorted) row, how
//     many of its children lie at or above the cut; the children are written out, bucketed, the
//     cut is updated, and the children above the new cut join the members.
//   * a parent with j better members of the same depth cannot have its child of rank b in the
//     tree once (j+1)(b+1) > N (every (better parent, lower rank) pair goes first), so its
//     children are cut at N/(j+1); j is taken from the bucket counts (a lower bound, hence a
//     looser cut).  Rounding can merge scores and void that counting argument, so the first child
//     left out of each cut is checked against the final cut of its level; if it would have
//     survived, the construction gives up.
//   * the end: the members above the cut are ranked exactly (bucket position plus an all-pairs
//     count inside the bucket, ties by rank tuple) and the first N become nodes 1..N.
//   * levels with at most 64 parents are run by one wave without barriers (see wave_levels); a
//     level whose candidates do not fit their arrays is counted by bucket first, the cut moves,
//     and its children are counted again.
//   * where the prefixes entered up front already give a cut (peaked rows), the members are not
//     found depth by depth at all but by generations: by the number of their non-zero ranks, of
//     which there are at most log2(N + 1) + 1 (see by_generations).
// Giving up (a cut that cannot be proven, or a capacity that heavy ties exceed) returns -1 and
// the caller runs the sequential pops instead.
// ------------------------------------------------------------------------------------------
__device__ unsigned int g_level_giveups;  // sequences the level construction handed to the pops

constexpr int kLvBuckets = 256;
constexpr float kLvNeg = -3.0e38f;   // scores at or below count as -inf: never part of a tree
constexpr int kLvSmall = 8;          // parents with at most this many children write them alone
constexpr int kLvSeedRanksMax = 64;  // at most so many ranks off the top-1 chain are entered before the first level
constexpr int kLvBigCap = 256;

__device__ __forceinline__ uint32_t pack_member(int parent, int rank, int depth)
{
    return (uint32_t)parent | ((uint32_t)rank << 13) | ((uint32_t)depth << 23);
}
__device__ __forceinline__ int member_parent(uint32_t x) { return (int)(x & 0x1FFFu); }
__device__ __forceinline__ int member_rank(uint32_t x) { return (int)((x >> 13) & 0x3FFu); }
__device__ __forceinline__ int member_depth(uint32_t x) { return (int)(x >> 23); }

struct LevelMem {
    float *m_score;     // [capm] member scores; member 0 is the root
    uint32_t *m_info;   // [capm] (parent member, rank, depth)
    uint16_t *m_jlo;    // [capm] lower bound on the better members of the same depth
    uint16_t *p_c;      // [capp] per parent of the level: child count | cut flag
    uint16_t *p_off;    // [capp] per parent: its first candidate (p_off = p_c + capp; together
                        // they hold the renumbering table when members are squeezed: capm <= 2 capp)
    float *c_score;     // [capc] candidates of the level; at the end, as u16: node id per member
    uint32_t *c_info;   // [capc]; at the end, as u16: the members sorted by bucket
    int capm, capp, capc;  // capm <= 2 * capc
};

// a goes before b in the total order (score, then rank tuple, a prefix before its extensions)
__device__ bool member_before(const float *m_score, const uint32_t *m_info, int a, int b)
{
    const float sa = m_score[a], sb = m_score[b];
    if (sa != sb) return sa > sb;
    uint32_t ia = m_info[a], ib = m_info[b];
    int da = member_depth(ia), db = member_depth(ib);
    const int da0 = da, db0 = db;
    int ra = member_rank(ia), rb = member_rank(ib);
    int pa = member_parent(ia), pb = member_parent(ib);
    while (da > db) {
        ia = m_info[pa];
        ra = member_rank(ia);
        pa = member_parent(ia);
        --da;
    }
    while (db > da) {
        ib = m_info[pb];
        rb = member_rank(ib);
        pb = member_parent(ib);
        --db;
    }
    while (pa != pb) {
        ia = m_info[pa];
        ra = member_rank(ia);
        pa = member_parent(ia);
        ib = m_info[pb];
        rb = member_rank(ib);
        pb = member_parent(ib);
    }
    if (ra != rb) return ra < rb;
    return da0 < db0;
}

// Exclusive prefix sum over the workgroup's kBuildThreads values; *total = their sum.
__device__ __forceinline__ int build_block_scan(int v, int *s_w, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_scan_inclusive_i32(v);
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kBuildThreads / 64; ++w) {
        const int x = s_w[w];
        base += w < wave ? x : 0;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// The same for two values at once; *a and *b are replaced by their exclusive prefixes.
__device__ __forceinline__ void build_block_scan2(int *a, int *b, int (*s_w2)[kBuildThreads / 64],
                                                  int *total_a, int *total_b)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ia = wave_scan_inclusive_i32(*a), ib = wave_scan_inclusive_i32(*b);
    if (lane == 63) {
        s_w2[0][wave] = ia;
        s_w2[1][wave] = ib;
    }
    __syncthreads();
    int base_a = 0, base_b = 0, ta = 0, tb = 0;
#pragma unroll
    for (int w = 0; w < kBuildThreads / 64; ++w) {
        const int xa = s_w2[0][w], xb = s_w2[1][w];
        base_a += w < wave ? xa : 0;
        base_b += w < wave ? xb : 0;
        ta += xa;
        tb += xb;
    }
    __syncthreads();
    *total_a = ta;
    *total_b = tb;
    *a = base_a + ia - *a;
    *b = base_b + ib - *b;
}

// Returns the number of nodes written to s_node / s_score (ids 1..n), or -1 after giving up.
__device__ int level_build(const float *s_lp, int Kp, int B, int K, int N, LevelMem L,
                           uint32_t *s_node, float *s_score)
{
    static_assert(kBuildThreads == kLvBuckets, "one bucket per thread");
    __shared__ __align__(16) int s_hist[kLvBuckets + 4];    // every prefix known so far, by bucket
    __shared__ __align__(16) int s_histc[kLvBuckets + 4];   // the candidates of the level; at the end: cursors
    __shared__ __align__(16) int s_histv[kLvBuckets + 4];   // the prefixes the level makes known
    __shared__ __align__(16) int s_pref[kLvBuckets + 4];    // exclusive prefix of s_histc, later of s_hist
    __shared__ int s_state[8];                // what the single-wave levels hand back to the workgroup
    __shared__ float s_cc[DDTREE_MAX_B + 1];  // scores of the top-1 chain's nodes
    __shared__ int s_w[kBuildThreads / 64];
    __shared__ int s_w2[2][kBuildThreads / 64];
    __shared__ int s_M, s_fail, s_nbig, s_bstar, s_chain;
    __shared__ uint16_t s_big[kLvBigCap];
    constexpr int NT = kBuildThreads;
    const int tid = threadIdx.x;

    if (tid == 0) {
        L.m_score[0] = 0.0f;
        L.m_info[0] = pack_member(0, 0, 0);
        L.m_jlo[0] = 0;
        s_M = 1;
        s_fail = 0;
    }
    s_hist[tid] = 0;
    if (tid == 0) s_hist[kLvBuckets] = 0;
    const float hi = s_lp[0];
    // lower end of the bucket range: with K >= N the N-th rank of row 0 is a lower bound on the
    // N-th best score; with fewer ranks than budget there is no such bound and a fixed span of 48
    // (nats) below the best score stands in (scores further down share the overflow bucket)
    const float lo_raw = s_lp[min(K, N) - 1];
    const float lo = (K >= N && lo_raw > kLvNeg) ? lo_raw : hi - 48.0f;
    // lo itself maps to the middle of the last regular bucket; scores further down go to bucket
    // kLvBuckets.  Monotone in the score: subtraction, scaling, clamping and truncation all
    // preserve order.
    const float inv = ((float)kLvBuckets - 0.5f) / fmaxf(hi - lo, 1e-30f);
    auto bucket_of = [&](float sc) { return (int)fminf((hi - sc) * inv, (float)kLvBuckets); };
    __syncthreads();
    // Known prefixes.  A prefix found with rank >= 1 makes its whole top-1 continuation known (the
    // same prefix followed by rank 0 at every further depth: real, distinct prefixes whose scores
    // are the running sums the construction itself will form), so the histogram takes those at
    // once and the cut settles levels earlier than the candidates alone would move it; a rank-0
    // child is then already counted when it turns up.  Continuations below the cut of the
    // moment are of no interest (the cut only tightens) and end the walk.  The increments are
    // fetched eight at a time: the running sum is the only dependency from step to step.
    auto count_continuation = [&](int *hist, float sc, int depth, int cutb) {
        float v = sc;
        bool live = true;
        for (int t0 = depth; t0 < B && live; t0 += 8) {
            float inc[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) inc[k] = s_lp[min(t0 + k, B - 1) * Kp];
            // (the empty statements keep the eight fetches together, ahead of the steps: sunk
            // into the steps each would wait for its own round trip and for the update before it)
#pragma unroll
            for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(inc[k]));
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                v += inc[k];
                const int b = bucket_of(v);
                live = live && t0 + k < B && v > kLvNeg && b <= cutb;
                // (a finished walk adds zero, to a word of its own: no branch, no shared address)
                atomicAdd(&hist[live ? b : (int)(threadIdx.x & 63)], live ? 1 : 0);
            }
        }
    };
    // Before the first level: the top-1 chain (the root's continuation) and, off every node of
    // that chain, the children of ranks 1 .. seed_ranks with their continuations, one (row,
    // rank) per thread and pass.  On peaked rows these are most of the tree, and the
    // first level already starts from a cut near the final one.  When they turn up as candidates
    // they are not counted again (the children of the chain's member, chain_m below, up to that
    // rank).  With K >= N the final cut lies inside the bucket range (the N children of the
    // root do), so whatever falls below the range is left out, here and in every later walk (all
    // of it would land in the one overflow bucket, lane after lane); otherwise everything is counted.
    const int cutb0 = (K >= N && lo_raw > kLvNeg) ? kLvBuckets - 1 : kLvBuckets;
    // None of this pays when the top-1 chain leaves the bucket range within three steps (flat
    // rows: continuations are out of range almost at once): then nothing is entered ahead, every
    // candidate counts when it is found, rank 0 included, and no continuation is walked.
    const float chain3 = B >= 3 ? (s_lp[0] + s_lp[Kp]) + s_lp[2 * Kp] : -INFINITY;
    const bool walks = chain3 > kLvNeg && bucket_of(chain3) < kLvBuckets;
    // ranks 1 .. seed_ranks off the chain are entered: 16 up to N = 256, N/16 beyond (at most 64)
    const int seed_ranks = min(kLvSeedRanksMax, max(32, N >> 3));
    if (walks) {
        // scores of the chain's nodes, summed in path order by one thread (the row maxima fetched
        // eight at a time, as in the walk above): s_cc[i] = node at depth i, s_cc[0] = 0
        if (tid == 0) {
            float cc = 0.0f;
            s_cc[0] = 0.0f;
            for (int u0 = 0; u0 < B; u0 += 8) {
                float inc[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) inc[k] = s_lp[min(u0 + k, B - 1) * Kp];
#pragma unroll
                for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(inc[k]));
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (u0 + k < B) {
                        cc += inc[k];
                        s_cc[u0 + k + 1] = cc;
                    }
            }
        }
        __syncthreads();
        // the chain itself (the scores fall along it, so the test is that of a walk that stops)
        if (tid >= 1 && tid <= B) {
            const float sc = s_cc[tid];
            const int b = bucket_of(sc);
            if (sc > kLvNeg && b <= cutb0) atomicAdd(&s_hist[b], 1);
        }
        // heads (row i, rank r): one per thread and pass
        const int n_heads = B * seed_ranks;
        for (int hx = tid; hx < n_heads; hx += NT) {
            const int i = hx / seed_ranks, r = 1 + hx % seed_ranks;
            if (r >= K) continue;
            const float head = s_cc[i] + s_lp[i * Kp + r];
            const int b = bucket_of(head);
            if (head > kLvNeg && b <= cutb0) {
                atomicAdd(&s_hist[b], 1);
                count_continuation(s_hist, head, i + 1, cutb0);
            }
        }
    }
    __syncthreads();

    // Children of a parent with score S that lie at or above the cut: a prefix of the sorted row,
    // at most cap long.  The first four ranks are probed in one round (most parents of a deep tree
    // have a few children at most); then eight probes at doubling distances bracket the count,
    // and a 9-ary search (eight independent probes per round) closes the bracket.
    // (four_only: stop after the first round, a result of 4 with cap > 4 then means "at least 4";
    // past_four: the first round is known to have passed)
    auto count_children = [&](const float *row, float S, int cap, int cutb, bool past_four = false,
                              bool four_only = false) {
        auto child_ok = [&](int r) {
            const float sc = S + row[r];
            return sc > kLvNeg && bucket_of(sc) <= cutb;
        };
        // first failing probe of eight increasing ones (the answers are monotone): the count lies
        // in [q[f-1] + 1, q[f]], with q[-1] + 1 = a and q[8] = b
        auto narrow8 = [&](const int (&q)[8], int &a, int &b) {
            bool ok[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) ok[k] = child_ok(q[k]);
            int f = 8;
#pragma unroll
            for (int k = 7; k >= 0; --k) f = ok[k] ? f : k;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k < f) a = q[k] + 1;
                if (k == f) b = q[k];
            }
        };
        if (!past_four) {
            bool lead[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) lead[k] = child_ok(min(k, cap - 1));
            const int n_lead = !lead[0] ? 0 : !lead[1] ? 1 : !lead[2] ? 2 : !lead[3] ? 3 : 4;
            if (n_lead < 4 || cap <= 4 || four_only) return min(n_lead, cap);
        }
        int a = 4, b = cap;  // the count lies in [a, b]
        {
            int q[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) q[k] = min(4 + (1 << k), cap - 1);  // ranks 5, 6, 8, 12, 20, 36, 68, 132
            narrow8(q, a, b);
        }
        while (a < b) {
            const int len = b - a;
            const int step = len <= 8 ? 1 : (len + 8) / 9;
            int q[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) q[k] = min(a + (k + 1) * step - 1, b - 1);
            narrow8(q, a, b);
        }
        return a;
    };

    int bstar = kLvBuckets;  // alive <=> bucket <= bstar
    int M = 1, ls = 0, le = 1;   // members so far; the previous level's members are [ls, le)
    int d = 1;
    int chain_m = 0;    // the member that is the top-1 chain's node of the previous level, -1 once it is dead
    int C_resume = -1;  // >= 0: level d was taken through its cut check by the single wave below
                        // and the workgroup continues with its C_resume candidates

    // a candidate that makes itself and its continuation known: rank >= 1 and not entered up front
    auto newly_known = [&](int parent_m, int r) {
        return !walks || (r > 0 && !(parent_m == chain_m && r <= seed_ranks));
    };

    // (the two helpers below are for wave 0 alone: lane = thread)
    const int lane = tid;
    // the cut: lane l adds what the level made known in buckets 4l .. 4l+3 to the running
    // histogram, takes the prefix sums and finds the bucket of the N-th best known prefix
    auto move_cut = [&]() {
        const int4 hc = *reinterpret_cast<const int4 *>(&s_histc[4 * lane]);
        const int4 hv = *reinterpret_cast<const int4 *>(&s_histv[4 * lane]);
        int4 ha = *reinterpret_cast<const int4 *>(&s_hist[4 * lane]);
        ha.x += hv.x;
        ha.y += hv.y;
        ha.z += hv.z;
        ha.w += hv.w;
        const int ta = ha.x + ha.y + ha.z + ha.w, tc = hc.x + hc.y + hc.z + hc.w;
        const int ia = wave_scan_inclusive_i32(ta), ic = wave_scan_inclusive_i32(tc);
        const int a0 = ia - ta, a1 = a0 + ha.x, a2 = a1 + ha.y, a3 = a2 + ha.z;
        const int c0 = ic - tc;
        *reinterpret_cast<int4 *>(&s_hist[4 * lane]) = ha;
        *reinterpret_cast<int4 *>(&s_pref[4 * lane]) = make_int4(c0, c0 + hc.x, c0 + hc.x + hc.y, c0 + hc.x + hc.y + hc.z);
        if (lane == 63) {
            s_pref[kLvBuckets] = ic;
            s_hist[kLvBuckets] += s_histv[kLvBuckets];
        }
        // (at most one bucket qualifies)
        uint32_t bn = (uint32_t)kLvBuckets;
        if (a0 < N && a0 + ha.x >= N) bn = 4 * lane;
        if (a1 < N && a1 + ha.y >= N) bn = 4 * lane + 1;
        if (a2 < N && a2 + ha.z >= N) bn = 4 * lane + 2;
        if (a3 < N && a3 + ha.w >= N) bn = 4 * lane + 3;
        bstar = min(bstar, (int)wave_min_u32(bn));
    };
    auto clear_level = [&]() {
        const int4 z = make_int4(0, 0, 0, 0);
        *reinterpret_cast<int4 *>(&s_histc[4 * lane]) = z;
        *reinterpret_cast<int4 *>(&s_histv[4 * lane]) = z;
        if (lane == 0) s_histc[kLvBuckets] = s_histv[kLvBuckets] = 0;
    };

    // The cut that the prefixes entered up front give (wave 0; the others wait for it).
    if (tid < kWave) {
        clear_level();
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        move_cut();
        if (tid == 0) s_state[5] = bstar;
    }
    __syncthreads();
    bstar = s_state[5];

    // By generations.  Where the up-front entries already give a cut (peaked rows), the members --
    // every prefix at or above it -- are enumerated by the number of their non-zero ranks instead
    // of by depth: generation g + 1 is found from generation g in one step of the whole workgroup,
    // and there are at most log2(N + 1) + 1 generations (a prefix with g non-zero ranks has 2^g - 1
    // better ones: itself with any subset of them set to rank 0), two or three on a tree from a
    // confident drafter, against B levels.  One step: (A) every head of the generation (a member
    // that ends in a non-zero rank; the root for generation 0) walks its top-1 continuation while
    // it stays at or above the cut, and those nodes become members; (B) every head and every
    // continuation node counts its children of rank >= 1 at or above the cut (a prefix of its
    // sorted row): they are the heads of the next generation.  The cut is left where it is
    // (allowed: see the settled levels below), so nothing is bucketed and no histogram is kept;
    // if that lets in far more members than a tight cut would (beyond 3.5 N + 64), the
    // construction starts over level by level; a smaller surplus is shed when the members are
    // ranked.  Returns the number of members, or -1.
    auto by_generations = [&]() -> int {
        const int limit = min(L.capm, 3 * N + N / 2 + 64);
        const int cap = min(K, N);
        auto alive = [&](float v) { return v > kLvNeg && bucket_of(v) <= bstar; };
        int hs = 0, he = 1, Mg = 1;
        if (tid == 0) s_nbig = 0;  // (the scan below has barriers before the first use)
        for (;;) {
            // A. the continuations of the heads [hs, he)
            const int n_heads = he - hs;
            const int chain_base = Mg;
            int Cn = 0;
            for (int i0 = 0; i0 < n_heads; i0 += NT) {
                const int i = i0 + tid, h = hs + i;
                float S = 0.0f;
                int dh = 0, len = 0;
                if (i < n_heads) {
                    S = L.m_score[h];
                    dh = member_depth(L.m_info[h]);
                    float v = S;
                    bool live = true;
                    for (int t0 = dh; t0 < B && live; t0 += 8) {
                        float inc[8];
#pragma unroll
                        for (int k = 0; k < 8; ++k) inc[k] = s_lp[min(t0 + k, B - 1) * Kp];
#pragma unroll
                        for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(inc[k]));
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            v += inc[k];
                            live = live && t0 + k < B && alive(v);
                            len += live ? 1 : 0;
                        }
                    }
                }
                int total;
                const int off = Cn + build_block_scan(len, s_w, &total);
                if (chain_base + Cn + total > limit) return -1;  // (before anything of it is written)
                if (len > 0) {
                    float v = S;
                    for (int j = 0; j < len; ++j) {
                        v += s_lp[(dh + j) * Kp];
                        const int id = chain_base + off + j;
                        L.m_score[id] = v;
                        L.m_info[id] = pack_member(j == 0 ? h : id - 1, 0, dh + 1 + j);
                        L.m_jlo[id] = 0;
                    }
                }
                Cn += total;
            }
            Mg = chain_base + Cn;
            __syncthreads();
            // B. the children of rank >= 1 of the heads and of their continuation nodes
            const int n_par = n_heads + Cn;
            const int head_base = Mg;
            int H = 0;
            for (int p0 = 0; p0 < n_par; p0 += NT) {
                const int p = p0 + tid;
                const int pm = p < n_heads ? hs + p : chain_base + (p - n_heads);
                float S = 0.0f;
                int dp = 0, c = 0;
                if (p < n_par) {
                    S = L.m_score[pm];
                    dp = member_depth(L.m_info[pm]);
                    if (dp < B) c = max(0, count_children(s_lp + dp * Kp, S, cap, bstar) - 1);
                }
                int total;
                const int off = H + build_block_scan(c, s_w, &total);
                if (head_base + H + total > limit) return -1;
                // small families are written by their parent's thread, large ones are queued and
                // written by the whole workgroup (s_nbig is 0 here: see the end of the round)
                bool own = c > 0;
                if (c > kLvSmall) {
                    const int slot = atomicAdd(&s_nbig, 1);
                    if (slot < kLvBigCap) {
                        s_big[slot] = (uint16_t)pm;
                        L.p_c[slot] = (uint16_t)c;
                        L.p_off[slot] = (uint16_t)off;  // (below limit <= capm <= 8192)
                        own = false;
                    }
                }
                if (own) {
                    const float *row = s_lp + dp * Kp;
                    for (int r = 1; r <= c; ++r) {
                        const int id = head_base + off + r - 1;
                        L.m_score[id] = S + row[r];
                        L.m_info[id] = pack_member(pm, r, dp + 1);
                        L.m_jlo[id] = 0;
                    }
                }
                __syncthreads();
                const int nbig = min(s_nbig, kLvBigCap);
                for (int qb = 0; qb < nbig; ++qb) {
                    const int bpm = s_big[qb], bc = L.p_c[qb], boff = L.p_off[qb];
                    const float bS = L.m_score[bpm];
                    const int bdp = member_depth(L.m_info[bpm]);
                    const float *row = s_lp + bdp * Kp;
                    for (int r = 1 + tid; r <= bc; r += NT) {
                        const int id = head_base + boff + r - 1;
                        L.m_score[id] = bS + row[r];
                        L.m_info[id] = pack_member(bpm, r, bdp + 1);
                        L.m_jlo[id] = 0;
                    }
                }
                __syncthreads();
                if (tid == 0) s_nbig = 0;
                H += total;
            }
            __syncthreads();
            hs = head_base;
            he = head_base + H;
            Mg = he;
            if (H == 0) return Mg;
        }
    };

    // Levels with at most 64 parents are run by wave 0 alone, as many in a row as there are: no
    // barriers, prefix sums and the compaction of survivors by cross-lane operations, the level's
    // histogram filled while the candidates are written.  LDS operations of one wave execute in
    // program order, so a lane reads what another lane of the wave wrote by an earlier
    // instruction; the wavefront-scope fences keep the compiler from reordering them.  Hands back
    // 0: level d has more than 64 parents; 1: no level is left; 2: level d needs members squeezed
    // out before its survivors fit (state[6] = its candidate count); -1: give up.
    auto wave_levels = [&]() {
        int status = 1, C_out = 0;
        bool calm = false;    // the last level that moved the cut left it where it was
        int fresh_total = 0;  // prefixes made known since
        for (; d <= B; ++d) {
            const int n_par = le - ls;
            // (a first level without a cut takes every rank of row 0 and walks the continuation
            // of most: work for the whole workgroup)
            if (n_par > kWave || (d == 1 && bstar == kLvBuckets && min(K, N) > kWave)) {
                status = 0;
                break;
            }
            const float *row = s_lp + (d - 1) * Kp;
            clear_level();
            const int m = ls + lane;
            int c = 0, cap = 0;
            bool cut = false, open = false;
            float S = 0.0f;
            if (lane < n_par) {
                S = L.m_score[m];
                if (m == 0 || bucket_of(S) <= bstar) {
                    const int jlo = L.m_jlo[m];
                    cap = N;
                    if (jlo != 0) cap = max(1, N / (jlo + 1));  // (members of settled levels carry 0)
                    cap = min(K, cap);
                    c = count_children(row, S, cap, bstar, false, true);
                    open = c == 4 && cap > 4;
                }
            }
            // Parents with more than four children: a few of them (a deep tree has the chain's
            // node and little else) are finished one after the other by the whole wave, lane j
            // probing rank 4 + j, which takes one round per 64 ranks; many of them each finish
            // their own search.
            {
                unsigned long long om = __ballot(open);
                if (__popcll(om) > 8) {
                    if (open) c = count_children(row, S, cap, bstar, true);
                } else {
                    while (om) {
                        const int src = __ffsll((long long)om) - 1;
                        om &= om - 1;
                        const float pS = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(S), src));
                        const int pcap = __builtin_amdgcn_readlane(cap, src);
                        int cnt = pcap;
                        for (int base = 4; base < pcap; base += kWave) {
                            const int r = base + lane;
                            bool ok = false;
                            if (r < pcap) {
                                const float sc = pS + row[r];
                                ok = sc > kLvNeg && bucket_of(sc) <= bstar;
                            }
                            const unsigned long long okm = __ballot(ok);
                            if (~okm != 0ull) {
                                cnt = min(pcap, base + __ffsll((long long)~okm) - 1);
                                break;
                            }
                        }
                        if (lane == src) c = cnt;
                    }
                }
            }
            cut = cap > 0 && c == cap && cap < K;
            const int incl = wave_scan_inclusive_i32(c);
            const int C = __builtin_amdgcn_readlane(incl, 63);
            const int off = incl - c;
            if (C == 0) break;
            if (C > L.capc) {  // too many to hold: the workgroup's path knows what to do
                status = 0;
                break;
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            // The cut has settled (on a deep tree: from the first level or two on): the level
            // leaves the cut alone, its candidates are alive as they stand and become members
            // directly.  What it makes known still enters the histogram, and once that adds up
            // the next level moves the cut again.  A rank cut that the cut as it is cannot
            // justify sends the level the long way (moving the cut may justify it).
            bool settled = calm && M + C <= L.capm;
            if (settled) {
                bool bad = false;
                if (cut) {
                    const float sc = S + row[c];
                    bad = sc > kLvNeg && bucket_of(sc) <= bstar;
                }
                settled = __ballot(bad) == 0ull;
            }
            if (settled) {
                int fresh = 0;
                // small families rank by rank, as many ranks as the largest of them has (on a
                // deep tree one or two: a wave runs its instructions one after the other, so a
                // step that no lane needs is best not issued at all)
                const int csmall = c <= kLvSmall ? c : 0;
#pragma unroll 1
                for (int r = 0; __ballot(r < csmall) != 0ull; ++r)
                    if (r < csmall) {
                        const float sc = S + row[r];
                        L.m_score[M + off + r] = sc;
                        L.m_info[M + off + r] = pack_member(m, r, d);
                        L.m_jlo[M + off + r] = 0;
                        if (newly_known(m, r)) {
                            atomicAdd(&s_hist[bucket_of(sc)], 1);
                            if (walks) count_continuation(s_hist, sc, d, min(bstar, cutb0));
                            ++fresh;
                        }
                    }
                unsigned long long bigf = __ballot(c > kLvSmall);
                while (bigf) {
                    const int src = __ffsll((long long)bigf) - 1;
                    bigf &= bigf - 1;
                    const int bc = __builtin_amdgcn_readlane(c, src), boff = __builtin_amdgcn_readlane(off, src);
                    const float bS = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(S), src));
                    for (int r = lane; r < bc; r += kWave) {
                        const float sc = bS + row[r];
                        L.m_score[M + boff + r] = sc;
                        L.m_info[M + boff + r] = pack_member(ls + src, r, d);
                        L.m_jlo[M + boff + r] = 0;
                        if (newly_known(ls + src, r)) {
                            atomicAdd(&s_hist[bucket_of(sc)], 1);
                            if (walks) count_continuation(s_hist, sc, d, min(bstar, cutb0));
                            ++fresh;
                        }
                    }
                }
                fresh_total += __popcll(__ballot(fresh > 0));  // (lanes, not prefixes: a rough gauge is enough)
                if (16 * fresh_total > N) {
                    calm = false;
                    fresh_total = 0;
                }
                // the chain's next member: the rank-0 child of the chain's member, if it has one
                const unsigned long long chm = __ballot(lane < n_par && m == chain_m && c > 0);
                chain_m = chm != 0ull ? M + __builtin_amdgcn_readlane(off, __ffsll((long long)chm) - 1) : -1;
                ls = M;
                M += C;
                le = M;
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                continue;
            }
            const int bstar_before = bstar;
            // candidates: small families by their parent's lane, large ones by the whole wave
            if (c <= kLvSmall) {
                float v[kLvSmall];
#pragma unroll
                for (int r = 0; r < kLvSmall; ++r) v[r] = row[min(r, K - 1)];
#pragma unroll
                for (int r = 0; r < kLvSmall; ++r)
                    if (r < c) {
                        const float sc = S + v[r];
                        L.c_score[off + r] = sc;
                        L.c_info[off + r] = pack_member(m, r, d);
                        const int bk = bucket_of(sc);
                        atomicAdd(&s_histc[bk], 1);
                        if (newly_known(m, r)) {
                            atomicAdd(&s_histv[bk], 1);
                            if (walks) count_continuation(s_histv, sc, d, min(bstar, cutb0));
                        }
                    }
            }
            unsigned long long bigm = __ballot(c > kLvSmall);
            while (bigm) {
                const int src = __ffsll((long long)bigm) - 1;
                bigm &= bigm - 1;
                const int bc = __builtin_amdgcn_readlane(c, src), boff = __builtin_amdgcn_readlane(off, src);
                const float bS = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(S), src));
                for (int r = lane; r < bc; r += kWave) {
                    const float sc = bS + row[r];
                    L.c_score[boff + r] = sc;
                    L.c_info[boff + r] = pack_member(ls + src, r, d);
                    const int bk = bucket_of(sc);
                    atomicAdd(&s_histc[bk], 1);
                    if (newly_known(ls + src, r)) {
                        atomicAdd(&s_histv[bk], 1);
                        if (walks) count_continuation(s_histv, sc, d, min(bstar, cutb0));
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            move_cut();
            // every rank cut must have left out only children below the new cut
            {
                bool bad = false;
                if (cut) {
                    const float sc = S + row[c];
                    bad = sc > kLvNeg && bucket_of(sc) <= bstar;
                }
                if (__ballot(bad) != 0ull) {
                    status = -1;
                    break;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            const int n_surv = s_pref[bstar] + s_histc[bstar];
            if (M + n_surv > L.capm) {
                status = 2;
                C_out = C;
                break;
            }
            // candidates at or above the cut become members, in candidate order
            int base = M, chain_next = -1;
            for (int t0 = 0; t0 < C; t0 += kWave) {
                const int t = t0 + lane;
                float sc = 0.0f;
                int bk = 0;
                bool keep = false;
                if (t < C) {
                    sc = L.c_score[t];
                    bk = bucket_of(sc);
                    keep = bk <= bstar;
                }
                const unsigned long long km = __ballot(keep);
                const int pos = base + __popcll(km & ((1ull << lane) - 1ull));
                bool on_chain = false;
                if (keep) {
                    const uint32_t info = L.c_info[t];
                    L.m_score[pos] = sc;
                    L.m_info[pos] = info;
                    L.m_jlo[pos] = (uint16_t)min(s_pref[bk], 0xFFFF);
                    on_chain = member_parent(info) == chain_m && member_rank(info) == 0;
                }
                const unsigned long long cm = __ballot(on_chain);
                if (cm != 0ull) chain_next = __builtin_amdgcn_readlane(pos, __ffsll((long long)cm) - 1);
                base += __popcll(km);
            }
            chain_m = chain_next;
            calm = bstar == bstar_before;
            fresh_total = 0;
            ls = M;
            M = base;
            le = M;
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            if (ls == le) break;
        }
        if (lane == 0) {
            s_state[0] = status;
            s_state[1] = d;
            s_state[2] = M;
            s_state[3] = ls;
            s_state[4] = le;
            s_state[5] = bstar;
            s_state[6] = C_out;
            s_state[7] = chain_m;
            s_M = M;
            s_chain = -1;
        }
    };

    bool by_workgroup = false;  // the single wave has handed this level over
    if (walks && bstar < kLvBuckets) {
        const int Mgen = by_generations();
        if (Mgen >= 0) {
            M = Mgen;
            d = B + 1;  // no level is left
        }
        __syncthreads();
    }
    while (d <= B) {
        if (le - ls <= kWave && C_resume < 0 && !by_workgroup) {
            if (tid < kWave) wave_levels();
            __syncthreads();
            const int status = s_state[0];
            d = s_state[1];
            M = s_state[2];
            ls = s_state[3];
            le = s_state[4];
            bstar = s_state[5];
            chain_m = s_state[7];
            if (status < 0) return -1;
            if (status == 1) break;
            if (status == 2) C_resume = s_state[6];
            by_workgroup = true;
            continue;  // level d goes on below: it has more than 64 parents, or its survivors need room
        }
        const float *row = s_lp + (d - 1) * Kp;
        const int n_par = le - ls;
        int C = 0;
        if (C_resume >= 0) {
            C = C_resume;
            C_resume = -1;
        } else {
            if (n_par > L.capp) return -1;
            // (a level whose candidates do not fit is counted by bucket without being written, the
            // cut moves, and the children are counted once more against the new cut)
            for (int attempt = 0;; ++attempt) {
                C = 0;
                if (tid == 0) {
                    s_nbig = 0;
                    s_bstar = bstar;
                    s_chain = -1;
                }
                s_histc[tid] = 0;
                s_histv[tid] = 0;
                if (tid == 0) s_histc[kLvBuckets] = s_histv[kLvBuckets] = 0;
                // 1. children at or above the cut, per parent, and where they go; small families
                //    are written on the spot by their parent's thread, large ones are queued
                for (int i0 = 0; i0 < n_par; i0 += NT) {
                    const int i = i0 + tid;
                    const int m = ls + i;
                    int c = 0;
                    bool cut = false;
                    float S = 0.0f;
                    if (i < n_par) {
                        S = L.m_score[m];
                        if (m == 0 || bucket_of(S) <= bstar) {
                            const int cap = min(K, max(1, N / ((int)L.m_jlo[m] + 1)));
                            c = count_children(row, S, cap, bstar);
                            cut = c == cap && cap < K;
                        }
                    }
                    int total;
                    const int off = C + build_block_scan(c, s_w, &total);
                    if (i < n_par) {
                        L.p_c[i] = (uint16_t)(c | (cut ? 0x8000 : 0));
                        L.p_off[i] = (uint16_t)min(off, 0xFFFF);
                        if (c > kLvSmall) {
                            const int slot = atomicAdd(&s_nbig, 1);
                            if (slot < kLvBigCap) s_big[slot] = (uint16_t)i; else s_fail = 1;
                        } else if (c > 0 && off + c <= L.capc) {  // (too many candidates: given up below)
                            float v[kLvSmall];
#pragma unroll
                            for (int r = 0; r < kLvSmall; ++r) v[r] = row[min(r, K - 1)];
#pragma unroll
                            for (int r = 0; r < kLvSmall; ++r)
                                if (r < c) {
                                    L.c_score[off + r] = S + v[r];
                                    L.c_info[off + r] = pack_member(m, r, d);
                                }
                        }
                    }
                    C += total;
                }
                if (C <= L.capc) break;
                if (attempt == 1) return -1;
                __syncthreads();
                if (s_fail) return -1;
                for (int i = tid; i < n_par; i += NT) {
                    const int pc = L.p_c[i] & 0x7FFF;
                    if (pc > 0 && pc <= kLvSmall) {
                        const float S = L.m_score[ls + i];
                        for (int r = 0; r < pc; ++r)
                            if (newly_known(ls + i, r)) atomicAdd(&s_histv[bucket_of(S + row[r])], 1);
                    }
                }
                const int nbig0 = s_nbig;
                for (int q = 0; q < nbig0; ++q) {
                    const int i = s_big[q];
                    const int c = L.p_c[i] & 0x7FFF;
                    const float S = L.m_score[ls + i];
                    for (int r = tid; r < c; r += NT)
                        if (newly_known(ls + i, r)) atomicAdd(&s_histv[bucket_of(S + row[r])], 1);
                }
                __syncthreads();
                const int ha0 = s_hist[tid] + s_histv[tid];
                int total0;
                const int ex0 = build_block_scan(ha0, s_w, &total0);
                if (ex0 < N && ex0 + ha0 >= N) s_bstar = tid;
                __syncthreads();
                bstar = min(bstar, s_bstar);
                __syncthreads();
            }
            if (C == 0) break;
            __syncthreads();
            if (s_fail) return -1;
            // 2. the large families, each written by all threads
            const int nbig = s_nbig;
            for (int q = 0; q < nbig; ++q) {
                const int i = s_big[q];
                const int m = ls + i, off = L.p_off[i], c = L.p_c[i] & 0x7FFF;
                const float S = L.m_score[m];
                for (int r = tid; r < c; r += NT) {
                    L.c_score[off + r] = S + row[r];
                    L.c_info[off + r] = pack_member(m, r, d);
                }
            }
            __syncthreads();
            // 3. bucket the candidates, move the cut
            for (int t = tid; t < C; t += NT) {
                const float sc = L.c_score[t];
                const int bk = bucket_of(sc);
                atomicAdd(&s_histc[bk], 1);
                const uint32_t info = L.c_info[t];
                if (newly_known(member_parent(info), member_rank(info))) {
                    atomicAdd(&s_histv[bk], 1);
                    if (walks) count_continuation(s_histv, sc, d, min(bstar, cutb0));
                }
            }
            __syncthreads();
            const int hc = s_histc[tid];
            const int ha = s_hist[tid] + s_histv[tid];
            int total_a, total_c;
            int ex_a = ha, ex_c = hc;
            build_block_scan2(&ex_a, &ex_c, s_w2, &total_a, &total_c);
            s_pref[tid] = ex_c;
            s_hist[tid] = ha;
            if (tid == 0) {
                s_pref[kLvBuckets] = total_c;
                s_hist[kLvBuckets] += s_histv[kLvBuckets];
            }
            if (ex_a < N && ex_a + ha >= N) s_bstar = tid;  // the bucket that holds the N-th best
            __syncthreads();
            bstar = min(bstar, s_bstar);
            // 4. every rank cut must have left out only children below the new cut
            for (int i = tid; i < n_par; i += NT) {
                const int pc = L.p_c[i];
                if (pc & 0x8000) {
                    const float sc = L.m_score[ls + i] + row[pc & 0x7FFF];
                    if (sc > kLvNeg && bucket_of(sc) <= bstar) s_fail = 1;
                }
            }
            __syncthreads();
            if (s_fail) return -1;
        }
        // 5. room for the survivors: when the member arrays would overflow, the members that
        //    have fallen below the cut are squeezed out (the order is kept, so the previous
        //    level stays a contiguous range; parent references are renumbered)
        const int n_surv = s_pref[bstar] + s_histc[bstar];
        if (M + n_surv > L.capm) {
            uint16_t *remap = L.p_c;  // p_c and p_off (contiguous, 2 * capp >= capm) are free now
            const bool chain_kept = chain_m >= 0 && bucket_of(L.m_score[chain_m]) <= bstar;
            int base = 1;
            if (tid == 0) remap[0] = 0;
            for (int m0 = 1; m0 < M; m0 += NT) {
                const int m = m0 + tid;
                float sc = 0.0f;
                uint32_t info = 0;
                uint16_t jl = 0;
                bool keep = false;
                if (m < M) {
                    sc = L.m_score[m];
                    keep = bucket_of(sc) <= bstar;
                    info = L.m_info[m];
                    jl = L.m_jlo[m];
                }
                int tot;
                const int dst = base + build_block_scan(keep ? 1 : 0, s_w, &tot);
                if (keep) {  // dst <= m, and every entry up to this chunk's end has been read
                    remap[m] = (uint16_t)dst;
                    L.m_score[dst] = sc;
                    L.m_info[dst] = info;
                    L.m_jlo[dst] = jl;
                }
                base += tot;
            }
            __syncthreads();
            chain_m = chain_kept ? (int)remap[chain_m] : -1;
            const int M2 = base;
            for (int m = 1 + tid; m < M2; m += NT) {
                const uint32_t info = L.m_info[m];
                L.m_info[m] = pack_member(remap[member_parent(info)], member_rank(info), member_depth(info));
            }
            for (int t = tid; t < C; t += NT) {
                if (bucket_of(L.c_score[t]) <= bstar) {  // (a survivor's parent is alive)
                    const uint32_t info = L.c_info[t];
                    L.c_info[t] = pack_member(remap[member_parent(info)], member_rank(info), member_depth(info));
                }
            }
            M = M2;
            if (tid == 0) s_M = M2;
            __syncthreads();
            if (M + n_surv > L.capm) return -1;
        }
        // 6. candidates at or above the cut become members
        for (int t = tid; t < C; t += NT) {
            const float sc = L.c_score[t];
            const int bk = bucket_of(sc);
            if (bk <= bstar) {
                const int slot = atomicAdd(&s_M, 1);
                if (slot < L.capm) {
                    const uint32_t info = L.c_info[t];
                    L.m_score[slot] = sc;
                    L.m_info[slot] = info;
                    L.m_jlo[slot] = (uint16_t)min(s_pref[bk], 0xFFFF);
                    if (member_parent(info) == chain_m && member_rank(info) == 0) s_chain = slot;
                } else {
                    s_fail = 1;
                }
            }
        }
        __syncthreads();
        if (s_fail) return -1;
        ls = M;
        M = s_M;
        le = M;
        chain_m = s_chain;
        if (ls == le) break;
        __syncthreads();  // s_M, s_nbig, s_chain and the level's histograms are rewritten by the next level
        by_workgroup = false;
        ++d;
    }
    __syncthreads();

    // ---- exact order of the members at or above the cut ----
    // (the members are counted per bucket afresh: the running histogram also holds prefixes that
    // were entered ahead of being found)
    s_histv[tid] = 0;
    s_histc[tid] = 0;
    if (tid == 0) s_histv[kLvBuckets] = s_histc[kLvBuckets] = 0;
    __syncthreads();
    for (int m = 1 + tid; m < M; m += NT) {
        const int bk = bucket_of(L.m_score[m]);
        if (bk <= bstar) atomicAdd(&s_histv[bk], 1);
    }
    __syncthreads();
    const int hb = tid <= bstar ? s_histv[tid] : 0;
    if (tid == 0) s_bstar = bstar;
    int total_alive;
    const int start = build_block_scan(hb, s_w, &total_alive);
    s_pref[tid] = start;
    if (tid == 0) s_pref[kLvBuckets] = total_alive;
    // The members are every prefix at or above the cut, so the N best of them are the tree: the
    // cut moves up to the bucket that holds the N-th best member, and whatever the construction
    // let in beyond it (a cut left alone while members were enumerated) is not ranked at all.
    if (start < N && start + hb >= N) s_bstar = tid;
    uint16_t *sorted = reinterpret_cast<uint16_t *>(L.c_info);
    uint16_t *node_id = reinterpret_cast<uint16_t *>(L.c_score);
    __syncthreads();
    bstar = min(bstar, s_bstar);
    if (bstar == kLvBuckets) total_alive += s_histv[kLvBuckets];
    else total_alive = s_pref[bstar] + s_histv[bstar];
    for (int m = 1 + tid; m < M; m += NT) {
        const int bk = bucket_of(L.m_score[m]);
        if (bk <= bstar) sorted[s_pref[bk] + atomicAdd(&s_histc[bk], 1)] = (uint16_t)m;
    }
    __syncthreads();
    for (int e = tid; e < total_alive; e += NT) {
        const int m = sorted[e];
        const int bk = bucket_of(L.m_score[m]);
        const int bs = s_pref[bk], nb = s_histv[bk];
        const float sm = L.m_score[m];
        int g = 0;
        // the bucket's members eight at a time: ids and scores are fetched together (the empty
        // statements keep the fetches ahead of the comparisons), and only equal scores, which
        // the rank tuples decide, take the full comparison
        for (int j0 = 0; j0 < nb; j0 += 8) {
            int o[8];
            float so[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] = sorted[bs + min(j0 + k, nb - 1)];
#pragma unroll
            for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(o[k]));
#pragma unroll
            for (int k = 0; k < 8; ++k) so[k] = L.m_score[o[k]];
#pragma unroll
            for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(so[k]));
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (j0 + k >= nb || o[k] == m) continue;
                if (so[k] != sm) g += so[k] > sm ? 1 : 0;
                else g += member_before(L.m_score, L.m_info, o[k], m) ? 1 : 0;
            }
        }
        const int pos = bs + g;
        node_id[m] = (uint16_t)(pos < N ? pos + 1 : 0);
    }
    __syncthreads();
    for (int e = tid; e < total_alive; e += NT) {
        const int m = sorted[e];
        const int id = node_id[m];
        if (id == 0) continue;
        const uint32_t info = L.m_info[m];
        const int pm = member_parent(info);
        s_node[id] = pack_node(pm == 0 ? 0 : node_id[pm], member_rank(info), member_depth(info));
        s_score[id] = L.m_score[m];
    }
    __syncthreads();
    return min(N, total_alive);
}

template <int NSLOT>
__global__ __launch_bounds__(kBuildThreads) void build_kernel(
    const int32_t *__restrict__ topk_tok, const float *__restrict__ topk_lp, int B, int K, int N,
    const int32_t *__restrict__ root_token, int32_t *__restrict__ tokens,
    int32_t *__restrict__ parent, int32_t *__restrict__ depth, int32_t *__restrict__ rank,
    float *__restrict__ node_score, uint64_t *__restrict__ ancestor_mask,
    int32_t *__restrict__ n_nodes, int algo, int capm, int capp, int capc)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int Kp = K + 3;
    const int T = N + 1;
    float *s_lp = reinterpret_cast<float *>(smem);                     // [B][Kp], -inf padded
    uint32_t *s_node = reinterpret_cast<uint32_t *>(s_lp + B * Kp);     // [T]
    float *s_score = reinterpret_cast<float *>(s_node + T);             // [T]
    // the level-synchronous construction's arrays follow
    LevelMem lv;
    lv.capm = capm;
    lv.capp = capp;
    lv.capc = capc;
    lv.m_score = reinterpret_cast<float *>(s_score + T);
    lv.m_info = reinterpret_cast<uint32_t *>(lv.m_score + capm);
    lv.c_score = reinterpret_cast<float *>(lv.m_info + capm);
    lv.c_info = reinterpret_cast<uint32_t *>(lv.c_score + capc);
    lv.m_jlo = reinterpret_cast<uint16_t *>(lv.c_info + capc);
    lv.p_c = lv.m_jlo + capm;
    lv.p_off = lv.p_c + capp;
    __shared__ int s_built;

    const int tid = threadIdx.x;
    const int seq = blockIdx.x;
    const float *lp = topk_lp + (size_t)seq * B * K;
    const int32_t *tk = topk_tok + (size_t)seq * B * K;

    // log-probabilities into LDS, rows padded with -inf.  The [B][K] table is contiguous: thread
    // t takes the 16-byte pieces t, t + 256, ..., sixteen loads in flight at a time (one round trip
    // to memory up to B K = 16384), and keeps (row, column) of its first element by stepping both.
    {
        const int n_el = B * K;
        // whole pieces of four, if this sequence's table starts on a 16-byte boundary (else, and
        // for the last one to three elements, the plain loop below)
        const int n_q = (reinterpret_cast<uintptr_t>(lp) & 15) == 0 ? n_el >> 2 : 0;
        const int dq = (4 * kBuildThreads) / K, dr = (4 * kBuildThreads) % K;  // one step of 1024 elements
        int d = (4 * tid) / K, k = (4 * tid) % K;
        const float4 *lp4 = reinterpret_cast<const float4 *>(lp);
        for (int q0 = tid; q0 < n_q; q0 += 16 * kBuildThreads) {
            float4 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int q = q0 + u * kBuildThreads;
                v[u] = q < n_q ? lp4[q] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (q0 + u * kBuildThreads < n_q) {
                    const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
                    int dd = d, kk = k;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        s_lp[dd * Kp + kk] = x[c];
                        if (++kk == K) {
                            kk = 0;
                            ++dd;
                        }
                    }
                }
                d += dq;
                k += dr;
                if (k >= K) {
                    k -= K;
                    ++d;
                }
            }
        }
        for (int e = 4 * n_q + tid; e < n_el; e += kBuildThreads) s_lp[(e / K) * Kp + e % K] = lp[e];
        for (int i = tid; i < 3 * B; i += kBuildThreads) s_lp[(i / 3) * Kp + K + i % 3] = -INFINITY;
    }
    if (tid == 0) {
        s_node[0] = pack_node(0, 0, 0);
        s_score[0] = 0.0f;
    }
    __syncthreads();

    // Which construction: the sequential pops win on small budgets and on stars (nearly all nodes
    // at depth 1: their sibling runs pop in batches); the level-synchronous construction wins on
    // large budgets and wherever pops alternate between parents, each a step of its own.  A star
    // is recognised by the top-1 chain falling below the worst useful rank of row 0 within two
    // steps and by the best depth-1 node having fewer than four children above that rank.
    // Both constructions give the same tree; algo 1 / 2 force one of them.
    bool use_levels = capm > 0 && algo != DDTREE_BUILD_POPS;
    if (use_levels && algo == DDTREE_BUILD_AUTO) {
        const float worst = s_lp[min(K, N) - 1];
        float chain = 0.0f;
        int deep = 0;
        for (int d = 0; d < B; ++d) {
            chain += s_lp[d * Kp];
            deep += chain >= worst ? 1 : 0;
        }
        const bool bushy = B >= 2 && s_lp[0] + s_lp[Kp + min(3, K - 1)] >= worst;
        use_levels = N > 256 || (N >= 48 && (deep >= 3 || bushy));
    }
    int level_n = -1;
    if (use_levels) {
        level_n = level_build(s_lp, Kp, B, K, N, lv, s_node, s_score);
        if (level_n < 0 && tid == 0) atomicAdd(&g_level_giveups, 1u);
    }
    if (level_n >= 0) {
        if (tid == 0) s_built = level_n;
    } else if (tid < kWave) {
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

    // Node ids are dealt so that T = 257 (a budget of 256 and the root) takes one pass: the last
    // thread also takes the root, whose row is trivial, before its own node.
    for (int i0 = 1; i0 < T; i0 += kBuildThreads) {
        const int i = i0 + tid;
        if (i0 == 1 && tid == kBuildThreads - 1) {
            const size_t o0 = (size_t)seq * T;
            tokens[o0] = root_token[seq];
            parent[o0] = -1;
            depth[o0] = 0;
            if (rank) rank[o0] = -1;
            if (node_score) node_score[o0] = 0.0f;
            uint64_t *m0 = ancestor_mask + o0 * W;
            m0[0] = 1ull;
            for (int w = 1; w < W; ++w) m0[w] = 0ull;
        }
        if (i >= T) continue;
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
        // (depth and rank are clamped to the table: whatever the records hold, every read below
        // stays inside topk_tok and the workgroup's LDS)
        const int d = min(max(node_depth(nd), 1), B);
        tokens[o] = tk[(d - 1) * K + min(node_rank(nd), K - 1)];
        parent[o] = node_parent(nd);
        depth[o] = d;
        if (rank) rank[o] = node_rank(nd);
        if (node_score) node_score[o] = s_score[i];
        if constexpr (NSLOT <= 5) {
            // ancestors of i (itself first, the root last), folded into the W <= NSLOT mask words as
            // the chain is walked: the words stay in registers (compile-time indices), so the only
            // dependent LDS reads are the d parent look-ups
            uint64_t word[NSLOT];
#pragma unroll
            for (int w = 0; w < NSLOT; ++w) word[w] = 0ull;
            int j = i;
            for (int t = 0; t <= d; ++t) {
                const uint64_t bit = 1ull << (j & 63);
                const int wj = j >> 6;
#pragma unroll
                for (int w = 0; w < NSLOT; ++w) word[w] |= wj == w ? bit : 0ull;
                j = node_parent(s_node[j]);
            }
#pragma unroll
            for (int w = 0; w < NSLOT; ++w)
                if (w < W) mrow[w] = word[w];
        } else {
            // many words, few ancestors: the row is cleared, then the chain is walked with one word
            // in hand (a parent's id is below its child's, so the word index never rises) and
            // every word that received bits is stored over its zero (stores of one thread to
            // one address keep their order)
            for (int w = 0; w < W; ++w) mrow[w] = 0ull;
            int j = i, cur_w = i >> 6;
            uint64_t cur = 0ull;
            for (int t = 0; t <= d; ++t) {
                const int wj = min(j >> 6, W - 1);  // (clamped like every index taken from a record)
                if (wj != cur_w) {
                    mrow[cur_w] = cur;
                    cur = 0ull;
                    cur_w = wj;
                }
                cur |= 1ull << (j & 63);
                j = node_parent(s_node[j]);
            }
            mrow[cur_w] = cur;
        }
    }
}

static size_t build_lds_bytes(int B, int K, int N)
{
    return (size_t)B * (K + 3) * 4 + (size_t)(N + 1) * 8;
}

// Dynamic LDS of the kernel and the capacities of the level-synchronous construction (members,
// candidates per level).  capm = 0: no room,
// sequential pops only.
struct BuildLds {
    size_t bytes;
    int capm, capp, capc;
};
static BuildLds build_lds_plan(int B, int K, int N, bool level)
{
    const size_t base = (size_t)B * (K + 3) * 4 + (size_t)(N + 1) * 8;
    BuildLds r{base, 0, 0, 0};
    if (!level) return r;
    const size_t limit = 150 * 1024;
    if (base >= limit) return r;
    const size_t avail = limit - base;
    const int capp = 2 * N + 256;       // members of one depth that can be parents
    const int min_m = 2 * N + 64;
    int capc = 4 * N + 512;             // candidates of one level
    // large budgets leave little room beside the log-probability table: favour the members
    if (4 * (size_t)capp + 8 * (size_t)capc + 10 * (size_t)(4 * N + 256) > avail) capc = 3 * N + 256;
    if (4 * (size_t)capp + 8 * (size_t)capc + 10 * (size_t)min_m > avail) capc = 2 * N + 256;
    const size_t fixed = 4 * (size_t)capp + 8 * (size_t)capc;
    if (fixed + 10 * (size_t)min_m > avail) return r;
    size_t capm = (avail - fixed) / 10 / 2 * 2;
    if (capm > (size_t)8 * N + 256) capm = (size_t)8 * N + 256;
    if (capm > 8192) capm = 8192;       // member ids are 13 bits wide
    if (capm > 2 * (size_t)capc) capm = 2 * (size_t)capc;
    if (capm > 2 * (size_t)capp) capm = 2 * (size_t)capp;
    r.capm = (int)capm;
    r.capp = capp;
    r.capc = capc;
    const size_t lv = 10 * capm + fixed;
    r.bytes = base + lv;
    return r;
}

static std::atomic<int> g_build_algo{DDTREE_BUILD_AUTO};

template <int NSLOT>
static int launch_build(const int32_t *topk_tok, const float *topk_lp, int batch, int B, int K, int N,
                        const int32_t *root_token, int32_t *tokens, int32_t *parent, int32_t *depth,
                        int32_t *rank, float *node_score, uint64_t *ancestor_mask, int32_t *n_nodes,
                        hipStream_t st)
{
    const int algo = g_build_algo.load();
    const BuildLds lds = build_lds_plan(B, K, N, algo != DDTREE_BUILD_POPS);
    static std::atomic<bool> lds_allowed{false};
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(build_kernel<NSLOT>), 150 * 1024, lds_allowed))
        return DDTREE_ERR_HIP;
    DDT_LAUNCH(DDTREE_KERNEL_BUILD, st, build_kernel<NSLOT>, dim3(batch), dim3(kBuildThreads), lds.bytes,
                       st, topk_tok, topk_lp, B, K, N, root_token, tokens, parent, depth, rank,
                       node_score, ancestor_mask, n_nodes, algo, lds.capm, lds.capp, lds.capc);
    return launch_status();
}

}  // namespace ddt

extern "C" int ddtree_set_build_algorithm(int algo)
{
    if (algo != DDTREE_BUILD_AUTO && algo != DDTREE_BUILD_POPS && algo != DDTREE_BUILD_LEVELS)
        return DDTREE_ERR_ARG;
    ddt::g_build_algo.store(algo);
    return DDTREE_OK;
}

extern "C" int ddtree_build_giveups(unsigned int *count)
{
    if (!count) return DDTREE_ERR_ARG;
    if (hipMemcpyFromSymbol(count, HIP_SYMBOL(ddt::g_level_giveups), sizeof(unsigned int)) != hipSuccess)
        return DDTREE_ERR_HIP;
    return DDTREE_OK;
}

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
