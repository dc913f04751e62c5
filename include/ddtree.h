/*
 * ddtree.h -- C ABI of the DDTree draft-tree step for AMD MI355X (gfx950).
 *
 * One decoding round of the paper's method (Section 4.1, steps 2-4) is
 *     ddtree_topk -> ddtree_build -> ddtree_verify_attn (per target layer) -> ddtree_accept
 * followed by ddtree_compact to close the round (Section 4.4, last sentence).
 *
 * Notation (the paper's own letters in brackets):
 *   batch  independent sequences handled by one call
 *   B      number of draft positions = rows of drafter logits            [L]
 *   V      vocabulary size                                               [|V|]
 *   N      node budget, the root not counted                             [B]
 *   K      candidates kept per position, K = min(N, V)  (Lemma 1)        [K]
 *   T      N + 1 verifier rows per sequence; row 0 is the root, i.e. the bonus token b
 *   W      ceil(T / 64) 64-bit words per ancestor-mask row
 *   L      context rows already in the KV cache of a sequence
 *
 * Conventions shared by every entry point
 *   - Return value: DDTREE_OK or a negative DDTREE_ERR_* code.  Arguments are validated on
 *     the host before anything is launched; a call that returns an error has launched nothing.
 *   - Pointers marked [device] are device memory owned by the caller; the library never
 *     allocates, frees or retains them.  Pointers marked [host] are read during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     kernels on it (no allocation, no memset or copy, no synchronisation); consecutive calls
 *     on one stream are ordered.  A caller may therefore record them into a HIP graph; the
 *     [host] arrays of a call (kv_offset, kv_start, kv_len, dst_row) travel as kernel arguments
 *     and are fixed in a recorded graph.
 *   - `workspace` [device] is scratch of at least ddtree_workspace_bytes(...) bytes, 256-byte
 *     aligned, whose contents need not survive between calls.  Calls on different streams need
 *     different workspaces.
 *   - All arrays are dense, row-major, in the index order written next to them, and aligned
 *     to their element size; the q / k / v / out tensors of ddtree_verify_attn to 16 bytes
 *     (DDTREE_ERR_ARG otherwise).
 *   - Logits must be finite (the paper assumes probabilities in (0,1), Section 4.2).
 */
#ifndef DDTREE_H
#define DDTREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DDTREE_OK 0
#define DDTREE_ERR_ARG (-1)       /* null pointer, bad shape, unsupported size or dtype */
#define DDTREE_ERR_WORKSPACE (-2) /* workspace missing, misaligned or too small          */
#define DDTREE_ERR_HIP (-3)       /* the HIP runtime reported a launch failure           */

#define DDTREE_DTYPE_BF16 0
#define DDTREE_DTYPE_FP32 1

#define DDTREE_MAX_B 32      /* draft positions                 */
#define DDTREE_MAX_N 1024    /* node budget                     */
#define DDTREE_MAX_BATCH 64  /* sequences per call              */

/* Library version, major * 100 + minor. */
int ddtree_version(void);

/* Static text for a return code. */
const char *ddtree_error_string(int code);

/*
 * Scratch size, in bytes, that covers every entry point for the given problem:
 * max_sum_L is an upper bound on the total number of cache rows over the batch.
 * Returns 0 if the shape is not supported.  Pure host arithmetic.
 */
size_t ddtree_workspace_bytes(int batch, int B, int V, int N, int Hq, int Hkv, int D,
                              int max_sum_L);

/*
 * Scratch that one ddtree_verify_attn call uses for exactly this shape and total cache length
 * sum_L (0 for the shapes that take no scratch).  Never more than ddtree_workspace_bytes for the
 * same shape and any cache length.  Pure host arithmetic.
 */
size_t ddtree_verify_attn_workspace_bytes(int batch, int T, int Hq, int Hkv, int D, int dtype,
                                          long long sum_L);

/*
 * Per-position log-probabilities and rank ordering (Section 4.3: q_i = softmax(l_i), tokens
 * ordered so that q_i^(1) >= q_i^(2) >= ..., and the scores sigma are sums of log q; Lemma 1
 * bounds the ranks that can matter by K).
 *   logits    [device] fp32 [batch, B, V]
 *   topk_tok  [device] int32 [batch, B, K]  token of rank k at position d; equal logits are
 *                                           ranked by ascending token id
 *   topk_lp   [device] fp32 [batch, B, K]   log q_d(topk_tok[d][k]) = logit - logsumexp(row),
 *                                           evaluated in fp64 as (logit - max) - log1p(sum of
 *                                           exp(x - max) over every entry but the first maximum)
 *                                           and rounded once: a token that holds nearly all the
 *                                           probability keeps its tiny negative log-probability
 * Requires 1 <= K <= min(V, DDTREE_MAX_N), 1 <= B <= DDTREE_MAX_B, and that the candidates of one
 * row fit the merge workgroup's LDS: ceil(V / 12288) * min(K, 12288) <= 14336, i.e. any K up to
 * V = 172032 (K = 1024), V <= 344064 at K = 512, V <= 688128 at K = 256.  Other shapes return
 * DDTREE_ERR_ARG (and ddtree_workspace_bytes returns 0 for them).  Calls with batch * B >= 128
 * rows scan each row with one workgroup and have no such limit.
 */
int ddtree_topk(const float *logits, int batch, int B, int V, int K, int32_t *topk_tok,
                float *topk_lp, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Best-first tree construction (Algorithm 1) plus the tensors the verifier needs
 * (Section 4.4, first paragraph: token ids rooted at b, depth as position id, ancestor-only
 * visibility).  Node 0 is the root; nodes 1..n_nodes are numbered in pop order, so
 * parent[i] < i and node scores are non-increasing.  Scores are fp32 left folds of topk_lp
 * along the rank tuple; of two equal scores the lexicographically smaller rank tuple is
 * popped first (a prefix before its extensions).
 *   topk_tok, topk_lp [device] as produced by ddtree_topk, [batch, B, K]
 *   root_token  [device] int32 [batch]        the bonus token of each sequence
 *   tokens      [device] int32 [batch, N+1]   tokens[0] = root_token
 *   parent      [device] int32 [batch, N+1]   parent[0] = -1
 *   depth       [device] int32 [batch, N+1]   depth[0] = 0; position id = L + depth
 *   rank        [device] int32 [batch, N+1]   0-based rank of the node's token, rank[0] = -1
 *                                             (nullable)
 *   node_score  [device] fp32 [batch, N+1]    sigma of the node, node_score[0] = 0 (nullable)
 *   ancestor_mask [device] uint64 [batch, N+1, W]  bit j of row i (word j/64, bit j%64) is set
 *                                             iff j is the root, an ancestor of i, or i
 *   n_nodes     [device] int32 [batch]        nodes built, = N unless fewer prefixes exist
 * Rows past n_nodes hold tokens = parent = depth = rank = -1, score 0 and a zero mask row.
 * A prefix of score -inf (it contains a token of probability zero; the paper assumes
 * probabilities in (0,1)) never becomes a node: n_nodes counts prefixes of finite score only.
 * Requires 1 <= N <= DDTREE_MAX_N, 1 <= K <= DDTREE_MAX_N, 1 <= B <= DDTREE_MAX_B (the
 * log-probability table and the node records, 4 B (K + 3) + 8 (N + 1) bytes, then fit the
 * workgroup's LDS); anything else returns DDTREE_ERR_ARG.
 */
int ddtree_build(const int32_t *topk_tok, const float *topk_lp, int batch, int B, int K, int N,
                 const int32_t *root_token, int32_t *tokens, int32_t *parent, int32_t *depth,
                 int32_t *rank, float *node_score, uint64_t *ancestor_mask, int32_t *n_nodes,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * One layer of tree attention (Section 4.4, first paragraph): query row i of a sequence
 * attends to all of that sequence's cache rows and to the tree rows j whose bit is set in
 * ancestor_mask[i]; softmax(q.k * softmax_scale) weighted sum of the value rows.  Query head h
 * reads KV head h / (Hq / Hkv).  Rows whose own mask bit is clear (padding rows) produce zeros.
 *   q          [device] [batch*T, Hq, D]
 *   k_cache, v_cache [device] [sum_L, Hkv, D]   sequence s owns rows kv_offset[s]..kv_offset[s+1]
 *   k_tree, v_tree   [device] [batch*T, Hkv, D] sequence s owns rows s*T..(s+1)*T; all T rows
 *                                               must hold finite values, those of padding nodes
 *                                               too: a key that a row does not see has weight
 *                                               zero but is still multiplied (0 * NaN = NaN)
 *   ancestor_mask    [device] uint64 [batch, T, W]
 *   kv_offset        [host]   int32 [batch+1], non-decreasing, kv_offset[0] >= 0
 *   dtype      DDTREE_DTYPE_BF16 (bf16 in/out, fp32 accumulation and softmax; any finite bf16
 *              values: partial results of split key ranges are kept relative to their row's
 *              magnitude, so large value rows do not overflow on the way) or
 *              DDTREE_DTYPE_FP32 (fp32 throughout)
 *   out        [device] [batch*T, Hq, D], same dtype as q
 * Requires Hq % Hkv == 0, D a multiple of 8 and <= 256, T <= DDTREE_MAX_N + 1,
 * batch <= DDTREE_MAX_BATCH.  bf16 with D = 128 (and Hkv <= 32768) runs on the matrix cores.
 */
int ddtree_verify_attn(const void *q, const void *k_cache, const void *v_cache,
                       const void *k_tree, const void *v_tree, const uint64_t *ancestor_mask,
                       const int32_t *kv_offset, int batch, int T, int Hq, int Hkv, int D,
                       float softmax_scale, int dtype, void *out, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * The same attention with each sequence's cache rows given as a span: sequence s owns rows
 * kv_start[s] .. kv_start[s] + kv_len[s] - 1 of k_cache / v_cache ([host] int32 [batch] each,
 * kv_start >= 0, kv_len >= 0).  The spans need not touch or be ordered, so a serving loop can keep
 * room behind every sequence and let ddtree_compact append the accepted rows in place
 * (Section 4.4, last sentence); ddtree_verify_attn is this call with kv_start = kv_offset[s] and
 * kv_len = kv_offset[s + 1] - kv_offset[s].  Workspace as for ddtree_verify_attn, with the sum of
 * the lengths in place of sum_L.
 */
int ddtree_verify_attn_spans(const void *q, const void *k_cache, const void *v_cache,
                             const void *k_tree, const void *v_tree, const uint64_t *ancestor_mask,
                             const int32_t *kv_start, const int32_t *kv_len, int batch, int T, int Hq,
                             int Hkv, int D, float softmax_scale, int dtype, void *out,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Greedy verifier walk (Section 4.4, second paragraph; Figure 1b): posterior[i] is the argmax
 * of the target's logits at node i (lowest id among equal maxima).  Starting at the root, the
 * walk moves to the child of the current node whose token equals the posterior of the current
 * node, and stops when there is none.
 *   target_logits [device] fp32 [batch, T, V]
 *   tokens, parent, depth [device] int32 [batch, T]   from ddtree_build
 *   n_nodes       [device] int32 [batch]              rows past n_nodes are not read
 *   path          [device] int32 [batch, B+1]  path[0] = 0, then the accepted node ids; unused
 *                                              slots are -1
 *   n_accepted    [device] int32 [batch]       accepted drafted nodes, 0..B (the accepted length
 *                                              "including the bonus token" is n_accepted + 1)
 *   bonus_token   [device] int32 [batch]       posterior of the last node on the path
 *   posterior     [device] int32 [batch, T]    nullable; -1 on rows past n_nodes
 */
int ddtree_accept(const float *target_logits, int batch, int T, int V, const int32_t *tokens,
                  const int32_t *parent, const int32_t *depth, const int32_t *n_nodes,
                  int32_t *path, int32_t *n_accepted, int32_t *bonus_token, int32_t *posterior,
                  int B, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ddtree_accept for callers that cannot allocate device memory or bring a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid the allocator): the same kernels,
 * with the partial argmaxes kept in a static device array inside the library, DDTREE_NOALLOC_SCRATCH_BYTES
 * (256 KiB) on every GPU the library runs on, held until the process ends.  The call allocates and
 * frees nothing.  Arguments and results as in ddtree_accept, without the workspace.
 *   - Shapes whose partials exceed the array return DDTREE_ERR_WORKSPACE and launch nothing:
 *     batch * T * segments * 8 bytes must fit, segments = min(ceil(3072 / (batch * T)), max(1, V / 8192))
 *     (the headline shape, 257 rows of 151936 logits, takes 24 KB; 16 sequences of 129 rows 33 KB;
 *     the largest call the other entry points accept, 64 sequences of 1025 rows, 525 KB, is refused).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams or host threads) race and must be serialised by the caller.  Nothing in the array
 *     needs clearing between calls: every entry a call reads it has written itself.
 *   - The array's device address is looked up on the first call on each device (with that device
 *     current); DDTREE_ERR_HIP if the runtime refuses.
 */
#define DDTREE_NOALLOC_SCRATCH_BYTES ((size_t)256 << 10)
int ddtree_accept_noalloc(const float *target_logits, int batch, int T, int V, const int32_t *tokens,
                          const int32_t *parent, const int32_t *depth, const int32_t *n_nodes,
                          int32_t *path, int32_t *n_accepted, int32_t *bonus_token,
                          int32_t *posterior, int B, void *stream);

/*
 * The same walk at temperature > 0 (Section 4.4, second paragraph: verification follows the
 * target model's own decoding rule, greedy or temperature-based sampling).  The token the target
 * selects at node i is a sample from softmax(target_logits[i] / temperature), drawn by the
 * Gumbel-max rule argmax_v (logit[v] / temperature - log(-log u)) with u in (0,1) from a
 * counter-based generator keyed by (seed, row s*T+i, v):
 *     mix(x):  x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16
 *     h = mix(mix(v ^ seed_lo) + 0x9E3779B9 * row + seed_hi),   u = ((h >> 8) + 0.5) / 2^24
 * so a (seed, row) pair always selects the same token, whatever the launch shape.  Keys are
 * formed in fp32; two tokens whose keys differ by less than about 1e-4 may be selected either way.
 * posterior receives the selected tokens.  Arguments otherwise as in ddtree_accept;
 * temperature must be positive and finite (DDTREE_ERR_ARG otherwise).
 */
int ddtree_accept_sampled(const float *target_logits, int batch, int T, int V,
                          const int32_t *tokens, const int32_t *parent, const int32_t *depth,
                          const int32_t *n_nodes, float temperature, uint64_t seed, int32_t *path,
                          int32_t *n_accepted, int32_t *bonus_token, int32_t *posterior, int B,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Cache compaction (Section 4.4, last sentence): the cache keeps only the accepted path.  For
 * every sequence s and j = 0..n_accepted[s]: cache[dst_row[s] + j] = tree[s*T + path[s][j]]
 * (j = 0 is the root, whose key/value rows were not in the cache before this round).
 *   k_tree, v_tree   [device] [batch*T, Hkv, D]
 *   path             [device] int32 [batch, B+1], n_accepted [device] int32 [batch]
 *   dst_row          [host]   int32 [batch]  first cache row to write for each sequence
 *                                            (normally the sequence's current length)
 *   k_cache, v_cache [device] [cache_rows, Hkv, D]; rows dst_row[s] .. dst_row[s]+B must exist
 *   elem_bytes       2 (bf16) or 4 (fp32)
 */
int ddtree_compact(const void *k_tree, const void *v_tree, const int32_t *path,
                   const int32_t *n_accepted, const int32_t *dst_row, int batch, int T, int B,
                   int Hkv, int D, int elem_bytes, void *k_cache, void *v_cache, void *stream);

/*
 * Construction used by ddtree_build (Algorithm 1 defines the result; both constructions produce
 * it bit for bit).  DDTREE_BUILD_POPS runs the best-first pops one after the other on one
 * wavefront; DDTREE_BUILD_LEVELS finds the same N best prefixes (Proposition 2) as a set, depth
 * by depth or, on peaked rows, by the number of non-zero ranks in a prefix, orders them, and
 * falls back to the pops when heavy score ties defeat its bounds;
 * DDTREE_BUILD_AUTO (the default) picks per sequence from the budget and the shape of the
 * log-probabilities.  Process-wide, takes effect at the next ddtree_build call; meant for
 * tests and tuning.  Returns DDTREE_ERR_ARG for any other value.
 */
#define DDTREE_BUILD_AUTO 0
#define DDTREE_BUILD_POPS 1
#define DDTREE_BUILD_LEVELS 2
int ddtree_set_build_algorithm(int algo);

/* Host-side self-check of the launch arithmetic behind ddtree_verify_attn's matrix-core kernel
 * (paper Section 4.4: every tree node attends to the whole context -- the decomposition of
 * that work into workgroups must cover every (sequence, KV head, query row, key) exactly once).
 * For a fixed list of shapes it builds the plan, the per-XCD runs of work items and the
 * reciprocals a launch would pass, decodes every workgroup index the way the kernel does, and
 * holds the result against plain division and against that coverage; it also checks, over a
 * grid of sizes, that the chunks of ddtree_topk and the segments of ddtree_accept tile a logits
 * row and that their scratch holds what the kernels index.  No GPU is touched and nothing is
 * launched.  Returns 0, or 100 * (number of the failing shape) + (number of the failed check)
 * for the attention (values below 100 concern the reciprocal division itself), 10000 + (number
 * of the failed check) for the plans. */
int ddtree_selftest_host(void);
/*
 * Number of sequences, since the library was loaded, for which the level-synchronous
 * construction gave up and the pops built the tree instead.  count is a host pointer; the call
 * waits for the device.  Meant for tests.
 */
int ddtree_build_giveups(unsigned int *count);

/*
 * Kernel timing hook for benchmarks (no passage of the paper: measurement only).  While a
 * kernel's bit is set in kernel_mask, every launch of that kernel carries a pair of HIP events
 * that take the begin and end time stamps of the dispatch itself (no marker packets on the
 * stream), up to `capacity` launches per kernel; the events are created here, never inside the
 * hot calls.  kernel_mask = 0 switches the hook off and destroys
 * the events.  ddtree_profile_enable_every times one launch in `every` (the first, the
 * (every+1)-th, ...), for timed loops that want to be disturbed as little as possible.  ddtree_profile_read copies the elapsed milliseconds of the recorded launches of
 * one kernel to host memory and returns how many there were (or a negative error); the caller
 * must have synchronised the stream(s) first.  ddtree_profile_reset forgets recorded launches.
 * Not thread-safe; meant for a single benchmarking thread.
 */
#define DDTREE_KERNEL_TOPK_CHUNK 0
#define DDTREE_KERNEL_TOPK_MERGE 1
#define DDTREE_KERNEL_BUILD 2
#define DDTREE_KERNEL_ATTN 3
#define DDTREE_KERNEL_ATTN_MERGE 4
#define DDTREE_KERNEL_ACCEPT_ARGMAX 5
#define DDTREE_KERNEL_ACCEPT_WALK 6
#define DDTREE_KERNEL_ATTN_GENERIC 7
#define DDTREE_KERNEL_COUNT 8
int ddtree_profile_enable(unsigned kernel_mask, int capacity);
int ddtree_profile_enable_every(unsigned kernel_mask, int capacity, int every);
int ddtree_profile_reset(void);
int ddtree_profile_read(int kernel_id, float *ms_out /* [host] */, int max_records);

#ifdef __cplusplus
}
#endif
#endif /* DDTREE_H */
