/*
 * DDTree draft-tree step: CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP sources, and nothing in the product path may call it.
 *
 * Everything here follows the paper's Section 4 ("The Proposed Method"):
 *   - per-position log-softmax and rank ordering  (Section 4.3, the ordering
 *     q_i^(1) >= q_i^(2) >= ... and sigma(rho) = sum log q_i^(rho_i))
 *   - best-first heap construction                (Algorithm 1)
 *   - tree attention visibility                   (Section 4.4, first paragraph)
 *   - verifier walk                               (Section 4.4, second paragraph,
 *                                                  and Figure 1b)
 *   - cache compaction                            (Section 4.4, last sentence)
 *
 * Notation used in this file (the paper's letters in brackets):
 *   B  number of draft positions / drafter logit rows        [paper: L]
 *   N  node budget, root not counted                         [paper: B]
 *   V  vocabulary size                                       [paper: |V|]
 *   K  per-depth candidate width, min(N, V)                  [paper: K]
 *   T  N + 1 rows handed to the verifier, node 0 = root (the bonus token b)
 *   L  number of context rows already in the KV cache
 *
 * Readings taken where the paper leaves a choice (each one is a legal instance
 * of "ties broken arbitrarily" in Proposition 2 or of an unstated default):
 *   R1  equal logits inside a row: the lower token id gets the lower rank.
 *   R2  equal prefix scores: the prefix whose rank tuple is lexicographically
 *       smaller comes first, a proper prefix coming before its extensions.
 *   R3  sigma is the fp32 left fold ((lp_1 + lp_2) + ...) over the rank tuple;
 *       a sibling's score is score(parent node) + lp[d][rank+1] (equal in exact
 *       arithmetic to Algorithm 1's "sigma - log q^(r) + log q^(r+1)").
 *   R4  nodes are numbered in pop order, node 0 being the root.
 *   R5  log-sum-exp is evaluated in fp64 and lp is rounded to fp32 once.
 *   R6  attention scale is 1/sqrt(D) (passed in), masked keys are excluded.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Section 4.3: per-position distributions, ordered by probability.    */
/* ------------------------------------------------------------------ */

typedef struct {
    float logit;
    int32_t id;
} tok_entry;

/* (logit descending, token id ascending): reading R1. */
static int cmp_tok_entry(const void *pa, const void *pb)
{
    const tok_entry *a = (const tok_entry *)pa;
    const tok_entry *b = (const tok_entry *)pb;
    if (a->logit > b->logit) return -1;
    if (a->logit < b->logit) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

/*
 * For every row d of logits[B][V]: q_d = softmax(logits[d]); order the tokens
 * by q_d descending; keep the first K.  tok[d][k] is the rank-k token and
 * lp[d][k] = log q_d(tok[d][k]) = logit - logsumexp(row), in fp64, rounded to
 * fp32 (reading R5).  lse_out (nullable) receives the fp64 log-sum-exp per row.
 */
int oracle_topk(const float *logits, int B, int V, int K, int32_t *tok, float *lp,
                double *lse_out)
{
    if (B < 1 || V < 1 || K < 1 || K > V) return -1;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int d = 0; d < B; ++d) {
        const float *row = logits + (size_t)d * V;
        tok_entry *e = (tok_entry *)malloc((size_t)V * sizeof(tok_entry));
        if (!e) {
            status = -2;
            continue;
        }
        /* log-sum-exp as max + log1p(sum over every element but the first maximum): the same
         * number as max + log(sum over all), without the cancellation that the leading 1 causes
         * when one token holds nearly all the probability (its log-probability is -log1p(tiny)) */
        float m = row[0];
        int vmax = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > m) {
                m = row[v];
                vmax = v;
            }
        double S1 = 0.0;
        for (int v = 0; v < V; ++v)
            if (v != vmax) S1 += exp((double)row[v] - (double)m);
        const double excess = log1p(S1);
        double lse = (double)m + excess;
        if (lse_out) lse_out[d] = lse;
        for (int v = 0; v < V; ++v) {
            e[v].logit = row[v];
            e[v].id = v;
        }
        qsort(e, (size_t)V, sizeof(tok_entry), cmp_tok_entry);
        for (int k = 0; k < K; ++k) {
            tok[(size_t)d * K + k] = e[k].id;
            lp[(size_t)d * K + k] = (float)(((double)e[k].logit - (double)m) - excess);
        }
        free(e);
    }
    return status;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1: best-first construction with a max-heap.               */
/* ------------------------------------------------------------------ */

typedef struct {
    float score;     /* sigma of the candidate prefix (reading R3)            */
    int32_t parent;  /* node id of the candidate's parent prefix (0 = root)   */
    int32_t depth;   /* length d of the rank tuple, 1-based                   */
    int32_t rank;    /* last rank rho_d, 0-based                              */
} cand;

typedef struct {
    const int32_t *parent; /* per already-popped node */
    const int32_t *rank;
} tree_view;

/*
 * Reading R2.  A candidate's rank tuple is (tuple of its parent node, rank).
 * Walk both tuples up to a common depth, then up together until they hang off
 * the same parent; the ranks at that level are the first position where the
 * two tuples differ.  If they never differ one tuple is a prefix of the other
 * and the shorter one comes first.
 */
static int tuple_before(const tree_view *t, const cand *a, const cand *b)
{
    int32_t pa = a->parent, ra = a->rank, da = a->depth;
    int32_t pb = b->parent, rb = b->rank, db = b->depth;
    while (da > db) {
        ra = t->rank[pa];
        pa = t->parent[pa];
        --da;
    }
    while (db > da) {
        rb = t->rank[pb];
        pb = t->parent[pb];
        --db;
    }
    while (pa != pb) {
        ra = t->rank[pa];
        pa = t->parent[pa];
        rb = t->rank[pb];
        pb = t->parent[pb];
    }
    if (ra != rb) return ra < rb;
    return a->depth < b->depth;
}

/* 1 if candidate a must be popped before candidate b. */
static int cand_before(const tree_view *t, const cand *a, const cand *b)
{
    if (a->score > b->score) return 1;
    if (a->score < b->score) return 0;
    return tuple_before(t, a, b);
}

static void heap_push(cand *h, int *n, cand c, const tree_view *t)
{
    int i = (*n)++;
    h[i] = c;
    while (i > 0) {
        int up = (i - 1) / 2;
        if (!cand_before(t, &h[i], &h[up])) break;
        cand tmp = h[i];
        h[i] = h[up];
        h[up] = tmp;
        i = up;
    }
}

static cand heap_pop(cand *h, int *n, const tree_view *t)
{
    cand top = h[0];
    h[0] = h[--(*n)];
    int i = 0;
    for (;;) {
        int l = 2 * i + 1, r = l + 1, best = i;
        if (l < *n && cand_before(t, &h[l], &h[best])) best = l;
        if (r < *n && cand_before(t, &h[r], &h[best])) best = r;
        if (best == i) break;
        cand tmp = h[i];
        h[i] = h[best];
        h[best] = tmp;
        i = best;
    }
    return top;
}

/*
 * Inputs: tok[B][K], lp[B][K] (rank-ordered per depth), node budget N, the
 * bonus token that becomes the root.
 * Outputs, all of length N+1: tokens, parent (parent[0] = -1), depth
 * (depth[0] = 0), rank (rank[0] = -1), score (score[0] = 0).  Rows past
 * *n_nodes (the heap ran dry, only possible when fewer than N prefixes exist)
 * hold -1 / 0.  *max_heap (nullable) receives the largest heap occupancy seen,
 * so that the Remark's "heap size O(N)" bound can be tested.
 * Returns 0, or a negative number for bad arguments.
 */
int oracle_build(const int32_t *tok, const float *lp, int B, int K, int N, int32_t root_token,
                 int32_t *tokens, int32_t *parent, int32_t *depth, int32_t *rank, float *score,
                 int32_t *n_nodes, int32_t *max_heap)
{
    if (B < 1 || K < 1 || N < 1) return -1;
    cand *heap = (cand *)malloc((size_t)(2 * N + 2) * sizeof(cand));
    if (!heap) return -2;
    for (int i = 0; i <= N; ++i) {
        tokens[i] = -1;
        parent[i] = -1;
        depth[i] = -1;
        rank[i] = -1;
        score[i] = 0.0f;
    }
    tokens[0] = root_token;
    depth[0] = 0;
    tree_view view = {parent, rank};

    int hn = 0, hmax = 0, n = 0;
    /* H <- {((1), sigma((1)))} */
    cand first = {lp[0], 0, 1, 0};
    heap_push(heap, &hn, first, &view);
    hmax = hn;
    while (n < N && hn > 0) {
        cand c = heap_pop(heap, &hn, &view);
        int id = ++n;
        tokens[id] = tok[(size_t)(c.depth - 1) * K + c.rank];
        parent[id] = c.parent;
        depth[id] = c.depth;
        rank[id] = c.rank;
        score[id] = c.score;
        if (c.rank + 1 < K) { /* next sibling */
            cand s = {score[c.parent] + lp[(size_t)(c.depth - 1) * K + c.rank + 1], c.parent,
                      c.depth, c.rank + 1};
            heap_push(heap, &hn, s, &view);
        }
        if (c.depth < B) { /* first child */
            cand ch = {c.score + lp[(size_t)c.depth * K + 0], id, c.depth + 1, 0};
            heap_push(heap, &hn, ch, &view);
        }
        if (hn > hmax) hmax = hn;
    }
    *n_nodes = n;
    if (max_heap) *max_heap = hmax;
    free(heap);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Section 4.4: tree attention visibility.                             */
/* ------------------------------------------------------------------ */

/*
 * mask[i][w] bit b set  <=>  node j = 64*w + b is the root, an ancestor of i,
 * or i itself.  T rows of W = ceil(T/64) words; rows >= n_nodes+1 are zero.
 */
int oracle_ancestor_mask(const int32_t *parent, int n_nodes, int T, uint64_t *mask)
{
    if (T < 1 || n_nodes + 1 > T) return -1;
    int W = (T + 63) / 64;
    memset(mask, 0, (size_t)T * W * sizeof(uint64_t));
    for (int i = 0; i <= n_nodes; ++i) {
        int j = i;
        while (j >= 0) {
            mask[(size_t)i * W + (j >> 6)] |= (uint64_t)1 << (j & 63);
            j = parent[j];
        }
    }
    return 0;
}

/*
 * One (node i, query head h) attention row, exactly as defined: the visible
 * keys are all L cache rows, then the tree rows whose mask bit is set; scores
 * q.k * scale in fp64; softmax; weighted sum of the value rows in fp64.
 * Layouts are token-major: q[T][Hq][D], k_cache/v_cache[L][Hkv][D],
 * k_tree/v_tree[T][Hkv][D].  Query head h reads KV head h / (Hq/Hkv).
 */
static void attn_row(const float *q, const float *k_cache, const float *v_cache,
                     const float *k_tree, const float *v_tree, const uint64_t *mask, int L, int T,
                     int Hq, int Hkv, int D, double scale, int i, int h, double *w, double *out)
{
    int W = (T + 63) / 64;
    int hk = h / (Hq / Hkv);
    const float *qi = q + ((size_t)i * Hq + h) * D;
    int n = 0;
    for (int c = 0; c < D; ++c) out[c] = 0.0;
    /* every real node sees itself; a row whose own bit is clear is padding: output zero */
    if (!((mask[(size_t)i * W + (i >> 6)] >> (i & 63)) & 1)) return;
    double mx = -INFINITY;
    for (int j = 0; j < L; ++j) {
        const float *kj = k_cache + ((size_t)j * Hkv + hk) * D;
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += (double)qi[c] * (double)kj[c];
        s *= scale;
        w[n++] = s;
        if (s > mx) mx = s;
    }
    for (int j = 0; j < T; ++j) {
        if (!((mask[(size_t)i * W + (j >> 6)] >> (j & 63)) & 1)) continue;
        const float *kj = k_tree + ((size_t)j * Hkv + hk) * D;
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += (double)qi[c] * (double)kj[c];
        s *= scale;
        w[n++] = s;
        if (s > mx) mx = s;
    }
    double Z = 0.0;
    for (int t = 0; t < n; ++t) {
        w[t] = exp(w[t] - mx);
        Z += w[t];
    }
    n = 0;
    for (int j = 0; j < L; ++j) {
        const float *vj = v_cache + ((size_t)j * Hkv + hk) * D;
        double p = w[n++] / Z;
        for (int c = 0; c < D; ++c) out[c] += p * (double)vj[c];
    }
    for (int j = 0; j < T; ++j) {
        if (!((mask[(size_t)i * W + (j >> 6)] >> (j & 63)) & 1)) continue;
        const float *vj = v_tree + ((size_t)j * Hkv + hk) * D;
        double p = w[n++] / Z;
        for (int c = 0; c < D; ++c) out[c] += p * (double)vj[c];
    }
}

/*
 * Attention for a list of (node, head) pairs: out[r][D] for pair r.  With
 * pairs == NULL all T*Hq rows are computed in (node, head) order, i.e. out has
 * the layout [T][Hq][D].
 */
int oracle_verify_attn(const float *q, const float *k_cache, const float *v_cache,
                       const float *k_tree, const float *v_tree, const uint64_t *mask, int L,
                       int T, int Hq, int Hkv, int D, double scale, const int32_t *pairs,
                       int n_pairs, double *out)
{
    if (L < 0 || T < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1) return -1;
    int total = pairs ? n_pairs : T * Hq;
    int status = 0;
#pragma omp parallel
    {
        double *w = (double *)malloc((size_t)(L + T) * sizeof(double));
        if (!w) status = -2;
#pragma omp for schedule(dynamic, 4)
        for (int r = 0; r < total; ++r) {
            if (!w) continue;
            int i = pairs ? pairs[2 * r] : r / Hq;
            int h = pairs ? pairs[2 * r + 1] : r % Hq;
            attn_row(q, k_cache, v_cache, k_tree, v_tree, mask, L, T, Hq, Hkv, D, scale, i, h, w,
                     out + (size_t)r * D);
        }
        free(w);
    }
    return status;
}

/* ------------------------------------------------------------------ */
/* Section 4.4 / Figure 1b: greedy verifier walk.                      */
/* ------------------------------------------------------------------ */

/*
 * posterior[i] = argmax_v target_logits[i][v] (first maximum, so the lower id
 * wins a tie).  Walk from the root: while the current node has a child whose
 * token equals the target's choice at the current node, accept that child.
 * path[0] = 0 and path[1..n_accepted] are the accepted node ids (path has
 * B + 1 slots, unused ones are -1); bonus = the target's choice at the last
 * node of the path, i.e. the first unmatched target token.
 * Rows i > n_nodes are ignored (posterior -1).
 */
int oracle_accept(const float *target_logits, int T, int V, const int32_t *tokens,
                  const int32_t *parent, int n_nodes, int B, int32_t *path, int32_t *n_accepted,
                  int32_t *bonus, int32_t *posterior)
{
    if (T < 1 || V < 1 || n_nodes + 1 > T || B < 1) return -1;
    int32_t *post = posterior ? posterior : (int32_t *)malloc((size_t)T * sizeof(int32_t));
    if (!post) return -2;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < T; ++i) {
        if (i > n_nodes) {
            post[i] = -1;
            continue;
        }
        const float *row = target_logits + (size_t)i * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > row[best]) best = v;
        post[i] = best;
    }
    for (int s = 0; s <= B; ++s) path[s] = -1;
    int cur = 0, len = 0;
    path[0] = 0;
    for (;;) {
        int next = -1;
        for (int c = 1; c <= n_nodes; ++c) {
            if (parent[c] == cur && tokens[c] == post[cur]) {
                next = c;
                break;
            }
        }
        if (next < 0 || len >= B) break;
        cur = next;
        path[++len] = cur;
    }
    *n_accepted = len;
    *bonus = post[cur];
    if (!posterior) free(post);
    return 0;
}

/*
 * Section 4.4, second paragraph: verification "follows the target model's own decoding rule,
 * whether greedy or temperature-based sampling".  At temperature tau > 0 the token the target
 * selects at node i is a sample from softmax(target_logits[i] / tau).  The sample is drawn by
 * the Gumbel-max rule, argmax_v (logit[v] / tau + g[v]) with g = -log(-log(u)) and u uniform on
 * (0,1), which is distributed exactly as that softmax; u comes from a counter-based generator
 * keyed by (seed, row, v) so that the draw does not depend on any order of evaluation:
 *     mix(x):  x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16
 *     h = mix(mix(v ^ seed_lo) + 0x9E3779B9 * row + seed_hi)          (32-bit arithmetic)
 *     u = ((h >> 8) + 0.5) / 2^24
 * with row = first_row + i.  Everything here is fp64.  Besides the selected token the function
 * reports the runner-up and the gap between their keys, so that a caller comparing against an
 * fp32 implementation knows which decisions are closer than fp32 can resolve.
 */
static uint32_t sample_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

double oracle_sample_uniform(uint64_t seed, uint32_t row, uint32_t v)
{
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
    const uint32_t h = sample_mix(sample_mix(v ^ lo) + 0x9E3779B9u * row + hi);
    return ((double)(h >> 8) + 0.5) / 16777216.0;
}

int oracle_sample_tokens(const float *target_logits, int T, int V, int n_nodes, double temperature,
                         uint64_t seed, int first_row, int32_t *token, int32_t *runner_up,
                         double *gap)
{
    if (T < 1 || V < 1 || n_nodes + 1 > T || !(temperature > 0.0)) return -1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < T; ++i) {
        if (i > n_nodes) {
            token[i] = -1;
            if (runner_up) runner_up[i] = -1;
            if (gap) gap[i] = 0.0;
            continue;
        }
        const float *row = target_logits + (size_t)i * V;
        int best = -1, second = -1;
        double kbest = 0.0, ksecond = 0.0;
        for (int v = 0; v < V; ++v) {
            const double u = oracle_sample_uniform(seed, (uint32_t)(first_row + i), (uint32_t)v);
            const double key = (double)row[v] / temperature - log(-log(u));
            if (best < 0 || key > kbest) {
                second = best;
                ksecond = kbest;
                best = v;
                kbest = key;
            } else if (second < 0 || key > ksecond) {
                second = v;
                ksecond = key;
            }
        }
        token[i] = best;
        if (runner_up) runner_up[i] = second;
        if (gap) gap[i] = second >= 0 ? kbest - ksecond : INFINITY;
    }
    return 0;
}

/* The walk of Section 4.4 with `selected[i]` as the token the target chose at node i. */
int oracle_walk(const int32_t *selected, const int32_t *tokens, const int32_t *parent, int n_nodes,
                int B, int32_t *path, int32_t *n_accepted, int32_t *bonus)
{
    if (B < 1) return -1;
    for (int s = 0; s <= B; ++s) path[s] = -1;
    int cur = 0, len = 0;
    path[0] = 0;
    for (;;) {
        int next = -1;
        for (int c = 1; c <= n_nodes; ++c) {
            if (parent[c] == cur && tokens[c] == selected[cur]) {
                next = c;
                break;
            }
        }
        if (next < 0 || len >= B) break;
        cur = next;
        path[++len] = cur;
    }
    *n_accepted = len;
    *bonus = selected[cur];
    return 0;
}

/*
 * Section 4.4, last sentence: after the walk the cache keeps only the accepted
 * path.  Rows path[0..n_accepted] of the tree K (or V) are appended to the
 * cache at rows L, L+1, ...; row_elems = Hkv * D.
 */
int oracle_compact(const float *tree_rows, const int32_t *path, int n_accepted, int row_elems,
                   int L, float *cache)
{
    if (n_accepted < 0 || row_elems < 1 || L < 0) return -1;
    for (int s = 0; s <= n_accepted; ++s)
        memcpy(cache + (size_t)(L + s) * row_elems, tree_rows + (size_t)path[s] * row_elems,
               (size_t)row_elems * sizeof(float));
    return 0;
}
