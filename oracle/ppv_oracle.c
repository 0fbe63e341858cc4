/*
 * CPU oracle for set-constrained decoding.  TEST INFRASTRUCTURE ONLY: it exists to check the
 * HIP path and to be timed beside it.  It shares no code with the HIP path and the product
 * never calls it.
 *
 * What it computes, and where the paper defines it:
 *   - the valid set A_{x,S} = { v : exists s in S with x+[v] a prefix of s }   (Section 2.1,
 *     "Constrained decoding"), obtained by walking a pointer-based prefix tree in which V is a
 *     child of node x iff V is in A_{x,S}                                      (Section 2.1,
 *     "Prefix-tree");
 *   - the rank range [lo,hi) that the prefix x occupies in S sorted lexicographically by token
 *     id, left to right, a proper prefix before its extensions                 (Section 3.2,
 *     "Array Preparation"; Algorithm 2, "Prepare").  lo = #{s in S : s < x}; hi - lo =
 *     #{s in S : x is a prefix of s}.  For an x that is a prefix of no member, lo = hi = the
 *     rank at which x would be inserted (the lower bound the binary search of Section 3.2,
 *     "Parallel Verification", ends on);
 *   - member = (x in S), the loop condition of Algorithm 1, SampleCandidate;
 *   - one constrained decoding step of Algorithm 1 (the body of SampleCandidate's loop: next-token
 *     distribution, valid set, draw, update of x): with P = softmax(logits / T), T the temperature that Algorithm 1 takes as input
 *     (the experiments of Section 4.1 "Methods" use T = 1),
 *     logZ_valid = log |P (.) mask|_1 = LSE_{v in mask} l_v - LSE_{all v} l_v, and a token drawn
 *     from P (.) mask / |P (.) mask|_1.  The paper names no sampling procedure; this oracle fixes
 *     inverse-CDF over the valid tokens in increasing token id with a supplied uniform u:
 *     the first valid v whose cumulative weight exceeds u * (total valid weight).
 *
 *   - Algorithm 2 as printed, with M candidates instead of the whole vocabulary (second half of
 *     this file): sorted array, top M, one binary search per candidate row, prefix check.
 *
 * Every function here is pinned by tests that do not go through this file's own arithmetic (brute force from
 * the definitions, closed forms, library routines on special cases, the paper's worked numbers).  One worked
 * example of the paper could not be used -- parity unpinned: the PPV illustration (input [0,31,555] with
 * candidates {35,145,111}), whose array and resulting mask exist only in a figure.
 *
 * Everything floating point is done in double, sequentially in increasing token id.
 * Query tokens are compared as unsigned 32-bit integers, so a token outside [0,V) simply
 * matches nothing and sorts after every real token.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct onode {
    struct onode **child; /* children, sorted by key */
    uint32_t *key;        /* key[i] = token on the edge to child[i] */
    int64_t count;        /* members of S in this subtree, this node included if terminal */
    int32_t nchild, cap;
    int32_t terminal;     /* 1 iff the path from the root to here is a member of S */
} onode;

#define POOL_CHUNK (1 << 16)
typedef struct pool_chunk {
    struct pool_chunk *next;
    onode nodes[POOL_CHUNK];
} pool_chunk;

typedef struct {
    onode *root;
    pool_chunk *chunks;
    int32_t used_in_chunk;
    int64_t n_nodes, n_members;
    int32_t vocab, l_max;
} otrie;

static onode *new_node(otrie *t) {
    if (!t->chunks || t->used_in_chunk == POOL_CHUNK) {
        pool_chunk *c = (pool_chunk *)malloc(sizeof(pool_chunk));
        if (!c) return NULL;
        c->next = t->chunks;
        t->chunks = c;
        t->used_in_chunk = 0;
    }
    onode *n = &t->chunks->nodes[t->used_in_chunk++];
    memset(n, 0, sizeof(*n));
    t->n_nodes++;
    return n;
}

/* index of the first child whose key is >= k (unsigned compare) */
static int32_t child_lower_bound(const onode *n, uint32_t k) {
    int32_t a = 0, b = n->nchild;
    while (a < b) {
        int32_t m = a + (b - a) / 2;
        if (n->key[m] < k) a = m + 1; else b = m;
    }
    return a;
}

static onode *get_or_add_child(otrie *t, onode *n, uint32_t k) {
    int32_t i = child_lower_bound(n, k);
    if (i < n->nchild && n->key[i] == k) return n->child[i];
    if (n->nchild == n->cap) {
        int32_t cap = n->cap ? n->cap * 2 : 2;
        onode **c = (onode **)realloc(n->child, (size_t)cap * sizeof(onode *));
        if (!c) return NULL;
        n->child = c;
        uint32_t *kk = (uint32_t *)realloc(n->key, (size_t)cap * sizeof(uint32_t));
        if (!kk) return NULL;
        n->key = kk;
        n->cap = cap;
    }
    memmove(n->child + i + 1, n->child + i, (size_t)(n->nchild - i) * sizeof(onode *));
    memmove(n->key + i + 1, n->key + i, (size_t)(n->nchild - i) * sizeof(uint32_t));
    onode *c = new_node(t);
    if (!c) return NULL;
    n->child[i] = c;
    n->key[i] = k;
    n->nchild++;
    return c;
}

void oracle_trie_free(otrie *t);

/* S as CSR on the host.  Returns NULL on invalid input (no sequences, an empty sequence, a token
 * outside [0,vocab)) or when memory runs out.  Duplicates are inserted once: S is a set. */
otrie *oracle_trie_build(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab) {
    if (n_seq <= 0 || vocab <= 0) return NULL;
    otrie *t = (otrie *)calloc(1, sizeof(otrie));
    if (!t) return NULL;
    t->vocab = vocab;
    t->root = new_node(t);
    if (!t->root) { free(t); return NULL; }
    for (int64_t i = 0; i < n_seq; i++) {
        int64_t a = offsets[i], b = offsets[i + 1];
        if (b <= a) { oracle_trie_free(t); return NULL; }
        onode *n = t->root;
        for (int64_t j = a; j < b; j++) {
            if (tokens[j] < 0 || tokens[j] >= vocab) { oracle_trie_free(t); return NULL; }
            n = get_or_add_child(t, n, (uint32_t)tokens[j]);
            if (!n) { oracle_trie_free(t); return NULL; }
        }
        if (!n->terminal) {
            n->terminal = 1;
            t->n_members++;
            if (b - a > t->l_max) t->l_max = (int32_t)(b - a);
            /* a new member: one more in every subtree along its path */
            onode *p = t->root;
            p->count++;
            for (int64_t j = a; j < b; j++) {
                p = p->child[child_lower_bound(p, (uint32_t)tokens[j])];
                p->count++;
            }
        }
    }
    return t;
}

void oracle_trie_free(otrie *t) {
    if (!t) return;
    for (pool_chunk *c = t->chunks; c;) {
        int32_t used = (c == t->chunks) ? t->used_in_chunk : POOL_CHUNK;
        for (int32_t i = 0; i < used; i++) { free(c->nodes[i].child); free(c->nodes[i].key); }
        pool_chunk *nx = c->next;
        free(c);
        c = nx;
    }
    free(t);
}

int64_t oracle_trie_members(const otrie *t) { return t->n_members; }
int64_t oracle_trie_nodes(const otrie *t) { return t->n_nodes; }
int32_t oracle_trie_lmax(const otrie *t) { return t->l_max; }

/* One prefix.  mask is one byte per token (0/1), length vocab, fully written. */
void oracle_query(const otrie *t, const int32_t *prefix, int32_t len, uint8_t *mask /* [vocab], may be NULL */,
                  int64_t *lo, int64_t *hi, int32_t *member) {
    if (mask) memset(mask, 0, (size_t)t->vocab);
    const onode *n = t->root;
    int64_t acc = 0; /* members known to sort before the prefix */
    for (int32_t i = 0; i < len; i++) {
        uint32_t k = (uint32_t)prefix[i];
        if (n->terminal) acc += 1;             /* the member ending here is a proper prefix: smaller */
        int32_t c = -1;
        for (int32_t j = 0; j < n->nchild; j++) { /* whole subtrees under smaller tokens are smaller */
            if (n->key[j] < k) acc += n->child[j]->count;
            else { if (n->key[j] == k) c = j; break; }
        }
        if (c < 0) { *lo = acc; *hi = acc; *member = 0; return; }
        n = n->child[c];
    }
    *lo = acc;
    *hi = acc + n->count;
    *member = (len > 0) ? n->terminal : 0;
    if (mask)
        for (int32_t j = 0; j < n->nchild; j++) mask[n->key[j]] = 1;
}

/* One row of the constrained step.  logits are fp32 (a bf16 logit is widened exactly by the
 * caller), mask is one byte per token, T > 0 is the temperature: every logit is divided by T (in
 * double) before anything else.  Outputs:
 *   id          sampled token, -1 when the mask is empty
 *   logZ_valid  log of the probability mass on valid tokens (-inf when the mask is empty)
 *   logZ_all    log-sum-exp of all logits
 *   cdf_lo/hi   the normalised cumulative weights just before and just after the chosen token,
 *               so that a caller can tell how close u was to a boundary. */
void oracle_masked_sample(const float *logits, int64_t V, const uint8_t *mask, double u, double T, int32_t *id,
                          double *logZ_valid, double *logZ_all, double *cdf_lo, double *cdf_hi) {
    double m_all = -INFINITY, m_val = -INFINITY;
    for (int64_t v = 0; v < V; v++) {
        double l = (double)logits[v] / T;
        if (l > m_all) m_all = l;
        if (mask[v] && l > m_val) m_val = l;
    }
    double z_all = 0.0;
    for (int64_t v = 0; v < V; v++) z_all += exp((double)logits[v] / T - m_all);
    *logZ_all = m_all + log(z_all);
    int any = 0;
    for (int64_t v = 0; v < V; v++) any |= mask[v];
    /* no valid token, or none with positive probability: nothing can be sampled */
    if (!any || m_val == -INFINITY) { *id = -1; *logZ_valid = -INFINITY; *cdf_lo = 0.0; *cdf_hi = 0.0; return; }
    double z_val = 0.0;
    for (int64_t v = 0; v < V; v++)
        if (mask[v]) z_val += exp((double)logits[v] / T - m_val);
    *logZ_valid = (m_val + log(z_val)) - *logZ_all;
    double tau = u * z_val, c = 0.0, c_prev = 0.0;
    int64_t pick = -1, last_pos = -1;
    double last_lo = 0.0, last_hi = 0.0;
    for (int64_t v = 0; v < V; v++) {
        if (!mask[v]) continue;
        double w = exp((double)logits[v] / T - m_val);
        c_prev = c;
        c += w;
        if (w > 0.0) { last_pos = v; last_lo = c_prev; last_hi = c; }
        if (c > tau) { pick = v; break; }
    }
    if (pick < 0) { pick = last_pos; c_prev = last_lo; c = last_hi; } /* rounding: u*Z never exceeded */
    *id = (int32_t)pick;
    *cdf_lo = c_prev / z_val;
    *cdf_hi = c / z_val;
}

/* A batch of independent rows: query + constrained step per row, `threads` OpenMP threads over
 * rows (1 = plain serial loop).  Any output pointer may be NULL.  mask_out is [B, vocab] bytes. */
void oracle_step_batch(const otrie *t, const int32_t *prefixes, int32_t stride, const int32_t *lens, int32_t B,
                       const float *logits /* [B, V] or NULL: query only */, const float *uniforms,
                       uint8_t *mask_out, int64_t *lo, int64_t *hi, int32_t *member, int32_t *ids,
                       double *logZ_valid, double *logZ_all, double *cdf_lo, double *cdf_hi, int32_t threads,
                       double temperature) {
    int64_t V = t->vocab;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int32_t b = 0; b < B; b++) {
        uint8_t *mrow = mask_out ? mask_out + (size_t)b * (size_t)V : (uint8_t *)malloc((size_t)V);
        int64_t l, h;
        int32_t mem;
        oracle_query(t, prefixes + (size_t)b * (size_t)stride, lens[b], mrow, &l, &h, &mem);
        if (lo) lo[b] = l;
        if (hi) hi[b] = h;
        if (member) member[b] = mem;
        if (logits) {
            int32_t id;
            double zv, za, cl, ch;
            oracle_masked_sample(logits + (size_t)b * (size_t)V, V, mrow, (double)uniforms[b], temperature, &id, &zv, &za, &cl,
                                 &ch);
            if (ids) ids[b] = id;
            if (logZ_valid) logZ_valid[b] = zv;
            if (logZ_all) logZ_all[b] = za;
            if (cdf_lo) cdf_lo[b] = cl;
            if (cdf_hi) cdf_hi[b] = ch;
        }
        if (!mask_out) free(mrow);
    }
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 2 as printed (the variant with M < |V| candidates), by its own steps and on its own
 * data structure: the array X of all members in lexicographic order, searched row against row.
 * Nothing here uses the prefix tree above.
 *
 *   Prepare        X = the distinct members of S sorted by token id, left to right; the padding
 *                  that fills a shorter row sorts before every token, so a member precedes its
 *                  extensions (rows are kept at their own length; "past the end" plays the pad).
 *   top M          the M tokens of largest probability.  P = softmax(logits) is increasing in the
 *                  logit, so the order is the logits' order; equal logits (always present with
 *                  bf16) are ordered by increasing token id so that the set is unique.
 *   candidates     V_i = a + [t_i]
 *   search         i_m = the first row of X that is not smaller than V_i (binary search)
 *   check          mask_V[i] = 1 iff V_i is a prefix of X[i_m]
 *   extend         mask[t_i] = mask_V[i], every other token 0
 */
typedef struct {
    int32_t *tok;   /* rows back to back */
    int64_t *off;   /* [n + 1] */
    int64_t n;
    int32_t vocab;
} osorted;

static const int32_t *g_sort_tok;   /* qsort has no context argument; builds are not concurrent */
static const int64_t *g_sort_off;

/* lexicographic order of two token strings, unsigned token compare, the shorter first on a tie */
static int lex_cmp(const int32_t *a, int64_t la, const int32_t *b, int64_t lb) {
    int64_t m = la < lb ? la : lb;
    for (int64_t i = 0; i < m; i++) {
        uint32_t x = (uint32_t)a[i], y = (uint32_t)b[i];
        if (x != y) return x < y ? -1 : 1;
    }
    return la < lb ? -1 : (la > lb ? 1 : 0);
}
static int row_cmp(const void *pa, const void *pb) {
    int64_t a = *(const int64_t *)pa, b = *(const int64_t *)pb;
    return lex_cmp(g_sort_tok + g_sort_off[a], g_sort_off[a + 1] - g_sort_off[a], g_sort_tok + g_sort_off[b],
                   g_sort_off[b + 1] - g_sort_off[b]);
}

void oracle_sorted_free(osorted *x) {
    if (!x) return;
    free(x->tok);
    free(x->off);
    free(x);
}

osorted *oracle_sorted_build(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab) {
    if (n_seq <= 0 || vocab <= 0) return NULL;
    for (int64_t i = 0; i < n_seq; i++) {
        if (offsets[i + 1] <= offsets[i]) return NULL;
        for (int64_t j = offsets[i]; j < offsets[i + 1]; j++)
            if (tokens[j] < 0 || tokens[j] >= vocab) return NULL;
    }
    int64_t *order = (int64_t *)malloc((size_t)n_seq * sizeof(int64_t));
    osorted *x = (osorted *)calloc(1, sizeof(osorted));
    if (!order || !x) { free(order); free(x); return NULL; }
    for (int64_t i = 0; i < n_seq; i++) order[i] = i;
    g_sort_tok = tokens;
    g_sort_off = offsets;
    qsort(order, (size_t)n_seq, sizeof(int64_t), row_cmp);
    x->tok = (int32_t *)malloc((size_t)(offsets[n_seq] > 0 ? offsets[n_seq] : 1) * sizeof(int32_t));
    x->off = (int64_t *)malloc((size_t)(n_seq + 1) * sizeof(int64_t));
    if (!x->tok || !x->off) { free(order); oracle_sorted_free(x); return NULL; }
    x->vocab = vocab;
    x->off[0] = 0;
    for (int64_t i = 0; i < n_seq; i++) {
        int64_t r = order[i], len = offsets[r + 1] - offsets[r];
        if (x->n > 0 && lex_cmp(tokens + offsets[r], len, x->tok + x->off[x->n - 1], x->off[x->n] - x->off[x->n - 1]) == 0)
            continue; /* S is a set */
        memcpy(x->tok + x->off[x->n], tokens + offsets[r], (size_t)len * sizeof(int32_t));
        x->off[x->n + 1] = x->off[x->n] + len;
        x->n++;
    }
    free(order);
    return x;
}
int64_t oracle_sorted_rows(const osorted *x) { return x->n; }

typedef struct { float l; int32_t id; } scored;
static int scored_cmp(const void *pa, const void *pb) { /* larger logit first, then smaller id */
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (a->l > b->l) return -1;
    if (a->l < b->l) return 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

/* One row.  top_ids[M] and mask_V[M]: candidate i and its verdict, in order of decreasing
 * probability; only the first min(M, V) are meaningful, the rest are -1 / 0.  mask[V] (may be
 * NULL): one byte per token.  Returns the number of candidates, or -1 when memory runs out. */
int32_t oracle_topm_row(const osorted *x, const int32_t *prefix, int32_t len, const float *logits, int32_t M,
                        int32_t *top_ids, uint8_t *mask_V, uint8_t *mask) {
    const int64_t V = x->vocab;
    scored *sc = (scored *)malloc((size_t)V * sizeof(scored));
    int32_t *cand = (int32_t *)malloc(((size_t)len + 1) * sizeof(int32_t));
    if (!sc || !cand) { free(sc); free(cand); return -1; }
    for (int64_t v = 0; v < V; v++) { sc[v].l = logits[v]; sc[v].id = (int32_t)v; }
    qsort(sc, (size_t)V, sizeof(scored), scored_cmp);
    const int32_t m = M < V ? M : (int32_t)V;
    if (mask) memset(mask, 0, (size_t)V);
    memcpy(cand, prefix, (size_t)len * sizeof(int32_t));
    for (int32_t i = 0; i < M; i++) {
        top_ids[i] = -1;
        mask_V[i] = 0;
        if (i >= m) continue;
        top_ids[i] = sc[i].id;
        cand[len] = sc[i].id;
        int64_t lo = 0, hi = x->n; /* first row that is not smaller than the candidate */
        while (lo < hi) {
            int64_t mid = lo + (hi - lo) / 2;
            if (lex_cmp(x->tok + x->off[mid], x->off[mid + 1] - x->off[mid], cand, (int64_t)len + 1) < 0) lo = mid + 1;
            else hi = mid;
        }
        if (lo < x->n && x->off[lo + 1] - x->off[lo] >= (int64_t)len + 1 &&
            lex_cmp(x->tok + x->off[lo], (int64_t)len + 1, cand, (int64_t)len + 1) == 0)
            mask_V[i] = 1;
        if (mask && mask_V[i]) mask[sc[i].id] = 1;
    }
    free(sc);
    free(cand);
    return m;
}

void oracle_topm_batch(const osorted *x, const int32_t *prefixes, int32_t stride, const int32_t *lens, int32_t B,
                       const float *logits /* [B, V] */, int32_t M, int32_t *top_ids /* [B, M] */,
                       uint8_t *mask_V /* [B, M] */, uint8_t *mask /* [B, V] or NULL */, int32_t threads) {
    const int64_t V = x->vocab;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int32_t b = 0; b < B; b++)
        oracle_topm_row(x, prefixes + (size_t)b * (size_t)stride, lens[b], logits + (size_t)b * (size_t)V, M,
                        top_ids + (size_t)b * (size_t)M, mask_V + (size_t)b * (size_t)M,
                        mask ? mask + (size_t)b * (size_t)V : NULL);
}

/* masked softmax mass + inverse-CDF sample for rows whose masks are given (one byte per token) */
void oracle_sample_batch(const float *logits, int64_t V, const uint8_t *mask, const float *uniforms, int32_t B,
                         int32_t *ids, double *logZ_valid, double *logZ_all, double *cdf_lo, double *cdf_hi,
                         int32_t threads, double temperature) {
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int32_t b = 0; b < B; b++)
        oracle_masked_sample(logits + (size_t)b * (size_t)V, V, mask + (size_t)b * (size_t)V, (double)uniforms[b],
                             temperature, ids + b, logZ_valid + b, logZ_all + b, cdf_lo + b, cdf_hi + b);
}

/* which ppv_oracle.c this library was compiled from (the build passes the digest of the source file) */
#ifndef ORACLE_SOURCE_DIGEST
#define ORACLE_SOURCE_DIGEST "unstamped"
#endif
const char *oracle_source_digest(void) { return ORACLE_SOURCE_DIGEST; }

int32_t oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
