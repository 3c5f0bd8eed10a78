/*
 * CPU oracle for approximate kNN-graph construction (EFANNA, arXiv 1609.07228):
 * randomized truncated KD-trees (Alg. 2), the conquer step of the
 * divide-and-conquer initialisation (Alg. 3: the point's own leaf in every tree
 * and, above the conquer-to depth, one leaf of every sibling subtree on the way
 * up), NN-descent refinement (Alg. 4) and the search with the finished index
 * (Alg. 1).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step statement of
 * what the method computes, used only to check the GPU library and to serve as
 * the timed CPU baseline.  It shares no code with the GPU library and nothing
 * in the product path may call it.
 *
 * The method is a randomized heuristic followed by an iteration, so there is no
 * closed form to write down; the oracle follows the algorithms' steps.  Every
 * random or order-dependent choice of the paper is replaced by a seeded,
 * order-independent rule, which makes the whole pipeline a deterministic
 * function of (X, parameters, seed):
 *
 *  - split dimension (Alg. 2, "randomly choose dimension"): uniform over the d
 *    dimensions from a counter-based generator keyed by (seed, tree, heap id of
 *    the node);
 *  - split value (Alg. 2, "mean over the point set"): the mean, evaluated in
 *    exact integer arithmetic on coordinates quantised to 2^-20, so that the
 *    order of summation cannot matter: a point goes left iff cnt*q(x) < sum q;
 *  - a node is a leaf when it holds at most S points (S = largest leaf
 *    population); if a mean split leaves one side empty the node is cut into
 *    positional halves;
 *  - distances are squared L2 in float32, accumulated in 16 interleaved
 *    partial sums that are then added pairwise in a fixed tree; every list is
 *    ordered by (distance, id);
 *  - NN-descent (Alg. 4) uses pool size P = K, takes the L closest new-flagged
 *    entries of each pool as the sampled "new" set, builds reverse lists as the
 *    transpose of the sampled lists capped at L entries by a seeded hash, and
 *    treats the pool update as a set operation: pool := the K smallest
 *    (distance, id) of pool U proposals, an id already present keeping its
 *    entry and flag.
 *
 * Parity pins: see tests/test_oracle_*.py (exact brute force on tiny inputs,
 * structural invariants recomputed independently in Python integers, special
 * cases that reduce to exact kNN).  The number of iterations NN-descent needs
 * to reach a given accuracy is not fixed by anything the paper prints:
 * convergence speed is "parity unpinned" beyond those properties.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* counter-based random numbers                                               */

static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Alg. 2 "randomly choose dimension": one draw per (tree, node). */
uint64_t oracle_node_rand(uint64_t seed, int32_t tree, uint64_t heap_id)
{
    uint64_t s = mix64(seed + 0x9E3779B97F4A7C15ULL * (uint64_t)(tree + 1));
    return mix64(s + heap_id);
}

/* priority of "u is a reverse neighbour of v" when a reverse list overflows */
uint32_t oracle_reverse_hash(uint64_t seed, int32_t iter, int32_t v, int32_t u)
{
    uint64_t s = mix64(seed + 0x9E3779B97F4A7C15ULL * (uint64_t)(iter + 1));
    return (uint32_t)(mix64(s + (((uint64_t)(uint32_t)v << 32) | (uint32_t)u)) >> 32);
}

/* ------------------------------------------------------------------------- */
/* distance: squared L2, float32, 16 interleaved partial sums, fixed tree      */

float oracle_dist(const float *a, const float *b, int32_t d)
{
    float acc[16];
    for (int l = 0; l < 16; ++l) acc[l] = 0.0f;
    for (int32_t j = 0; j < d; ++j) {
        float diff = a[j] - b[j];
        acc[j & 15] = fmaf(diff, diff, acc[j & 15]);
    }
    for (int s = 8; s >= 1; s >>= 1)
        for (int l = 0; l < s; ++l) acc[l] = acc[l] + acc[l + s];
    return acc[0];
}

/* ------------------------------------------------------------------------- */
/* Alg. 2: randomized truncated KD-trees                                       */

static int64_t quantise(float x) { return (int64_t)rint((double)x * 1048576.0); }

/* An internal node as the conquer step of Alg. 3 needs it: the split test
 * (dimension, sum of quantised coordinates, population: a point x goes left iff
 * cnt*q(x[dim]) < sum), its depth (root 0), and links.  Internal nodes are
 * numbered by the index of the leaf that starts their right part (1 ..
 * n_leaves-1: every boundary between two leaves is the split point of exactly
 * one internal node); child[s] >= 0 is such a number, child[s] < 0 is ~(leaf
 * index); parent is -1 at the root. */
typedef struct {
    int64_t sum;
    int32_t dim, cnt, parent, depth;
    int32_t child[2];
} oracle_node;

typedef struct {
    const float *X;
    int64_t n;
    int32_t d, S, tree;
    int32_t split_rule; /* 0: the dimension is drawn uniformly (Alg. 2 as printed), 1: by variance, 2: a random projection */
    uint64_t seed;
    int32_t *perm;     /* this tree's id array, partitioned in place */
    int32_t *tmp;      /* scratch of n ids */
    int32_t *leaf_off; /* this tree's leaf offsets */
    int32_t n_leaves;
    oracle_node *rec;  /* NULL, or n+1 records indexed by the position where the right part starts */
    int32_t *leaf_rec; /* NULL, or for the leaf starting at position b: parent position * 2 + side */
} tree_ctx;

/* What a node's split test looks at.  dim >= 0: the quantised coordinate dim.  dim <= -3: a random
 * projection (the trees the paper's last section proposes to try for high dimensions): the sum
 * of eight quantised coordinates with signs, both drawn from the 30-bit number r = -3 - dim that
 * the node's draw supplies - term k takes z = mix64((r << 8) + k + golden), coordinate z mod d,
 * minus if the top bit of z is set.  Exact in 64-bit integers for n * 8 * |x| < 2^43. */
#define RP_TERMS 8
static int64_t node_value(const float *x, int32_t d, int32_t dim)
{
    if (dim >= 0) return quantise(x[dim]);
    uint64_t r = (uint64_t)(uint32_t)(-3 - dim);
    int64_t v = 0;
    for (int k = 0; k < RP_TERMS; ++k) {
        uint64_t z = mix64((r << 8) + (uint64_t)k + 0x9E3779B97F4A7C15ULL);
        int64_t q = quantise(x[z % (uint64_t)d]);
        v += (z >> 63) ? -q : q;
    }
    return v;
}
/* the dimension code of a projection node from the node's draw */
static int32_t projection_code(uint64_t draw) { return -3 - (int32_t)((draw >> 34) & 0x3FFFFFFFULL); }

/* Split dimension by variance, the rule of the randomized KD-tree that Sec. 3.2 takes over
 * (its trees differ from that one in the leaf size only): estimate every dimension's variance
 * on a sample of the node's points, keep the five dimensions with the largest one and let the
 * node's draw choose among them.  Made exact here: the sample is the first 100 positions of
 * the node (all of them if it has fewer), the coordinates are the quantised ones, the
 * variances are compared as the integers m * sum(q^2) - sum(q)^2, equal ones by the smaller
 * dimension. */
static int32_t variance_dim(const tree_ctx *c, int64_t b, int64_t e, uint64_t draw)
{
    int64_t m = e - b < 100 ? e - b : 100;
    int32_t top[5], n_top = 0;
    __int128 topv[5];
    for (int32_t j = 0; j < c->d; ++j) {
        __int128 s = 0, s2 = 0;
        for (int64_t p = b; p < b + m; ++p) {
            int64_t q = quantise(c->X[(int64_t)c->perm[p] * c->d + j]);
            s += q;
            s2 += (__int128)q * q;
        }
        __int128 v = (__int128)m * s2 - s * s;
        int32_t pos = n_top; /* place among the largest so far: after every one that is >= v */
        while (pos > 0 && topv[pos - 1] < v) --pos;
        if (pos >= 5) continue;
        if (n_top < 5) ++n_top;
        for (int32_t r = n_top - 1; r > pos; --r) {
            top[r] = top[r - 1];
            topv[r] = topv[r - 1];
        }
        top[pos] = j;
        topv[pos] = v;
    }
    return top[draw % (uint64_t)n_top];
}

/* Returns the position where the node's right part starts (internal node) or
 * ~(start position) for a leaf; the caller links it. */
static int64_t build_node(tree_ctx *c, uint64_t heap_id, int32_t depth, int64_t b, int64_t e)
{
    int64_t cnt = e - b;
    if (cnt <= c->S) { /* leaf: record where it starts */
        c->leaf_off[c->n_leaves++] = (int32_t)b;
        return ~b;
    }
    int64_t mid = b; /* first position of the right part */
    int32_t dim = -1;
    int64_t sum = 0;
    if (depth < 60) {
        uint64_t draw = oracle_node_rand(c->seed, c->tree, heap_id);
        dim = c->split_rule == 1   ? variance_dim(c, b, e, draw)
              : c->split_rule == 2 ? projection_code(draw)
                                   : (int32_t)(draw % (uint64_t)c->d);
        for (int64_t p = b; p < e; ++p) sum += node_value(c->X + (int64_t)c->perm[p] * c->d, c->d, dim);
        int64_t nl = 0, nr = 0;
        for (int64_t p = b; p < e; ++p) { /* stable: both parts keep their order */
            int32_t id = c->perm[p];
            if (cnt * node_value(c->X + (int64_t)id * c->d, c->d, dim) < sum) c->perm[b + nl++] = id;
            else c->tmp[nr++] = id;
        }
        memcpy(c->perm + b + nl, c->tmp, (size_t)nr * sizeof(int32_t));
        mid = b + nl;
    }
    if (mid == b || mid == e) mid = b + cnt / 2; /* degenerate: positional halves */
    /* heap ids past depth 60 are never used for a draw; keep them from wrapping */
    uint64_t child = depth < 60 ? 2 * heap_id : heap_id;
    int64_t kid[2];
    kid[0] = build_node(c, child, depth + 1, b, mid);
    kid[1] = build_node(c, child + 1, depth + 1, mid, e);
    if (c->rec) {
        oracle_node *r = &c->rec[mid];
        r->sum = sum;
        r->dim = dim;
        r->cnt = (int32_t)cnt;
        r->depth = depth;
        r->parent = -1; /* the parent fills this in */
        for (int s = 0; s < 2; ++s) {
            r->child[s] = (int32_t)kid[s];
            if (kid[s] >= 0) c->rec[kid[s]].parent = (int32_t)mid;
            else c->leaf_rec[~kid[s]] = (int32_t)(mid * 2 + s);
        }
    }
    return mid;
}

/* perm: [T][n] ids, leaves contiguous, left-to-right.  leaf_off: [T][n+1] start
 * position of every leaf, terminated by n.  n_leaves: [T].
 * nodes (may be NULL): [T][n+1] internal nodes, numbered as described at
 * oracle_node; leaf_up (NULL iff nodes is): [T][n+1], for leaf l the number of its
 * parent node * 2 + (1 if l is the right child), -1 if the tree is one leaf. */
int oracle_build_trees_rule(const float *X, int64_t n, int32_t d, int32_t T, int32_t S,
                            uint64_t seed, int32_t split_rule, int32_t *perm, int32_t *leaf_off,
                            int32_t *n_leaves, oracle_node *nodes, int32_t *leaf_up)
{
    if (!X || n < 1 || d < 1 || T < 1 || S < 1 || (!nodes) != (!leaf_up)) return -1;
    if (split_rule < 0 || split_rule > 2) return -1;
    /* domain of the exact mean test: finite, |x| < 2^20 (so |q| <= 2^40), and n * |x| < 2^43, so
     * that cnt * q(x) and the sum of q over a node stay below 2^63 */
    for (int64_t i = 0; i < n * d; ++i)
        if (!(fabsf(X[i]) < 1048576.0f) ||
            (double)fabsf(X[i]) * (double)n * (split_rule == 2 ? RP_TERMS : 1) >= 8796093022208.0)
            return -3;
    int32_t *tmp = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    oracle_node *rec = nodes ? (oracle_node *)malloc((size_t)(n + 1) * sizeof(oracle_node)) : NULL;
    int32_t *leaf_rec = nodes ? (int32_t *)malloc((size_t)(n + 1) * sizeof(int32_t)) : NULL;
    int32_t *lidx = nodes ? (int32_t *)malloc((size_t)(n + 1) * sizeof(int32_t)) : NULL;
    if (!tmp || (nodes && (!rec || !leaf_rec || !lidx))) return -4;
    for (int32_t t = 0; t < T; ++t) {
        tree_ctx c = {X, n, d, S, t, split_rule, seed, perm + (int64_t)t * n, tmp,
                      leaf_off + (int64_t)t * (n + 1), 0, rec, leaf_rec};
        for (int64_t i = 0; i < n; ++i) c.perm[i] = (int32_t)i;
        if (nodes)
            for (int64_t i = 0; i <= n; ++i) leaf_rec[i] = -1;
        build_node(&c, 1, 0, 0, n);
        c.leaf_off[c.n_leaves] = (int32_t)n;
        n_leaves[t] = c.n_leaves;
        if (!nodes) continue;
        /* positions -> leaf numbers */
        oracle_node *out = nodes + (int64_t)t * (n + 1);
        int32_t *up = leaf_up + (int64_t)t * (n + 1);
        for (int32_t l = 0; l < c.n_leaves; ++l) lidx[c.leaf_off[l]] = l;
        for (int32_t l = 0; l < c.n_leaves; ++l) {
            int32_t b = c.leaf_off[l];
            up[l] = leaf_rec[b] < 0 ? -1 : lidx[leaf_rec[b] >> 1] * 2 + (leaf_rec[b] & 1);
            if (l == 0) continue;
            oracle_node r = rec[b]; /* the node whose right part starts with leaf l */
            r.parent = r.parent < 0 ? -1 : lidx[r.parent];
            for (int s = 0; s < 2; ++s)
                r.child[s] = r.child[s] >= 0 ? lidx[r.child[s]] : ~lidx[~r.child[s]];
            out[l] = r;
        }
    }
    free(tmp);
    free(rec);
    free(leaf_rec);
    free(lidx);
    return 0;
}

int oracle_build_trees_nodes(const float *X, int64_t n, int32_t d, int32_t T, int32_t S,
                             uint64_t seed, int32_t *perm, int32_t *leaf_off, int32_t *n_leaves,
                             oracle_node *nodes, int32_t *leaf_up)
{
    return oracle_build_trees_rule(X, n, d, T, S, seed, 0, perm, leaf_off, n_leaves, nodes, leaf_up);
}

int oracle_build_trees(const float *X, int64_t n, int32_t d, int32_t T, int32_t S, uint64_t seed,
                       int32_t *perm, int32_t *leaf_off, int32_t *n_leaves)
{
    return oracle_build_trees_nodes(X, n, d, T, S, seed, perm, leaf_off, n_leaves, NULL, NULL);
}

/* ------------------------------------------------------------------------- */
/* pools: per point up to K entries sorted by (dist, id); id -1 / +inf = empty  */

typedef struct { float dist; int32_t id; uint8_t is_new; } entry;

static int entry_less(float da, int32_t ia, float db, int32_t ib)
{
    return da < db || (da == db && ia < ib);
}

/* pool := K smallest of pool U {(dist,id,new)}; an id already present is kept
 * as it is.  Returns 1 if the entry went in. */
static int pool_insert_marked(entry *pool, int32_t *cnt, int32_t K, float dist, int32_t id, uint8_t is_new)
{
    for (int32_t s = 0; s < *cnt; ++s)
        if (pool[s].id == id) return 0;
    if (*cnt == K && !entry_less(dist, id, pool[K - 1].dist, pool[K - 1].id)) return 0;
    int32_t s = (*cnt < K) ? (*cnt)++ : K - 1;
    while (s > 0 && entry_less(dist, id, pool[s - 1].dist, pool[s - 1].id)) {
        pool[s] = pool[s - 1];
        --s;
    }
    pool[s].dist = dist;
    pool[s].id = id;
    pool[s].is_new = is_new;
    return 1;
}

static int pool_insert(entry *pool, int32_t *cnt, int32_t K, float dist, int32_t id)
{
    return pool_insert_marked(pool, cnt, K, dist, id, 1);
}

static void pools_load(entry *pool, int32_t *cnt, int64_t n, int32_t K, const int32_t *ids,
                       const float *dists, const uint8_t *flags)
{
    for (int64_t i = 0; i < n; ++i) {
        int32_t c = 0;
        for (int32_t s = 0; s < K; ++s)
            if (ids[i * K + s] >= 0) {
                entry *e = &pool[i * K + c++];
                e->id = ids[i * K + s];
                e->dist = dists[i * K + s];
                e->is_new = flags[i * K + s];
            }
        cnt[i] = c;
    }
}

static void pools_store(const entry *pool, const int32_t *cnt, int64_t n, int32_t K, int32_t *ids,
                        float *dists, uint8_t *flags)
{
    for (int64_t i = 0; i < n; ++i)
        for (int32_t s = 0; s < K; ++s) {
            int live = s < cnt[i];
            ids[i * K + s] = live ? pool[i * K + s].id : -1;
            dists[i * K + s] = live ? pool[i * K + s].dist : INFINITY;
            flags[i * K + s] = live ? pool[i * K + s].is_new : 0;
        }
}

/* ------------------------------------------------------------------------- */
/* Alg. 3, conquer step: for each point, the candidates are the other members   */
/* of its leaf in every tree and, above the conquer-to depth, the members of    */
/* one leaf of every sibling subtree on the way up; keep the K closest.         */

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Alg. 3, the walk up from the leaf: N is the ancestor of point i's leaf at
 * depth d, Sib the child of N that is not on i's path; i is sent down the
 * subtree of Sib by the split test of every node it meets (Section 3.3.1: the
 * subtree is used as a classifier for i) and the members of the leaf it reaches
 * join the candidates.  `up` is the link of the node below N on i's path.
 * A node without a split dimension (below depth 60) sends every point left. */
static int32_t sibling_leaf(const float *xi, int32_t d, const oracle_node *nodes, int32_t up)
{
    int32_t c = nodes[up >> 1].child[1 - (up & 1)];
    while (c >= 0) {
        const oracle_node *nd = &nodes[c];
        int left = nd->dim == -1 || (int64_t)nd->cnt * node_value(xi, d, nd->dim) < nd->sum;
        c = nd->child[left ? 0 : 1];
    }
    return ~c;
}

/* rows == NULL: all points, output row r belongs to point r.  Otherwise output
 * row r belongs to point rows[r].  Outputs are [n_rows][K].
 * nodes / leaf_up == NULL or dep above every leaf's depth: the conquer step
 * stops at the leaves.  Otherwise, per tree, for d = depth(leaf) - 1 down to
 * dep the leaf that i reaches in the sibling subtree of its ancestor at depth d
 * is added (Alg. 3, the while loop). */
int oracle_conquer_graph(const float *X, int64_t n, int32_t d, const int32_t *perm,
                         const int32_t *leaf_off, const int32_t *n_leaves,
                         const oracle_node *nodes, const int32_t *leaf_up, int32_t dep, int32_t T,
                         int32_t K, const int64_t *rows, int64_t n_rows, int32_t *ids,
                         float *dists, uint8_t *flags)
{
    if (!X || !perm || !leaf_off || !n_leaves || n < 1 || K < 1 || T < 1) return -1;
    if ((!nodes) != (!leaf_up)) return -1;
    if (!rows) n_rows = n;
    /* leaf_of[t][i] = index of the leaf of tree t that holds point i */
    int32_t *leaf_of = (int32_t *)malloc((size_t)T * n * sizeof(int32_t));
    if (!leaf_of) return -4;
    int32_t max_leaf = 0;
    for (int32_t t = 0; t < T; ++t) {
        const int32_t *off = leaf_off + (int64_t)t * (n + 1);
        for (int32_t l = 0; l < n_leaves[t]; ++l) {
            if (off[l + 1] - off[l] > max_leaf) max_leaf = off[l + 1] - off[l];
            for (int32_t p = off[l]; p < off[l + 1]; ++p)
                leaf_of[(int64_t)t * n + perm[(int64_t)t * n + p]] = l;
        }
    }
#pragma omp parallel
    {
        int64_t cap = 1024, nc;
        int32_t *cand = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
        entry *pool = (entry *)malloc((size_t)K * sizeof(entry));
#pragma omp for schedule(dynamic, 256)
        for (int64_t r = 0; r < n_rows; ++r) {
            int64_t i = rows ? rows[r] : r;
            nc = 0;
            for (int32_t t = 0; t < T; ++t) {
                const int32_t *off = leaf_off + (int64_t)t * (n + 1);
                const oracle_node *nd = nodes ? nodes + (int64_t)t * (n + 1) : NULL;
                int32_t l = leaf_of[(int64_t)t * n + i];
                int32_t up = nodes ? leaf_up[(int64_t)t * (n + 1) + l] : -1;
                for (;;) { /* the point's own leaf, then one leaf per ancestor */
                    if (nc + max_leaf > cap) {
                        cap = 2 * cap + max_leaf;
                        cand = (int32_t *)realloc(cand, (size_t)cap * sizeof(int32_t));
                    }
                    for (int32_t p = off[l]; p < off[l + 1]; ++p) {
                        int32_t j = perm[(int64_t)t * n + p];
                        if (j != i) cand[nc++] = j;
                    }
                    if (up < 0 || nd[up >> 1].depth < dep) break;
                    l = sibling_leaf(X + i * d, d, nd, up);
                    int32_t j = up >> 1, pj = nd[j].parent;
                    up = pj < 0 ? -1 : pj * 2 + (nd[pj].child[1] == j);
                }
            }
            qsort(cand, (size_t)nc, sizeof(int32_t), cmp_i32);
            int32_t cnt = 0;
            for (int64_t c = 0; c < nc; ++c) {
                if (c > 0 && cand[c] == cand[c - 1]) continue;
                int32_t j = cand[c];
                pool_insert(pool, &cnt, K, oracle_dist(X + i * d, X + (int64_t)j * d, d), j);
            }
            for (int32_t s = 0; s < K; ++s) {
                ids[r * K + s] = s < cnt ? pool[s].id : -1;
                dists[r * K + s] = s < cnt ? pool[s].dist : INFINITY;
                flags[r * K + s] = s < cnt ? 1 : 0; /* Alg. 4: G_new = G_init */
            }
        }
        free(cand);
        free(pool);
    }
    free(leaf_of);
    return 0;
}

int oracle_init_graph(const float *X, int64_t n, int32_t d, const int32_t *perm,
                      const int32_t *leaf_off, const int32_t *n_leaves, int32_t T, int32_t K,
                      const int64_t *rows, int64_t n_rows, int32_t *ids, float *dists,
                      uint8_t *flags)
{
    return oracle_conquer_graph(X, n, d, perm, leaf_off, n_leaves, NULL, NULL, 0, T, K, rows,
                                n_rows, ids, dists, flags);
}

/* ------------------------------------------------------------------------- */
/* Alg. 4: NN-descent refinement                                               */

typedef struct { uint32_t hash; int32_t id; } rcand;

static int cmp_rcand(const void *a, const void *b)
{
    const rcand *x = (const rcand *)a, *y = (const rcand *)b;
    if (x->hash != y->hash) return (x->hash > y->hash) - (x->hash < y->hash);
    return (x->id > y->id) - (x->id < y->id);
}

/* rev[v] = the (at most L) sources u with v in fwd[u] that have the smallest
 * (hash(seed, iter, v, u), u). */
static void reverse_lists(const int32_t *fwd, const int32_t *fwd_cnt, int32_t fwd_stride, int64_t n,
                          int32_t L, uint64_t seed, int32_t iter, int32_t *rev, int32_t *rev_cnt)
{
    int64_t *start = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    for (int64_t u = 0; u < n; ++u)
        for (int32_t s = 0; s < fwd_cnt[u]; ++s) start[fwd[u * fwd_stride + s] + 1]++;
    for (int64_t v = 0; v < n; ++v) start[v + 1] += start[v];
    rcand *all = (rcand *)malloc((size_t)(start[n] > 0 ? start[n] : 1) * sizeof(rcand));
    int64_t *fill = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    memcpy(fill, start, (size_t)n * sizeof(int64_t));
    for (int64_t u = 0; u < n; ++u)
        for (int32_t s = 0; s < fwd_cnt[u]; ++s) {
            int32_t v = fwd[u * fwd_stride + s];
            rcand *c = &all[fill[v]++];
            c->id = (int32_t)u;
            c->hash = oracle_reverse_hash(seed, iter, v, (int32_t)u);
        }
    for (int64_t v = 0; v < n; ++v) {
        int64_t m = start[v + 1] - start[v];
        qsort(all + start[v], (size_t)m, sizeof(rcand), cmp_rcand);
        int32_t keep = m < L ? (int32_t)m : L;
        for (int32_t s = 0; s < keep; ++s) rev[v * L + s] = all[start[v] + s].id;
        rev_cnt[v] = keep;
    }
    free(fill);
    free(all);
    free(start);
}

static int32_t sorted_union(const int32_t *a, int32_t na, const int32_t *b, int32_t nb, int32_t *out)
{
    int32_t m = 0;
    for (int32_t s = 0; s < na; ++s) out[m++] = a[s];
    for (int32_t s = 0; s < nb; ++s) out[m++] = b[s];
    qsort(out, (size_t)m, sizeof(int32_t), cmp_i32);
    int32_t u = 0;
    for (int32_t s = 0; s < m; ++s)
        if (s == 0 || out[s] != out[s - 1]) out[u++] = out[s];
    return u;
}

/* ids/dists/flags: [n][K] pools, in and out (sorted by (dist,id), empties last).
 * iter0: index of the first iteration (a resumed run passes the number already
 * done).  stats: [iters][2] = {distance evaluations, accepted insertions}; the
 * second figure counts insertions that may be evicted again within the same
 * iteration, so unlike the pools it depends on the order of evaluation. */
/* delta > 0: early termination (Section 1 names it among the techniques taken over from
 * NN-descent; Alg. 4 itself only has the iteration limit): stop after an iteration that
 * leaves fewer than delta*n*K entries carrying the new mark, i.e. fresh entries that were
 * still in their pool when the iteration ended.  iters_done (may be NULL) receives the
 * number of iterations carried out. */
/* cross_old != 0: the literal marking of Alg. 4's second inner loop (an entry that a pair of a
 * new and an old member inserts is marked old, one that a pair of two new members inserts is
 * marked new).  Which of the two an entry gets when both kinds of pair offer it in the same
 * iteration depends on the order of insertion in the listing; here the pairs of two new members
 * of all joins are inserted first, then the others, so that the new mark wins. */
int oracle_nndescent_opts(const float *X, int64_t n, int32_t d, int32_t K, int32_t *ids,
                          float *dists, uint8_t *flags, int32_t iters, int32_t L, uint64_t seed,
                          int32_t iter0, uint64_t *stats, double delta, int32_t *iters_done,
                          int32_t cross_old);

int oracle_nndescent_until(const float *X, int64_t n, int32_t d, int32_t K, int32_t *ids,
                           float *dists, uint8_t *flags, int32_t iters, int32_t L, uint64_t seed,
                           int32_t iter0, uint64_t *stats, double delta, int32_t *iters_done)
{
    return oracle_nndescent_opts(X, n, d, K, ids, dists, flags, iters, L, seed, iter0, stats, delta,
                                 iters_done, 0);
}

int oracle_nndescent_opts(const float *X, int64_t n, int32_t d, int32_t K, int32_t *ids,
                          float *dists, uint8_t *flags, int32_t iters, int32_t L, uint64_t seed,
                          int32_t iter0, uint64_t *stats, double delta, int32_t *iters_done,
                          int32_t cross_old)
{
    if (!X || !ids || !dists || !flags || n < 2 || K < 1 || L < 1 || iters < 0) return -1;
    if (iters_done) *iters_done = 0;
    entry *pool = (entry *)malloc((size_t)n * K * sizeof(entry));
    int32_t *cnt = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *nw = (int32_t *)malloc((size_t)n * L * sizeof(int32_t));
    int32_t *od = (int32_t *)malloc((size_t)n * K * sizeof(int32_t));
    int32_t *rnw = (int32_t *)malloc((size_t)n * L * sizeof(int32_t));
    int32_t *rod = (int32_t *)malloc((size_t)n * L * sizeof(int32_t));
    int32_t *nw_c = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *od_c = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *rnw_c = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *rod_c = (int32_t *)malloc((size_t)n * sizeof(int32_t));
#ifdef _OPENMP
    omp_lock_t *lock = (omp_lock_t *)malloc((size_t)n * sizeof(omp_lock_t));
    for (int64_t i = 0; i < n; ++i) omp_init_lock(&lock[i]);
#endif
    pools_load(pool, cnt, n, K, ids, dists, flags);

    for (int32_t it = 0; it < iters; ++it) {
        /* sample: walk each pool in ascending order; the first L new-flagged
         * entries become the "new" set (and lose their flag), old-flagged
         * entries met on the way become the "old" set. */
        for (int64_t i = 0; i < n; ++i) {
            int32_t a = 0, b = 0;
            for (int32_t s = 0; s < cnt[i] && a < L; ++s) {
                entry *e = &pool[i * K + s];
                if (e->is_new) {
                    nw[i * L + a++] = e->id;
                    e->is_new = 0;
                } else {
                    od[i * K + b++] = e->id;
                }
            }
            nw_c[i] = a;
            od_c[i] = b;
        }
        reverse_lists(nw, nw_c, L, n, L, seed, 2 * (iter0 + it), rnw, rnw_c);
        reverse_lists(od, od_c, K, n, L, seed, 2 * (iter0 + it) + 1, rod, rod_c);

        /* local join: every unordered pair inside U_new and every pair of
         * U_new x U_old is evaluated once and proposed to both end points. */
        uint64_t evals = 0, updates = 0;
        /* one pass over all joins, or (cross_old) two: pairs inside U_new, then U_new x U_old */
        for (int32_t pass = 0; pass < (cross_old ? 2 : 1); ++pass)
#pragma omp parallel reduction(+ : evals, updates)
        {
            int32_t *un = (int32_t *)malloc((size_t)2 * L * sizeof(int32_t));
            int32_t *uo = (int32_t *)malloc((size_t)(K + L) * sizeof(int32_t));
#pragma omp for schedule(dynamic, 64)
            for (int64_t i = 0; i < n; ++i) {
                int32_t n_new = sorted_union(nw + i * L, nw_c[i], rnw + i * L, rnw_c[i], un);
                int32_t n_all = sorted_union(od + i * K, od_c[i], rod + i * L, rod_c[i], uo);
                int32_t n_old = 0;
                for (int32_t s = 0; s < n_all; ++s) /* U_old \ U_new */
                    if (!bsearch(&uo[s], un, (size_t)n_new, sizeof(int32_t), cmp_i32))
                        uo[n_old++] = uo[s];
                for (int32_t a = 0; a < n_new; ++a) {
                    int32_t u = un[a];
                    int32_t b_lo = cross_old && pass == 1 ? n_new : a + 1;
                    int32_t b_hi = cross_old && pass == 0 ? n_new : n_new + n_old;
                    uint8_t mark = !(cross_old && pass == 1);
                    for (int32_t b = b_lo; b < b_hi; ++b) {
                        int32_t v = b < n_new ? un[b] : uo[b - n_new];
                        float dist = oracle_dist(X + (int64_t)u * d, X + (int64_t)v * d, d);
                        ++evals;
#ifdef _OPENMP
                        omp_set_lock(&lock[u]);
#endif
                        updates += pool_insert_marked(pool + (int64_t)u * K, &cnt[u], K, dist, v, mark);
#ifdef _OPENMP
                        omp_unset_lock(&lock[u]);
                        omp_set_lock(&lock[v]);
#endif
                        updates += pool_insert_marked(pool + (int64_t)v * K, &cnt[v], K, dist, u, mark);
#ifdef _OPENMP
                        omp_unset_lock(&lock[v]);
#endif
                    }
                }
            }
            free(un);
            free(uo);
        }
        if (stats) {
            stats[2 * it] = evals;
            stats[2 * it + 1] = updates;
        }
        if (iters_done) *iters_done = it + 1;
        if (delta > 0.0) {
            int64_t fresh = 0;
            for (int64_t i = 0; i < n; ++i)
                for (int32_t c = 0; c < cnt[i]; ++c) fresh += pool[i * K + c].is_new;
            if ((double)fresh < delta * (double)n * (double)K) break;
        }
    }
    pools_store(pool, cnt, n, K, ids, dists, flags);
#ifdef _OPENMP
    for (int64_t i = 0; i < n; ++i) omp_destroy_lock(&lock[i]);
    free(lock);
#endif
    free(rod_c); free(rnw_c); free(od_c); free(nw_c);
    free(rod); free(rnw); free(od); free(nw);
    free(cnt); free(pool);
    return 0;
}

int oracle_nndescent(const float *X, int64_t n, int32_t d, int32_t K, int32_t *ids, float *dists,
                     uint8_t *flags, int32_t iters, int32_t L, uint64_t seed, int32_t iter0,
                     uint64_t *stats)
{
    return oracle_nndescent_until(X, n, d, K, ids, dists, flags, iters, L, seed, iter0, stats, 0.0,
                                  NULL);
}

/* ------------------------------------------------------------------------- */
/* Alg. 1: search with the index (trees for the first candidates, the graph for  */
/* NN-expansion).                                                               */

typedef struct { double prio; int32_t link; } branch;

/* Alg. 1, "search tree i for the top N_node closest leaf nodes according to the
 * tree's search criteria": best-bin-first search as in randomized KD-trees.  Going
 * down, the child on the query's side of the split is taken (the test that built
 * the tree: left iff cnt*q(x) < sum) and the other child is put aside with the
 * priority of the branch being followed plus the squared distance from the query's
 * coordinate to the split value (the node's mean, sum / cnt, in coordinate units:
 * 2^-20 of the quantised ones); after a leaf the branch with the smallest
 * (priority, link) put aside so far is followed.  A node without a dimension sends
 * the query left and puts the right child aside at the same priority.  Returns the
 * number of leaves written to `leaves` (at most want). */
static int32_t tree_search(const float *q, int32_t d, const oracle_node *nodes, int32_t n_leaves, int32_t want,
                           int32_t *leaves, branch *heap, int32_t heap_cap)
{
    if (n_leaves == 1) {
        leaves[0] = 0;
        return want > 0 ? 1 : 0;
    }
    /* the root is the node without a parent */
    int32_t root = -1;
    for (int32_t j = 1; j < n_leaves; ++j)
        if (nodes[j].parent < 0) root = j;
    int32_t n_heap = 0, found = 0;
    int32_t link = root;
    double prio = 0.0;
    while (found < want) {
        while (link >= 0) { /* down to a leaf */
            const oracle_node *nd = &nodes[link];
            int left = 1;
            double other = prio;
            if (nd->dim != -1) {
                int64_t diff = (int64_t)nd->cnt * node_value(q, d, nd->dim) - nd->sum;
                left = diff < 0;
                double gap = (double)diff / ((double)nd->cnt * 1048576.0);
                other = fma(gap, gap, prio); /* (along a projection: in units of its length, the same for every node) */
            }
            if (n_heap == heap_cap) return -1; /* cannot happen with the caller's capacity */
            heap[n_heap].prio = other;
            heap[n_heap].link = nd->child[left ? 1 : 0];
            ++n_heap;
            link = nd->child[left ? 0 : 1];
        }
        leaves[found++] = ~link;
        if (n_heap == 0) break;
        int32_t best = 0;
        for (int32_t h = 1; h < n_heap; ++h)
            if (heap[h].prio < heap[best].prio ||
                (heap[h].prio == heap[best].prio && heap[h].link < heap[best].link))
                best = h;
        prio = heap[best].prio;
        link = heap[best].link;
        heap[best] = heap[--n_heap];
    }
    return found;
}

/* queries: [nq][d].  graph_ids: [n][Kg] neighbour ids (-1 = empty slot).  K <= P.
 * Alg. 1 with N_node = P / S / T + 1 leaves per tree (integer divisions), the E
 * closest points of those leaves as the first pool, then `iters` rounds in which
 * every pool member that has not been expanded yet contributes its graph
 * neighbours that have not been checked yet, and the pool keeps the P closest.
 * Ties by id.  out_ids / out_dists: [nq][K], padded with -1 / +inf.
 * n_checked (may be NULL): [nq] distances evaluated per query. */
int oracle_search(const float *X, int64_t n, int32_t d, const int32_t *perm,
                  const int32_t *leaf_off, const int32_t *n_leaves, const oracle_node *nodes,
                  int32_t T, int32_t S, const int32_t *graph_ids, int32_t Kg, const float *queries,
                  int64_t nq, int32_t K, int32_t P, int32_t E, int32_t iters, int32_t *out_ids,
                  float *out_dists, int32_t *n_checked)
{
    if (!X || !perm || !leaf_off || !n_leaves || !nodes || !graph_ids || !queries) return -1;
    if (n < 1 || T < 1 || S < 1 || K < 1 || P < K || E < 1 || E > P || iters < 0 || Kg < 1) return -1;
    const int32_t want = P / S / T + 1;
    int failed = 0;
#pragma omp parallel
    {
        uint8_t *checked = (uint8_t *)calloc((size_t)n, 1);
        entry *pool = (entry *)malloc((size_t)P * sizeof(entry));
        int32_t *expand = (int32_t *)malloc((size_t)P * sizeof(int32_t));
        int32_t *touched = (int32_t *)malloc((size_t)n * sizeof(int32_t));
        int32_t *leaves = (int32_t *)malloc((size_t)want * sizeof(int32_t));
        /* a descent puts aside one branch per level; trees are at most 60 + log2(n) deep */
        const int32_t heap_cap = (want + 1) * 128;
        branch *heap = (branch *)malloc((size_t)heap_cap * sizeof(branch));
#pragma omp for schedule(dynamic, 16)
        for (int64_t qi = 0; qi < nq; ++qi) {
            const float *q = queries + qi * d;
            int32_t cnt = 0, n_touched = 0, cap = E;
            for (int32_t t = 0; t < T; ++t) {
                const int32_t *off = leaf_off + (int64_t)t * (n + 1);
                int32_t found = tree_search(q, d, nodes + (int64_t)t * (n + 1), n_leaves[t], want, leaves,
                                            heap, heap_cap);
                if (found < 0) {
#pragma omp atomic write
                    failed = 1;
                    found = 0;
                }
                for (int32_t f = 0; f < found; ++f)
                    for (int32_t p = off[leaves[f]]; p < off[leaves[f] + 1]; ++p) {
                        int32_t j = perm[(int64_t)t * n + p];
                        if (checked[j]) continue;
                        checked[j] = 1;
                        touched[n_touched++] = j;
                        pool_insert(pool, &cnt, cap, oracle_dist(q, X + (int64_t)j * d, d), j);
                    }
            }
            /* pool_insert marks what it takes as new: here "not expanded yet" */
            cap = P;
            for (int32_t it = 0; it < iters; ++it) {
                int32_t n_exp = 0;
                for (int32_t s = 0; s < cnt; ++s)
                    if (pool[s].is_new) {
                        pool[s].is_new = 0;
                        expand[n_exp++] = pool[s].id;
                    }
                for (int32_t e = 0; e < n_exp; ++e)
                    for (int32_t c = 0; c < Kg; ++c) {
                        int32_t j = graph_ids[(int64_t)expand[e] * Kg + c];
                        if (j < 0 || checked[j]) continue;
                        checked[j] = 1;
                        touched[n_touched++] = j;
                        pool_insert(pool, &cnt, cap, oracle_dist(q, X + (int64_t)j * d, d), j);
                    }
            }
            for (int32_t s = 0; s < K; ++s) {
                out_ids[qi * K + s] = s < cnt ? pool[s].id : -1;
                out_dists[qi * K + s] = s < cnt ? pool[s].dist : INFINITY;
            }
            if (n_checked) n_checked[qi] = n_touched;
            for (int32_t s = 0; s < n_touched; ++s) checked[touched[s]] = 0;
        }
        free(checked); free(pool); free(expand); free(touched); free(leaves); free(heap);
    }
    return failed ? -6 : 0;
}

void oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
