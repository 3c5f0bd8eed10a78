/*
 * efanna.h - C ABI of the gfx950 (MI355X) kNN-graph construction library.
 *
 * The library builds an approximate K-nearest-neighbour graph over N float32 vectors
 * of dimension d under squared L2 distance, following the offline index-building
 * path of EFANNA (arXiv 1609.07228, Section 3.3): randomized truncated KD-trees
 * (Alg. 2) divide the points, a brute-force pass inside every leaf and, optionally,
 * against one leaf of every sibling subtree up to a chosen depth gives each point its
 * initial neighbours (Alg. 3), and NN-descent local joins refine the graph (Alg. 4).
 *
 * Conventions shared by every entry point
 *  - Pointers marked [device] are device (HBM) addresses owned by the caller; the
 *    library neither allocates nor frees device memory.  Temporary storage comes from
 *    a caller-provided workspace (`ws`, `ws_bytes`, 256-byte aligned); its required
 *    size is returned by the matching *_workspace_bytes function.  Workspace contents
 *    need not survive between calls.  (efanna_nndescent_noalloc uses a fixed device
 *    array of the library's own instead.)
 *  - Host-side resources: efanna_build_trees keeps one small pinned host buffer per
 *    calling thread (hipHostMalloc, 32 bytes, never freed) to read its level counters
 *    into; efanna_nndescent creates and destroys 5 * iters HIP events when phase_ms is
 *    given.  Nothing else is allocated on either side.
 *  - Pointers marked [host] are ordinary host addresses.
 *  - `stream` is a hipStream_t (NULL = the default stream).  Work is enqueued on it;
 *    entry points documented as synchronising wait for that stream before returning.
 *  - Return value: EFANNA_OK or a negative efanna_status.  Argument errors are
 *    detected on the host before anything is launched.
 *  - Distances are SQUARED Euclidean distances evaluated in float32 with a fixed
 *    order of operations: partial sum l (0..15) accumulates, by fused multiply-add
 *    and in ascending j, the squares of the differences of coordinates j = l mod 16;
 *    the sixteen partial sums are then added as l += l+8, l += l+4, l += l+2,
 *    l += l+1.  The value is symmetric in its arguments and is the one stored,
 *    compared and returned everywhere.  Lists are ordered by (distance, id).
 *  - Results are a deterministic function of the inputs and the seed: concurrent
 *    list updates are set operations (a list ends up holding the K smallest
 *    (distance, id) keys ever proposed to it), so scheduling cannot change them.
 *  - Calls that use the same graph, workspace or stream concurrently race; calls on
 *    distinct buffers and streams are independent.  Apart from the resources named above
 *    the library keeps no state between calls.
 */
#ifndef EFANNA_H
#define EFANNA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EFANNA_OK = 0,
    EFANNA_EINVAL = -1,     /* null pointer or parameter out of range                 */
    EFANNA_EWORKSPACE = -2, /* workspace missing, misaligned or too small             */
    EFANNA_EINPUT = -3,     /* X holds a non-finite value, |x| >= 2^20 or n*|x| >= 2^43 */
    EFANNA_EHIP = -4,       /* a HIP runtime call failed                              */
    EFANNA_ECAPACITY = -5,  /* a tree has more leaves than `max_leaves`               */
    EFANNA_EUNSUPPORTED = -6, /* shape outside what the kernels handle (see each call) */
    EFANNA_ESCRATCH = -7     /* efanna_nndescent_noalloc: the input needs more scratch memory
                                than EFANNA_NOALLOC_SCRATCH_BYTES                       */
} efanna_status;

/* Limits of this build (checked, EFANNA_EUNSUPPORTED / EFANNA_EINVAL beyond them). */
#define EFANNA_MAX_K 128        /* graph degree                                        */
#define EFANNA_MAX_SAMPLE 64    /* NN-descent sample size L                            */
#define EFANNA_MAX_LEAF 64      /* leaf population S                                   */
#define EFANNA_MAX_TREES 64
/* size of the fixed device array behind efanna_nndescent_noalloc (64 MiB per GPU in use) */
#define EFANNA_NOALLOC_SCRATCH_BYTES (64u << 20)

/* A graph entry: bits 63..32 float32 bit pattern of the squared distance, bits 31..1
 * neighbour id, bit 0 the "new" mark of Alg. 4.  An empty slot has distance +inf.
 * Rows of `graph` are K such entries in no particular order. */
typedef uint64_t efanna_entry;

/* An internal tree node as the conquer step of Alg. 3 uses it.  A point x goes to the left
 * child iff cnt * q(x[dim]) < sum, q(x) = x * 2^20 rounded to the nearest integer (ties to
 * even), which is the test the node's own points were divided by; dim -1 (nodes below depth
 * 60, which are cut by position) sends every point left; dim <= -3 names a random projection
 * that takes the place of q(x[dim]) (EFANNA_SPLIT_PROJECTION below).  The internal nodes of a tree are
 * numbered 1 .. n_leaves-1: node j is the one whose right part starts with leaf j.
 * child[s] >= 0 names an internal node, child[s] < 0 is ~(leaf index); parent is -1 at the
 * root; depth counts from 0 at the root. */
typedef struct {
    int64_t sum;
    int32_t dim, cnt, parent, depth;
    int32_t child[2];
} efanna_node;

const char *efanna_status_string(int status);

/* ---- Alg. 2: randomized truncated KD-trees ------------------------------------------
 * For each of n_trees trees the n point ids are partitioned recursively: a node with
 * more than leaf_size points draws a dimension uniformly (counter-based generator
 * keyed by seed, tree index and the node's heap id: root 1, children 2h and 2h+1),
 * and sends to the left the points whose coordinate is below the node's mean, keeping
 * the relative order of ids on both sides.  The mean test is exact: coordinates are
 * quantised to multiples of 2^-20 and compared as cnt*q(x) < sum(q).  If one side
 * would be empty (or below depth 60) the node is cut into positional halves.
 *
 * X        [device] n*d float32, row-major, finite, |x| < 2^20 and n * |x| < 2^43 (the latter
 *          only binds beyond 2^23 points: it keeps cnt*q(x) and the sums inside 64 bits);
 *          EFANNA_EINPUT otherwise.
 * perm     [device] out, n_trees*n int32: ids of tree t at perm[t*n ..], every leaf a
 *          contiguous run, leaves in left-to-right order, ids ascending inside a leaf.
 * leaf_off [device] out, n_trees*(max_leaves+1) int32: start of each leaf of tree t
 *          within perm[t*n ..], followed by n.
 * n_leaves [host]   out, n_trees int32.
 * max_leaves        capacity of leaf_off per tree (n always suffices).
 * nodes    [device] out or NULL, n_trees*(max_leaves+1) efanna_node: the internal nodes of
 *          tree t at nodes[t*(max_leaves+1) + j], j = 1 .. n_leaves[t]-1 (entry 0 unused).
 * leaf_up  [device] out or NULL (both or neither), n_trees*(max_leaves+1) int32: for leaf l of
 *          tree t, 2 * (its parent node) + (1 if it is the right child); -1 if the tree is a
 *          single leaf.  With nodes the workspace must be sized with with_nodes = 1.
 * tree_depth [host] out or NULL: depth of the deepest internal node over all trees (root 0),
 *          -1 if every tree is a single leaf or nodes is NULL.
 * Synchronises the stream (the host drives one launch group per tree level).
 * Limits: n*n_trees < 2^31, 1 <= leaf_size <= EFANNA_MAX_LEAF, n_trees <= EFANNA_MAX_TREES.
 */
size_t efanna_trees_workspace_bytes(int64_t n, int32_t d, int32_t n_trees, int32_t leaf_size,
                                    int32_t with_nodes);

int efanna_build_trees(const float *X, int64_t n, int32_t d, int32_t n_trees, int32_t leaf_size,
                       uint64_t seed, int32_t *perm, int32_t *leaf_off, int32_t max_leaves,
                       int32_t *n_leaves, efanna_node *nodes, int32_t *leaf_up,
                       int32_t *tree_depth, void *ws, size_t ws_bytes, void *stream);

/* The same with a choice of how a node takes its split dimension (Section 3.2: the trees
 * are the randomized KD-trees of the literature except for the leaf size).
 * split_rule EFANNA_SPLIT_UNIFORM: drawn uniformly over the d dimensions, Alg. 2 as printed
 *          (what efanna_build_trees does).
 * split_rule EFANNA_SPLIT_VARIANCE: that tree's own rule - among the five dimensions of largest
 *          variance the node's draw picks one.  The variance is estimated on the node's first
 *          100 positions (all of them in a smaller node), exactly: as the integer
 *          m*sum(q^2) - sum(q)^2 of the quantised coordinates, equal values ordered by the
 *          smaller dimension; with d < 5 all dimensions are candidates, in that order.
 * split_rule EFANNA_SPLIT_PROJECTION: a node splits on a random projection instead of a coordinate
 *          (the trees the paper's closing section proposes to try for high dimensions): the sum
 *          of eight quantised coordinates with signs, both drawn from a 30-bit number r taken
 *          from the node's draw (bits 34..63) - term k uses z = mix(256 r + k + golden),
 *          coordinate z mod d, minus if the top bit of z is set.  The mean test is the same,
 *          cnt*p(x) < sum(p), exact for n * 8 * |x| < 2^43 (EFANNA_EINPUT otherwise).  Such a
 *          node's efanna_node.dim is -3 - r; efanna_init_graph and efanna_search route through
 *          these nodes like through any other.
 * Any other value: EFANNA_EINVAL.  Everything else as efanna_build_trees. */
#define EFANNA_SPLIT_UNIFORM 0
#define EFANNA_SPLIT_VARIANCE 1
#define EFANNA_SPLIT_PROJECTION 2
int efanna_build_trees_rule(const float *X, int64_t n, int32_t d, int32_t n_trees, int32_t leaf_size,
                            uint64_t seed, int32_t split_rule, int32_t *perm, int32_t *leaf_off,
                            int32_t max_leaves, int32_t *n_leaves, efanna_node *nodes,
                            int32_t *leaf_up, int32_t *tree_depth, void *ws, size_t ws_bytes,
                            void *stream);

/* ---- Alg. 3, conquer step ---------------------------------------------------------------
 * Candidates of point i: in every tree, the other members of its leaf and - when nodes is
 * given - for every ancestor N of that leaf with depth >= conquer_depth, the members of the
 * leaf that i reaches when it is sent down the subtree of N's other child by the nodes' split
 * tests (Section 3.3.1: the sibling subtree classifies i).  Graph row i ends up holding the K
 * closest distinct candidates (fewer if there are fewer; the rest of the row is empty).
 * Every entry carries the "new" mark (Alg. 4 starts from G_new = G_init).
 *
 * perm, leaf_off, max_leaves, n_leaves, nodes, leaf_up: as produced by efanna_build_trees.
 * nodes, leaf_up NULL: the step stops at the leaves (tree_depth, conquer_depth are ignored).
 * tree_depth       as returned by efanna_build_trees (a larger value only costs workspace).
 * conquer_depth    >= 0; 0 walks up to the root.  levels = tree_depth - conquer_depth + 1 is
 *                  the number of ancestors a leaf can have in range; the workspace holds one
 *                  int32 per point and level (efanna_init_workspace_bytes(n, levels); levels
 *                  <= 0 or no nodes: 256 bytes).
 * graph    [device] out, n*k entries.
 * Asynchronous on `stream`.  Limits: k <= EFANNA_MAX_K, k < n, n < 2^31 - 256, a leaf
 * of leaf_size rows of d floats must fit the 160 KB LDS; with nodes: levels <= 64
 * (EFANNA_EUNSUPPORTED otherwise).  Leaves of at most 16 points with d a multiple of 4 and a
 * 16-byte aligned X take the fast kernels, every other shape general ones.
 */
size_t efanna_init_workspace_bytes(int64_t n, int32_t levels);

int efanna_init_graph(const float *X, int64_t n, int32_t d, const int32_t *perm,
                      const int32_t *leaf_off, int32_t max_leaves, const int32_t *n_leaves,
                      const efanna_node *nodes, const int32_t *leaf_up, int32_t tree_depth,
                      int32_t conquer_depth, int32_t n_trees, int32_t leaf_size, int32_t k, efanna_entry *graph,
                      void *ws, size_t ws_bytes, void *stream);

/* ---- Alg. 4: NN-descent refinement -----------------------------------------------------
 * Runs `iters` iterations with pool size P = k.  One iteration: (1) in every row the
 * sample_L closest entries carrying the new mark form the row's "new" set and lose the
 * mark, unmarked entries closer than the last of them form its "old" set; (2) reverse
 * lists are the transposes of those sets, each capped at sample_L members by keeping
 * the smallest seeded hash of (iteration, target, source); (3) for every point the
 * union of its new and reverse-new sets is joined with itself and with the union of
 * its old and reverse-old sets: each unordered pair is evaluated once and proposed to
 * both end points; (4) a row keeps the k smallest (distance, id) among its entries and
 * the proposals, an id already present keeping its entry and mark, fresh entries marked
 * new.
 *
 * delta    0: run all `iters` iterations.  > 0: early termination - stop after an iteration
 *          that leaves fewer than delta*n*k entries carrying the new mark (fresh entries that
 *          were still in their row when the iteration ended); the call then synchronises the
 *          stream after every iteration.
 * cross_old 0: every fresh entry is marked new.  1: the literal marking of Alg. 4's second inner
 *          loop - an entry inserted by a pair of a new and an old member of a join is marked old
 *          (it will not be sampled as new), one inserted by a pair of two new members is marked
 *          new.  To make the outcome independent of scheduling the joins then run twice per
 *          iteration: all pairs of two new members first, so that an entry offered by both kinds
 *          of pair is new.  Fewer joins later, lower accuracy: an ablation, not the default.
 * iters_done [host] out or NULL: iterations carried out.
 * graph    [device] in/out.  The call may be repeated to continue refining: pass the
 *          number of iterations already done as first_iter so that the hash stream
 *          continues (k calls of one iteration equal one call of k iterations).
 * stats    [device] out or NULL: iters*4 uint64 per iteration: {distance evaluations,
 *          accepted list insertions, vectors gathered by all joins, vectors gathered by
 *          the joins of at most 16 vectors}.  All but the second are deterministic; the
 *          second counts insertions that may be displaced later in the same iteration.
 * phase_ms [host] out or NULL: iters*4 float: milliseconds of {sampling + reverse lists
 *          + join lists, joins of at most 16 vectors, joins of 17..32 vectors, larger
 *          joins} per iteration, from HIP events on `stream`.  When given, the call
 *          synchronises the stream before returning.  (With cross_old the split by join size
 *          covers the second pass only; the first pass is booked under the smallest joins.)
 * Asynchronous on `stream` otherwise.  Limits: k <= EFANNA_MAX_K, sample_L <= EFANNA_MAX_SAMPLE,
 * where joins can gather more than 32 vectors (k + 2*sample_L > 32) of more than 128
 * coordinates, or d is not a multiple of 4, or X is not 16-byte aligned, k + 2*sample_L rows of
 * d floats must fit the 160 KB LDS (EFANNA_EUNSUPPORTED otherwise).
 */
size_t efanna_nndescent_workspace_bytes(int64_t n, int32_t k, int32_t sample_L);

int efanna_nndescent(const float *X, int64_t n, int32_t d, int32_t k, efanna_entry *graph,
                     int32_t iters, int32_t sample_L, uint64_t seed, int32_t first_iter,
                     float delta, int32_t cross_old, int32_t *iters_done,
                     uint64_t *stats, float *phase_ms, void *ws, size_t ws_bytes, void *stream);

/* The same refinement for callers that cannot allocate device memory and have no workspace
 * to hand in: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Everything efanna_nndescent keeps in its workspace lives in a fixed array of
 * EFANNA_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the
 * library runs on holds its own copy until the process ends); the call allocates and frees
 * nothing, on the device or through the HIP runtime, and creates no events.  Arguments as
 * for efanna_nndescent, without early termination and phase timing; the result is the same,
 * bit for bit.  Returns EFANNA_ESCRATCH when efanna_nndescent_workspace_bytes(n, k, sample_L)
 * exceeds EFANNA_NOALLOC_SCRATCH_BYTES (64 MiB: about 140 000 points at k = sample_L = 10).
 * All calls on one GPU share that GPU's array (it keeps the last call's contents; the call
 * resets what it needs): calls that overlap on one GPU race, whatever their streams.
 * Asynchronous on `stream`. */
int efanna_nndescent_noalloc(const float *X, int64_t n, int32_t d, int32_t k, efanna_entry *graph,
                             int32_t iters, int32_t sample_L, uint64_t seed, int32_t first_iter,
                             uint64_t *stats, void *stream);

/* ---- result ("Ensure: approximate kNN graph G") -------------------------------------
 * Sorts every row by (distance, id) and unpacks it.
 * ids   [device] out, n*k int32, -1 in empty slots (always at the tail).
 * dists [device] out, n*k float32 squared distances, +inf in empty slots.
 * flags [device] out or NULL, n*k uint8: the new marks.
 * Asynchronous on `stream`; does not modify graph.
 */
int efanna_get_graph(const efanna_entry *graph, int64_t n, int32_t k, int32_t *ids, float *dists,
                     uint8_t *flags, void *stream);

/* Inverse of efanna_get_graph: packs (ids, dists, flags) rows into graph entries, so
 * that NN-descent can start from any initial graph (for example a random one).
 * Empty slots are given by id < 0 (ids >= n are treated the same way).  flags NULL marks
 * every entry new.  Asynchronous on `stream`. */
int efanna_set_graph(efanna_entry *graph, int64_t n, int32_t k, const int32_t *ids,
                     const float *dists, const uint8_t *flags, void *stream);

/* Squared distances of m explicit pairs, in the library's fixed order of operations
 * (the definition at the top of this file).  a_ids, b_ids [device] m int32; out
 * [device] m float32.  Asynchronous on `stream`. */
int efanna_pair_distances(const float *X, int64_t n, int32_t d, const int32_t *a_ids,
                          const int32_t *b_ids, int64_t m, float *out, void *stream);

/* ---- Alg. 1: search with the finished index ---------------------------------------------
 * For each of nq queries: every tree is searched, best bin first, for its N_node = pool /
 * leaf_size / n_trees + 1 closest leaves (going down, the child on the query's side of the
 * split is taken and the other put aside with the priority of the branch followed plus the
 * squared distance, in float64, from the query's coordinate to the node's mean sum / cnt;
 * after a leaf the search continues from the smallest (priority, child link) put aside); the
 * `expand` closest members of those leaves form the first pool; then, `iters` times, every
 * pool member that has not been expanded yet hands in its graph neighbours, those never
 * checked before are evaluated, and the pool keeps the `pool` closest.  Ties by id.
 *
 * perm .. nodes, tree_depth: as produced by efanna_build_trees with nodes.
 * graph_ids [device] n*graph_k int32, neighbour ids as efanna_get_graph writes them (-1 = none).
 * queries  [device] nq*d float32, row-major, 16-byte aligned.
 * ids, dists [device] out, nq*k: the k closest pool members, ascending; -1 / +inf padding.
 * checked  [device] out or NULL, nq int32: distances evaluated per query.
 * Synchronises the stream.  Limits: k <= pool <= 1024, 1 <= expand <= pool, d a multiple of 4,
 * X 16-byte aligned (EFANNA_EUNSUPPORTED otherwise).
 */
size_t efanna_search_workspace_bytes(int64_t nq, int32_t d, int32_t n_trees, int32_t leaf_size,
                                     int32_t tree_depth, int32_t graph_k, int32_t pool,
                                     int32_t iters);

int efanna_search(const float *X, int64_t n, int32_t d, const int32_t *perm,
                  const int32_t *leaf_off, int32_t max_leaves, const int32_t *n_leaves,
                  const efanna_node *nodes, int32_t tree_depth, int32_t n_trees, int32_t leaf_size,
                  const int32_t *graph_ids, int32_t graph_k, const float *queries, int64_t nq,
                  int32_t k, int32_t pool, int32_t expand, int32_t iters, int32_t *ids,
                  float *dists, int32_t *checked, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EFANNA_H */
