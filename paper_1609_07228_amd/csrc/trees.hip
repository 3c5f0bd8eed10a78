// Randomized truncated KD-trees (Alg. 2) for gfx950.
//
// All trees are built together, one level per launch group.  The ids of tree t live in
// positions [t*n, (t+1)*n) of one array of T*n "positions"; a node is a segment of
// positions.  Per level:
//   1. sum      every position adds its quantised coordinate (on the node's dimension)
//               to the node's 64-bit integer sum (wave-reduced when a wave lies inside
//               one node, integer atomics otherwise: exact in any order);
//   2. scan     device-wide exclusive prefix sum of the "goes left" predicate
//               cnt*q(x) < sum, from which every position derives its rank inside
//               its node, i.e. a stable partition without any per-node launch;
//   3. children one thread per node fixes the split point, appends the children that
//               still hold more than leaf_size points to the next level's node table
//               and marks the first position of children that became leaves;
//   4. scatter  every position moves its id to its place in the child segment.
// The host reads one counter per level (the number of nodes of the next level).
#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kScanItems = 8;                       // per thread
constexpr int kScanTile = kBlock * kScanItems;      // positions per scan block

struct Node {
    int b, e;        // segment of positions [b, e)
    u64 heap;        // heap id: root 1, children 2h, 2h+1
    long long sum;   // sum of quantised coordinates
    int dim;         // split dimension, -1: positional split only (depth cap)
    int depth;
    int mid;         // first position of the right child
    int moved;       // 1: mean split, 0: positional halves (ids stay where they are)
    int child[2];    // index in the next level's table, -1 if that child is a leaf
    int parent;      // position where the parent's right part starts, -1 for a root
};

struct Counters {
    int n_nodes[2];     // live nodes of level l in n_nodes[l & 1]; children_kernel fills the other one
    int bad_input;
    int small_nodes;
    int max_depth;      // deepest internal node (only tracked with node export)
};

// A node small enough to be finished inside one workgroup (finish_kernel).
struct SmallNode {
    int b, e;
    u64 heap;
    int depth, parent;      // parent: as in Node
};

// Record of an internal node kept for the conquer step above the leaves (Alg. 3), stored at
// the position where the node's right part starts (unique per node).  child[s] >= 0: the
// position that identifies an internal child, < 0: ~(first position of a leaf child).  Every
// field is written exactly once: sum .. depth by the node itself, child[s] by the node for a
// leaf child and by the child for an internal one.
struct NodeRec {
    long long sum;
    int dim, cnt, parent, depth;
    int child[2];
};
static_assert(sizeof(NodeRec) == sizeof(efanna_node), "record and exported node share a layout");

__device__ inline void record_node(NodeRec *rec, int *leaf_rec, int mid, long long sum, int dim,
                                   int cnt, int parent, int depth)
{
    NodeRec &r = rec[mid];
    r.sum = sum;
    r.dim = dim;
    r.cnt = cnt;
    r.parent = parent;
    r.depth = depth;
    if (parent >= 0) rec[parent].child[mid > parent ? 1 : 0] = mid;
    (void)leaf_rec;
}
__device__ inline void record_leaf(NodeRec *rec, int *leaf_rec, int b, int parent)
{
    leaf_rec[b] = parent;
    if (parent >= 0) rec[parent].child[b >= parent ? 1 : 0] = ~b;
}

constexpr int kFinMax = 2048;      // largest segment finish_kernel takes
constexpr int kFinNodes = 256;     // nodes of one level inside such a segment
constexpr int kFinThreads = 512;    // threads of a finish_kernel block
inline int finish_limit(int S)
{
    long f = (long)kFinNodes * (S + 1);     // so that a level never has more than kFinNodes live nodes
    return f < kFinMax ? (int)f : kFinMax;
}


// Transposed copy XT[d][n] of the data, with the input check folded in.  The splits read
// one coordinate of many points: in the row-major layout the upper levels (ids still
// nearly consecutive) would touch one 4-byte word out of every row, a stride that keeps
// hitting the same memory channels; in the transposed copy those reads are contiguous.
__global__ void __launch_bounds__(kBlock)
transpose_check_kernel(const float *__restrict__ X, int n, int d, float *__restrict__ XT, Counters *c, double terms)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    bool bad = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = r0 + ty + 8 * k, col = c0 + tx;
        float v = 0.0f;
        if (row < n && col < d) {
            v = X[(size_t)row * d + col];
            // false for NaN and inf as well; n |x| < 2^43 keeps cnt * q(x) and the sums below 2^63
            // (terms: how many coordinates a node's test adds up, 1 or kProjectionTerms)
            bad |= !(fabsf(v) < 1048576.0f) || (double)fabsf(v) * (double)n * terms >= 8796093022208.0;
        }
        tile[ty + 8 * k][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int col = c0 + ty + 8 * k, row = r0 + tx;
        if (row < n && col < d) XT[(size_t)col * n + row] = tile[tx][ty + 8 * k];
    }
    if (__any(bad) && ef_lane() == 0) atomicOr(&c->bad_input, 1);
}

// ---------------------------------------------------------------------------------------
// Split dimension by variance (split_rule 1), the rule of the randomized KD-tree that Sec. 3.2
// takes over: over the node's first kVarSample positions, the kVarDims dimensions with the
// largest integer variance m * sum(q^2) - sum(q)^2 of the quantised coordinates (equal ones:
// the smaller dimension first); the node's draw picks one of them.  One whole wave per node:
// lane l takes dimensions l, l + 64, ... and keeps its own best five in registers, then five
// rounds of a wave-wide maximum pop the overall order.  `ids` may point into LDS or global
// memory; every lane of the wave must call with the same arguments.
constexpr int kVarSample = 100, kVarDims = 5;
constexpr int kDimPending = -2;      // Node::dim of a node whose dimension is still to be chosen

struct VarKey {
    __int128 v;
    int j;
};
__device__ inline bool var_before(const VarKey &a, const VarKey &b)
{
    return a.v > b.v || (a.v == b.v && a.j < b.j);
}

__device__ inline int variance_dim_wave(const float *__restrict__ X, int d, const int *ids, int cnt, u64 draw)
{
    const int lane = ef_lane();
    const int m = cnt < kVarSample ? cnt : kVarSample;
    VarKey top[kVarDims];
#pragma unroll
    for (int r = 0; r < kVarDims; ++r) {
        top[r].v = -1;      // below every variance
        top[r].j = 0x7FFFFFFF;
    }
    for (int j = lane; j < d; j += EF_WAVE) {
        long long s1 = 0;
        __int128 s2 = 0;
        for (int p = 0; p < m; ++p) {
            const long long q = ef_quantise(X[(size_t)ids[p] * d + j]);
            s1 += q;
            s2 += (__int128)q * q;
        }
        VarKey c;
        c.v = (__int128)m * s2 - (__int128)s1 * s1;
        c.j = j;
#pragma unroll
        for (int r = 0; r < kVarDims; ++r)
            if (var_before(c, top[r])) {
                const VarKey t = top[r];
                top[r] = c;
                c = t;
            }
    }
    const int n_top = d < kVarDims ? d : kVarDims;
    const int want = (int)(draw % (u64)n_top);
    int chosen = 0;
    for (int r = 0; r < n_top; ++r) {      // (uniform)
        VarKey best = top[0];
        for (int o = EF_WAVE / 2; o >= 1; o >>= 1) {
            VarKey other;
            const u64 lo = __shfl_xor((u64)best.v, o, EF_WAVE);
            const u64 hi = __shfl_xor((u64)(best.v >> 64), o, EF_WAVE);
            other.v = (__int128)(((unsigned __int128)hi << 64) | lo);
            other.j = __shfl_xor(best.j, o, EF_WAVE);
            if (var_before(other, best)) best = other;
        }
        if (r == want) chosen = best.j;
        if (top[0].j == best.j) {      // the winner's lane moves on to its next one
#pragma unroll
            for (int q = 0; q + 1 < kVarDims; ++q) top[q] = top[q + 1];
            top[kVarDims - 1].v = -1;
            top[kVarDims - 1].j = 0x7FFFFFFF;
        }
    }
    return chosen;
}

// a fresh node's dimension code from its draw: the coordinate, "to be chosen by variance", or a projection
__device__ inline int node_dim(int rule, u64 draw, int d)
{
    return rule == 1 ? kDimPending : rule == 2 ? ef_projection_code(draw) : (int)(draw % (u64)d);
}

// One wave per live node of the level: fixes the dimension of the nodes that wait for one.
__global__ void __launch_bounds__(kBlock)
choose_dims_kernel(const float *__restrict__ X, int d, int n, const int *__restrict__ perm, Node *nodes,
                   int *dims, const Counters *c, int level, u64 seed)
{
    const int n_cur = c->n_nodes[level & 1];
    const int n_waves = gridDim.x * (kBlock / EF_WAVE);
    for (int s = blockIdx.x * (kBlock / EF_WAVE) + threadIdx.x / EF_WAVE; s < n_cur; s += n_waves) {
        const int b = nodes[s].b, e = nodes[s].e;
        if (nodes[s].dim != kDimPending) continue;      // (uniform)
        const u64 draw = ef_mix64(ef_stream_key(seed, b / n) + nodes[s].heap);
        const int dim = variance_dim_wave(X, d, perm + b, e - b, draw);
        if (ef_lane() == 0) {
            nodes[s].dim = dim;
            dims[s] = dim;
        }
    }
}

__global__ void roots_kernel(Node *nodes, int *dims, int *node_of, unsigned char *leaf_flag, int n,
                             int T, int S, int fin, SmallNode *small, u64 seed, int d, Counters *c, int rule)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n * T;
    const bool live = n > fin;       // otherwise the whole tree is finished in one workgroup
    if (p < (size_t)T && !live && n > S) {
        SmallNode sn;
        sn.b = (int)p * n;
        sn.e = sn.b + n;
        sn.heap = 1;
        sn.depth = 0;
        sn.parent = -1;
        small[p] = sn;
        if (p == 0) c->small_nodes = T;
    }
    if (p < total) {
        node_of[p] = live ? (int)(p / (size_t)n) : -1;
        leaf_flag[p] = (n <= S && p % (size_t)n == 0) ? 1 : 0;
    }
    if (p < (size_t)T && live) {
        Node nd;
        nd.b = (int)p * n;
        nd.e = nd.b + n;
        nd.heap = 1;
        nd.sum = 0;
        const u64 draw = ef_mix64(ef_stream_key(seed, (int)p) + 1);
        nd.dim = rule == 1 ? kDimPending : rule == 2 ? ef_projection_code(draw) : (int)(draw % (u64)d);
        nd.depth = 0;
        nd.mid = nd.b;
        nd.moved = 0;
        nd.child[0] = nd.child[1] = -1;
        nd.parent = -1;
        nodes[p] = nd;
        dims[p] = nd.dim;
    }
    if (p == 0) {
        c->n_nodes[0] = live ? T : 0;
        c->n_nodes[1] = 0;
    }
}

// `tiles` consecutive tiles of kBlock positions per block.  Near the root every tile of a block
// lies in the same node: their sums are carried in a register and go out as one atomic (the
// few node records of the top levels would otherwise take one atomic per tile, all to the same
// few addresses, which serialise).
__global__ void __launch_bounds__(kBlock)
sum_kernel(const float *__restrict__ XT, int n, const int *__restrict__ perm,
           const int *__restrict__ node_of, Node *nodes, const int *__restrict__ dims,
           float *__restrict__ val, size_t total, Counters *c, int level, int tiles,
           const float *__restrict__ X, int d)      // X: the rows (a projection adds up coordinates of one row)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) c->n_nodes[(level + 1) & 1] = 0;      // filled by children_kernel
    __shared__ long long wave_tot[kBlock / EF_WAVE];
    __shared__ int wave_node[kBlock / EF_WAVE];
    int carry_node = -1;          // thread 0: node and sum of the uniform tiles seen so far
    long long carry = 0;
    for (int tile = 0; tile < tiles; ++tile) {
        const size_t p = ((size_t)blockIdx.x * tiles + tile) * kBlock + threadIdx.x;
        if (((size_t)blockIdx.x * tiles + tile) * kBlock >= total) break;
        int s = -1;
        long long q = 0;
        if (p < total) {
            s = node_of[p];
            if (s >= 0) {
                // the split dimension comes from its own array: the node records are being hit
                // by the sum atomics of this very kernel, and reads of such a line crawl
                int dim = dims[s];
                if (dim >= 0) {
                    float x = XT[(size_t)dim * n + perm[p]];
                    val[p] = x;
                    q = ef_quantise(x);
                } else if (dim <= -3) {
                    const float *row = X + (size_t)perm[p] * d;
                    q = ef_node_value([&](int j) { return row[j]; }, d, dim);
                } else {
                    s = -1;
                }
            }
        }
        // Positions of a node are contiguous, so inside a wave equal node indices form runs.
        // Segmented inclusive scan over the runs; the last lane of a run then holds its sum.
        const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE;
        for (int o = 1; o < EF_WAVE; o <<= 1) {
            const long long q_up = __shfl_up(q, o, EF_WAVE);
            const int s_up = __shfl_up(s, o, EF_WAVE);
            if (lane >= o && s_up == s) q += q_up;
        }
        const int s_next = __shfl_down(s, 1, EF_WAVE);
        const bool tail = lane == EF_WAVE - 1 || s_next != s;
        const int s_first = __shfl(s, 0, EF_WAVE);
        const bool uniform = __all(s == s_first);      // the whole wave lies in one node
        if (lane == EF_WAVE - 1) {
            wave_tot[wave] = q;
            wave_node[wave] = uniform ? s : -2;
        }
        __syncthreads();
        // near the root a whole tile lies in one node: one sum for the tile
        bool tile_uniform = true;
        for (int w = 0; w < kBlock / EF_WAVE; ++w) tile_uniform &= wave_node[w] == wave_node[0] && wave_node[0] != -2;
        if (tile_uniform) {
            if (threadIdx.x == 0 && wave_node[0] >= 0) {
                long long tot = 0;
                for (int w = 0; w < kBlock / EF_WAVE; ++w) tot += wave_tot[w];
                if (wave_node[0] != carry_node) {
                    if (carry_node >= 0) atomicAdd((u64 *)&nodes[carry_node].sum, (u64)carry);
                    carry_node = wave_node[0];
                    carry = 0;
                }
                carry += tot;
            }
        } else if (tail && s >= 0) {
            atomicAdd((u64 *)&nodes[s].sum, (u64)q);
        }
        __syncthreads();      // wave_tot / wave_node are free for the next tile
    }
    if (threadIdx.x == 0 && carry_node >= 0) atomicAdd((u64 *)&nodes[carry_node].sum, (u64)carry);
}

// predicate sources for the scan
struct LeftPred {
    const int *node_of;
    const Node *nodes;
    const float *val;
    const float *X;      // rows and ids, for the nodes that split on a projection
    const int *perm;
    int d;
    __device__ int operator()(size_t p) const
    {
        int s = node_of[p];
        if (s < 0) return 0;
        const Node &nd = nodes[s];
        if (!ef_has_test(nd.dim)) return 0;
        long long cnt = nd.e - nd.b;
        if (nd.dim >= 0) return cnt * ef_quantise(val[p]) < nd.sum ? 1 : 0;
        const float *row = X + (size_t)perm[p] * d;
        return cnt * ef_node_value([&](int j) { return row[j]; }, d, nd.dim) < nd.sum ? 1 : 0;
    }
};
struct FlagPred {
    const unsigned char *flag;
    __device__ int operator()(size_t p) const { return flag[p]; }
};
// a predicate that scan_reduce_kernel has evaluated and kept, one bit per position
struct BitsPred {
    const u64 *bits;
    __device__ int operator()(size_t p) const { return (int)((bits[p >> 6] >> (p & 63)) & 1); }
};

// A scan block covers kScanTile consecutive positions; thread t looks at positions t,
// t + kBlock, ... of the tile, so that a wave reads consecutive words.  The predicates are
// single bits: a wave counts them with a ballot.
// bits (or null): the predicate of positions 64 w .. 64 w + 63 goes to bits[w], for the kernels
// that need it again.
template <class Pred>
__global__ void scan_reduce_kernel(Pred pred, size_t total, int *block_sums, u64 *__restrict__ bits)
{
    __shared__ int sh[kBlock / EF_WAVE];
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    int v = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const size_t p = base + (size_t)k * kBlock;      // lane 0: a multiple of 64
        const u64 bal = __ballot(p < total && pred(p));
        v += __popcll(bal);
        if (bits && ef_lane() == 0 && p < total) bits[p >> 6] = bal;
    }
    if (ef_lane() == 0) sh[threadIdx.x / EF_WAVE] = v;      // the whole wave holds the same count
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int w = 0; w < kBlock / EF_WAVE; ++w) tot += sh[w];
        block_sums[blockIdx.x] = tot;
    }
}

// exclusive scan of block_sums in place, single block; block_sums[nb] = grand total
__global__ void scan_blocksums_kernel(int *block_sums, int nb)
{
    __shared__ int sh[kBlock / EF_WAVE];
    __shared__ int carry_sh;
    if (threadIdx.x == 0) carry_sh = 0;
    __syncthreads();
    for (int base = 0; base < nb; base += kBlock) {
        int i = base + threadIdx.x;
        int v = i < nb ? block_sums[i] : 0;
        int inc = ef_wave_scan_i32(v);
        if (ef_lane() == EF_WAVE - 1) sh[threadIdx.x / EF_WAVE] = inc;
        __syncthreads();
        int woff = 0;
        for (int w = 0; w < (int)(threadIdx.x / EF_WAVE); ++w) woff += sh[w];
        int carry = carry_sh;
        if (i < nb) block_sums[i] = carry + woff + inc - v;
        __syncthreads();
        if (threadIdx.x == kBlock - 1) carry_sh = carry + woff + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) block_sums[nb] = carry_sh;
}

// out[p] = number of set predicates before p; out[total] = grand total
template <class Pred>
__global__ void scan_apply_kernel(Pred pred, size_t total, const int *block_sums, int nb, int *out)
{
    __shared__ int sh[kScanItems][kBlock / EF_WAVE];      // set bits per row of kBlock positions and wave
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE;
    const size_t base = (size_t)blockIdx.x * kScanTile + threadIdx.x;
    int before[kScanItems];      // set bits before this position inside its wave's 64 positions
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const size_t p = base + (size_t)k * kBlock;
        const u64 bal = __ballot(p < total && pred(p));
        before[k] = __popcll(bal & ((1ULL << lane) - 1));
        if (lane == 0) sh[k][wave] = __popcll(bal);
    }
    __syncthreads();
    int off = block_sums[blockIdx.x];
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        const size_t p = base + (size_t)k * kBlock;
        int mine = off + before[k];
        for (int w = 0; w < kBlock / EF_WAVE; ++w) {
            const int c = sh[k][w];
            mine += w < wave ? c : 0;
            off += c;
        }
        if (p < total) out[p] = mine;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[total] = block_sums[nb];
}

__global__ void children_kernel(Node *cur, int level, Node *next, int *next_dims,
                                const int *__restrict__ lcount,
                                unsigned char *leaf_flag, int S, int fin, SmallNode *small, u64 seed,
                                int n, int d, Counters *c, NodeRec *rec, int *leaf_rec, int rule)
{
    int s = blockIdx.x * blockDim.x + threadIdx.x;
    int kind[2] = {0, 0};      // 0 leaf, 1 finished later inside one workgroup, 2 next level
    Node nd;
    const int n_cur = c->n_nodes[level & 1];      // the launch covers the most nodes a level can have
    if (s < n_cur) {
        nd = cur[s];
        int cnt = nd.e - nd.b;
        int nl = ef_has_test(nd.dim) ? lcount[nd.e] - lcount[nd.b] : 0;
        if (nl == 0 || nl == cnt) {
            nd.moved = 0;
            nd.mid = nd.b + cnt / 2;
        } else {
            nd.moved = 1;
            nd.mid = nd.b + nl;
        }
        const int sz[2] = {nd.mid - nd.b, nd.e - nd.mid};
        for (int side = 0; side < 2; ++side) kind[side] = sz[side] <= S ? 0 : (sz[side] <= fin ? 1 : 2);
    }
    // one counter bump per wave and list
    const int want = (kind[0] == 2) + (kind[1] == 2), want_s = (kind[0] == 1) + (kind[1] == 1);
    const int inc = ef_wave_scan_i32(want), inc_s = ef_wave_scan_i32(want_s);
    const int wave_total = __shfl(inc, EF_WAVE - 1, EF_WAVE), wave_total_s = __shfl(inc_s, EF_WAVE - 1, EF_WAVE);
    int base = 0, base_s = 0;
    if (ef_lane() == EF_WAVE - 1) {
        if (wave_total > 0) base = atomicAdd(&c->n_nodes[(level + 1) & 1], wave_total);
        if (wave_total_s > 0) base_s = atomicAdd(&c->small_nodes, wave_total_s);
    }
    base = __shfl(base, EF_WAVE - 1, EF_WAVE);
    base_s = __shfl(base_s, EF_WAVE - 1, EF_WAVE);
    if (s >= n_cur) return;
    int slot = base + inc - want, slot_s = base_s + inc_s - want_s;
    if (rec) {
        record_node(rec, leaf_rec, nd.mid, nd.sum, nd.dim, nd.e - nd.b, nd.parent, nd.depth);
        if (s == 0) atomicMax(&c->max_depth, nd.depth);      // all nodes of a level share their depth
    }
    const int tree = nd.b / n;
    const u64 key = ef_stream_key(seed, tree);
    for (int side = 0; side < 2; ++side) {
        int cb = side ? nd.mid : nd.b, ce = side ? nd.e : nd.mid;
        // below depth 60 heap ids would overflow: such nodes only split positionally
        const u64 ch_heap = nd.depth < 60 ? 2 * nd.heap + side : nd.heap;
        nd.child[side] = -1;
        if (kind[side] == 2) {
            Node ch;
            ch.b = cb;
            ch.e = ce;
            ch.depth = nd.depth + 1;
            ch.heap = ch_heap;
            ch.dim = ch.depth < 60 ? node_dim(rule, ef_mix64(key + ch.heap), d) : -1;
            ch.sum = 0;
            ch.mid = cb;
            ch.moved = 0;
            ch.child[0] = ch.child[1] = -1;
            ch.parent = nd.mid;
            next[slot] = ch;
            next_dims[slot] = ch.dim;
            nd.child[side] = slot++;
        } else if (kind[side] == 1) {
            SmallNode sn;
            sn.b = cb;
            sn.e = ce;
            sn.heap = ch_heap;
            sn.depth = nd.depth + 1;
            sn.parent = nd.mid;
            small[slot_s++] = sn;
        } else {
            leaf_flag[cb] = 1;
            if (rec) record_leaf(rec, leaf_rec, cb, nd.mid);
        }
    }
    cur[s] = nd;
}

__global__ void scatter_kernel(const int *__restrict__ perm_in, int *__restrict__ perm_out,
                               const int *__restrict__ node_in, int *__restrict__ node_out,
                               const Node *__restrict__ nodes, const u64 *__restrict__ left_bits,
                               const int *__restrict__ lcount, size_t total)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= total) return;
    int s = node_in[p];
    int id = perm_in[p];
    if (s < 0) {
        perm_out[p] = id;
        node_out[p] = -1;
        return;
    }
    const Node nd = nodes[s];
    size_t dst = p;
    if (nd.moved) {
        const bool left = (left_bits[p >> 6] >> (p & 63)) & 1;      // the split test, as the scan evaluated it
        int lc = lcount[p] - lcount[nd.b];
        dst = left ? (size_t)nd.b + lc : (size_t)nd.mid + ((int)(p - nd.b) - lc);
    }
    perm_out[dst] = id;
    node_out[dst] = nd.child[dst < (size_t)nd.mid ? 0 : 1];
}

// Finishes the subtree of one small node (at most kFinMax positions) inside a workgroup:
// the same four steps per level as the device-wide kernels (integer sums, prefix sum of
// the "goes left" predicate, children, stable scatter), but with the ids, the node table
// and the prefix sums in LDS, so the lower half of a tree costs one launch instead of
// half a dozen per level.
struct LNode {
    int b, e, mid, moved;      // local positions
    u64 heap;
    long long sum;
    int dim, depth;
    int child[2];
    int parent, pad;           // parent: global position, as in Node
};

__global__ void __launch_bounds__(kFinThreads)
finish_kernel(const float *__restrict__ XT, int d, int *perm, const SmallNode *__restrict__ small,
              unsigned char *leaf_flag, int S, u64 seed, int n, NodeRec *rec, int *leaf_rec,
              int *max_depth, const float *__restrict__ X, int rule)
{
    // One 16-byte aligned LDS block carved by hand (no separate static LDS variables, whose
    // size would shift the 8-byte node records off their alignment).
    extern __shared__ __align__(16) int fsm[];
    int *const ids_base = fsm, *const nidx_base = fsm + 2 * kFinMax;      // [2][kFinMax] each
    float *val = (float *)(fsm + 4 * kFinMax);
    int *lcnt = fsm + 5 * kFinMax;                                 // [kFinMax + 1]
    int *wave_tot = fsm + 6 * kFinMax + 4;                         // [kFinThreads / EF_WAVE]
    int &n_next_sh = fsm[6 * kFinMax + 2];
    int &depth_sh = fsm[6 * kFinMax + 3];                          // deepest node of this subtree
    LNode *const tabs_base = (LNode *)(fsm + 6 * kFinMax + 32);     // [2][kFinNodes], 8-byte aligned
    long long *const pval = (long long *)(tabs_base + 2 * kFinNodes);      // [kFinMax] projections (only with that rule)
    // the quantised value position p is tested on, in a node with the dimension code dim
    auto tested = [&](int p, int dim) { return dim >= 0 ? ef_quantise(val[p]) : pval[p]; };
    const SmallNode seg = small[blockIdx.x];
    const int cnt = seg.e - seg.b, tid = threadIdx.x;
    const u64 key = ef_stream_key(seed, seg.b / n);
    for (int p = tid; p < cnt; p += kFinThreads) {
        ids_base[p] = perm[seg.b + p];
        nidx_base[p] = 0;
    }
    if (tid == 0) {
        LNode r;
        r.b = 0;
        r.e = cnt;
        r.mid = 0;
        r.moved = 0;
        r.heap = seg.heap;
        r.sum = 0;
        r.depth = seg.depth;
        r.dim = seg.depth < 60 ? node_dim(rule, ef_mix64(key + seg.heap), d) : -1;
        r.child[0] = r.child[1] = -1;
        r.parent = seg.parent;
        r.pad = 0;
        tabs_base[0] = r;
        n_next_sh = 0;
        depth_sh = seg.depth;
    }
    __syncthreads();
    int cur = 0, n_cur = 1;
    const int chunk = (cnt + kFinThreads - 1) / kFinThreads;      // consecutive positions per thread in the scan
    while (n_cur > 0) {
        int *idc = ids_base + cur * kFinMax, *idn = ids_base + (cur ^ 1) * kFinMax;
        int *nc = nidx_base + cur * kFinMax, *nn = nidx_base + (cur ^ 1) * kFinMax;
        LNode *tc = tabs_base + cur * kFinNodes, *tn = tabs_base + (cur ^ 1) * kFinNodes;
        // 0. split dimensions by variance, one wave per node
        if (rule == 1) {
            for (int k = tid / EF_WAVE; k < n_cur; k += kFinThreads / EF_WAVE) {
                if (tc[k].dim != kDimPending) continue;      // (uniform)
                const int dim = variance_dim_wave(X, d, idc + tc[k].b, tc[k].e - tc[k].b, ef_mix64(key + tc[k].heap));
                if (ef_lane() == 0) tc[k].dim = dim;
            }
            __syncthreads();
        }
        // 1. sums
        for (int p = tid; p < cnt; p += kFinThreads) {
            const int k = nc[p];
            if (k >= 0 && tc[k].dim >= 0) {
                const float x = XT[(size_t)tc[k].dim * n + idc[p]];
                val[p] = x;
                atomicAdd((u64 *)&tc[k].sum, (u64)ef_quantise(x));
            } else if (k >= 0 && tc[k].dim <= -3) {
                const float *row = X + (size_t)idc[p] * d;
                const long long v = ef_node_value([&](int j) { return row[j]; }, d, tc[k].dim);
                pval[p] = v;
                atomicAdd((u64 *)&tc[k].sum, (u64)v);
            }
        }
        __syncthreads();
        // 2. exclusive prefix sum of the "goes left" predicate over the segment
        {
            const int p0 = tid * chunk, p1 = min(cnt, p0 + chunk);
            int mine = 0;
            for (int p = p0; p < p1; ++p) {
                const int k = nc[p];
                int f = 0;
                if (k >= 0 && ef_has_test(tc[k].dim))
                    f = (long long)(tc[k].e - tc[k].b) * tested(p, tc[k].dim) < tc[k].sum ? 1 : 0;
                lcnt[p] = f;
                mine += f;
            }
            const int incl = ef_wave_scan_i32(mine);
            if (ef_lane() == EF_WAVE - 1) wave_tot[tid / EF_WAVE] = incl;
            __syncthreads();
            int off = incl - mine;
            for (int v = 0; v < tid / EF_WAVE; ++v) off += wave_tot[v];
            for (int p = p0; p < p1; ++p) {
                const int f = lcnt[p];
                lcnt[p] = off;
                off += f;
            }
            if (tid == kFinThreads - 1) lcnt[cnt] = off;      // the last thread's running sum is the total
        }
        __syncthreads();
        // 3. children
        for (int k = tid; k < n_cur; k += kFinThreads) {
            LNode nd = tc[k];
            const int c = nd.e - nd.b;
            const int nl = ef_has_test(nd.dim) ? lcnt[nd.e] - lcnt[nd.b] : 0;
            if (nl == 0 || nl == c) {
                nd.moved = 0;
                nd.mid = nd.b + c / 2;
            } else {
                nd.moved = 1;
                nd.mid = nd.b + nl;
            }
            if (rec) {
                record_node(rec, leaf_rec, seg.b + nd.mid, nd.sum, nd.dim, c, nd.parent, nd.depth);
                if (k == 0) depth_sh = nd.depth;      // levels are visited in order of depth
            }
            for (int side = 0; side < 2; ++side) {
                const int cb = side ? nd.mid : nd.b, ce = side ? nd.e : nd.mid;
                nd.child[side] = -1;
                if (ce - cb > S) {
                    LNode ch;
                    ch.b = cb;
                    ch.e = ce;
                    ch.mid = cb;
                    ch.moved = 0;
                    ch.depth = nd.depth + 1;
                    ch.heap = nd.depth < 60 ? 2 * nd.heap + side : nd.heap;
                    ch.dim = ch.depth < 60 ? node_dim(rule, ef_mix64(key + ch.heap), d) : -1;
                    ch.sum = 0;
                    ch.child[0] = ch.child[1] = -1;
                    ch.parent = seg.b + nd.mid;
                    ch.pad = 0;
                    const int slot = atomicAdd(&n_next_sh, 1);
                    tn[slot] = ch;
                    nd.child[side] = slot;
                } else {
                    leaf_flag[seg.b + cb] = 1;
                    if (rec) record_leaf(rec, leaf_rec, seg.b + cb, seg.b + nd.mid);
                }
            }
            tc[k] = nd;
        }
        __syncthreads();
        // 4. stable scatter
        for (int p = tid; p < cnt; p += kFinThreads) {
            const int k = nc[p];
            const int id = idc[p];
            if (k < 0) {
                idn[p] = id;
                nn[p] = -1;
                continue;
            }
            const LNode &nd = tc[k];
            int dst = p;
            if (nd.moved) {
                const bool left = (long long)(nd.e - nd.b) * tested(p, nd.dim) < nd.sum;
                const int lc = lcnt[p] - lcnt[nd.b];
                dst = left ? nd.b + lc : nd.mid + (p - nd.b - lc);
            }
            idn[dst] = id;
            nn[dst] = nd.child[dst < nd.mid ? 0 : 1];
        }
        __syncthreads();
        n_cur = n_next_sh;
        cur ^= 1;
        __syncthreads();
        if (tid == 0) n_next_sh = 0;
        __syncthreads();
    }
    for (int p = tid; p < cnt; p += kFinThreads) perm[seg.b + p] = ids_base[cur * kFinMax + p];
    if (rec && tid == 0) atomicMax(max_depth, depth_sh);
}

__global__ void iota_kernel(int *perm, int n, size_t total)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < total) perm[p] = (int)(p % (size_t)n);
}

__global__ void leaf_offsets_kernel(const unsigned char *__restrict__ leaf_flag,
                                    const int *__restrict__ rank, int n, int T, int max_leaves,
                                    int *__restrict__ leaf_off, int *__restrict__ n_leaves_dev)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n * T;
    if (p < total && leaf_flag[p]) {
        int t = (int)(p / (size_t)n);
        int idx = rank[p] - rank[(size_t)t * n];
        if (idx < max_leaves) leaf_off[(size_t)t * (max_leaves + 1) + idx] = (int)(p - (size_t)t * n);
    }
    if (p < (size_t)T) {
        int t = (int)p;
        int cnt = rank[(size_t)(t + 1) * n] - rank[(size_t)t * n];
        n_leaves_dev[t] = cnt;
        if (cnt <= max_leaves) leaf_off[(size_t)t * (max_leaves + 1) + cnt] = n;
    }
}

// Internal nodes and leaf parents, renumbered by leaves: the node whose right part starts with
// leaf l becomes node l of its tree (l >= 1), a leaf is named by its index.
__global__ void export_nodes_kernel(const unsigned char *__restrict__ leaf_flag,
                                    const int *__restrict__ rank, const NodeRec *__restrict__ rec,
                                    const int *__restrict__ leaf_rec, int n, int T, int max_leaves,
                                    efanna_node *__restrict__ nodes, int *__restrict__ leaf_up)
{
    size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n * T;
    if (p >= total || !leaf_flag[p]) return;
    const int t = (int)(p / (size_t)n);
    const int r0 = rank[(size_t)t * n];
    const int l = rank[p] - r0;
    if (l >= max_leaves) return;
    const size_t base = (size_t)t * (max_leaves + 1);
    // positions read back from the records are clamped into the tree: a slip in the
    // bookkeeping then shows as a wrong table, never as a stray read
    const int lo = t * n, hi = lo + n - 1;
    auto at = [&](int pos) { return rank[min(max(pos, lo), hi)] - r0; };
    const int par = leaf_rec[p];
    leaf_up[base + l] = par < 0 ? -1 : at(par) * 2 + (p >= (size_t)par ? 1 : 0);
    if (p == (size_t)t * n) return;      // the first leaf starts no node's right part
    const NodeRec r = rec[p];
    efanna_node o;
    o.sum = r.sum;
    o.dim = r.dim;
    o.cnt = r.cnt;
    o.parent = r.parent < 0 ? -1 : at(r.parent);
    o.depth = r.depth;
    for (int s = 0; s < 2; ++s) o.child[s] = r.child[s] >= 0 ? at(r.child[s]) : ~at(~r.child[s]);
    nodes[base + l] = o;
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct TreeWs {
    int *perm_tmp, *node_a, *node_b, *lcount, *block_sums, *n_leaves_dev;
    float *val, *xt;
    unsigned char *leaf_flag;
    u64 *left_bits;      // the split test of every position, one bit each
    Node *nodes_a, *nodes_b;
    int *dims_a, *dims_b;
    SmallNode *small;
    Counters *counters;
    NodeRec *rec;        // only with node export
    int *leaf_rec;
    size_t bytes;
};

TreeWs carve(void *ws, int64_t n, int32_t d, int32_t T, int32_t S, bool with_nodes)
{
    size_t total = (size_t)n * T;
    size_t max_nodes = total / (size_t)(S + 1) + (size_t)T + 1;
    size_t nb = (total + kScanTile - 1) / kScanTile;
    char *p = (char *)ws;
    size_t off = 0;
    TreeWs w;
    auto take = [&](size_t bytes) {
        char *r = p ? p + off : nullptr;
        off += align_up(bytes);
        return r;
    };
    w.perm_tmp = (int *)take(total * 4);
    w.node_a = (int *)take(total * 4);
    w.node_b = (int *)take(total * 4);
    w.lcount = (int *)take((total + 1) * 4);
    w.val = (float *)take(total * 4);
    w.left_bits = (u64 *)take((total / 64 + 1) * 8);
    w.leaf_flag = (unsigned char *)take(total);
    w.block_sums = (int *)take((nb + 1) * 4);
    w.nodes_a = (Node *)take(max_nodes * sizeof(Node));
    w.nodes_b = (Node *)take(max_nodes * sizeof(Node));
    w.small = (SmallNode *)take(max_nodes * sizeof(SmallNode));
    w.dims_a = (int *)take(max_nodes * 4);
    w.dims_b = (int *)take(max_nodes * 4);
    w.n_leaves_dev = (int *)take((size_t)T * 4);
    w.counters = (Counters *)take(sizeof(Counters));
    w.xt = (float *)take((size_t)n * d * 4);
    w.rec = with_nodes ? (NodeRec *)take(total * sizeof(NodeRec)) : nullptr;
    w.leaf_rec = with_nodes ? (int *)take(total * 4) : nullptr;
    w.bytes = off;
    return w;
}

// bits (or null): room for one bit per position; the predicate is then evaluated once and its
// bits serve the second pass (and the caller afterwards).
template <class Pred>
void device_scan(Pred pred, size_t total, int *block_sums, int *out, u64 *bits, hipStream_t st)
{
    int nb = (int)((total + kScanTile - 1) / kScanTile);
    scan_reduce_kernel<<<nb, kBlock, 0, st>>>(pred, total, block_sums, bits);
    scan_blocksums_kernel<<<1, kBlock, 0, st>>>(block_sums, nb);
    if (bits)
        scan_apply_kernel<<<nb, kBlock, 0, st>>>(BitsPred{bits}, total, block_sums, nb, out);
    else
        scan_apply_kernel<<<nb, kBlock, 0, st>>>(pred, total, block_sums, nb, out);
}

}  // namespace

extern "C" size_t efanna_trees_workspace_bytes(int64_t n, int32_t d, int32_t n_trees,
                                               int32_t leaf_size, int32_t with_nodes)
{
    if (n < 1 || d < 1 || n_trees < 1 || leaf_size < 1) return 0;
    return carve(nullptr, n, d, n_trees, leaf_size, with_nodes != 0).bytes;
}

extern "C" int efanna_build_trees_rule(const float *X, int64_t n, int32_t d, int32_t n_trees,
                                       int32_t leaf_size, uint64_t seed, int32_t split_rule, int32_t *perm,
                                       int32_t *leaf_off, int32_t max_leaves, int32_t *n_leaves,
                                       efanna_node *nodes, int32_t *leaf_up, int32_t *tree_depth,
                                       void *ws, size_t ws_bytes, void *stream)
{
    if (!X || !perm || !leaf_off || !n_leaves || (!nodes) != (!leaf_up)) return EFANNA_EINVAL;
    if (split_rule != EFANNA_SPLIT_UNIFORM && split_rule != EFANNA_SPLIT_VARIANCE &&
        split_rule != EFANNA_SPLIT_PROJECTION)
        return EFANNA_EINVAL;
    if (n < 1 || d < 1 || n_trees < 1 || n_trees > EFANNA_MAX_TREES || leaf_size < 1 ||
        leaf_size > EFANNA_MAX_LEAF || max_leaves < 1)
        return EFANNA_EINVAL;
    if ((double)n * n_trees >= 2147483647.0 - 4096.0) return EFANNA_EINVAL;
    if (!ws || ((uintptr_t)ws & 255) ||
        ws_bytes < efanna_trees_workspace_bytes(n, d, n_trees, leaf_size, nodes != nullptr))
        return EFANNA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int T = n_trees, S = leaf_size;
    const size_t total = (size_t)n * T;
    const int grid_pos = (int)((total + kBlock - 1) / kBlock);
    TreeWs w = carve(ws, n, d, T, S, nodes != nullptr);

    EF_HIP_CHECK(hipMemsetAsync(w.counters, 0, sizeof(Counters), st));
    if (nodes) EF_HIP_CHECK(hipMemsetAsync(w.leaf_rec, 0xFF, total * 4, st));      // a lone root leaf has no parent
    transpose_check_kernel<<<dim3((unsigned)((n + 31) / 32), (unsigned)((d + 31) / 32)), kBlock, 0, st>>>(
        X, (int)n, d, w.xt, w.counters, split_rule == EFANNA_SPLIT_PROJECTION ? (double)kProjectionTerms : 1.0);
    iota_kernel<<<grid_pos, kBlock, 0, st>>>(perm, (int)n, total);
    const int fin = finish_limit(S);
    roots_kernel<<<grid_pos, kBlock, 0, st>>>(w.nodes_a, w.dims_a, w.node_a, w.leaf_flag, (int)n, T, S, fin,
                                              w.small, seed, d, w.counters, split_rule);
    // The level counters are read into pinned host memory (one small buffer per calling thread,
    // kept for the life of the process): a copy to pageable memory is staged and takes some 20 us
    // longer, during which the GPU has nothing to do.  Without pinned memory: a local variable.
    Counters host_local;
    thread_local Counters *host_pinned = nullptr;
    if (!host_pinned && hipHostMalloc((void **)&host_pinned, sizeof(Counters), hipHostMallocDefault) != hipSuccess) {
        host_pinned = nullptr;
        (void)hipGetLastError();
    }
    Counters &host_c = host_pinned ? *host_pinned : host_local;
    EF_HIP_CHECK(hipMemcpyAsync(&host_c, w.counters, sizeof(Counters), hipMemcpyDeviceToHost, st));
    EF_HIP_CHECK(hipStreamSynchronize(st));
    if (host_c.bad_input) return EFANNA_EINPUT;

    int *perm_cur = perm, *perm_nxt = w.perm_tmp;
    int *node_cur = w.node_a, *node_nxt = w.node_b;
    Node *nodes_cur = w.nodes_a, *nodes_nxt = w.nodes_b;
    int *dims_cur = w.dims_a, *dims_nxt = w.dims_b;
    // Nodes of more than `fin` positions are split level by level, device-wide.  While
    // 2^level * fin < n some node of the level is certainly that large, so those levels are
    // enqueued without asking; after them the host looks at the count after every level.
    // A level has at most total / (fin + 1) + T live nodes (they are disjoint).
    int sure = 0;
    if (n > fin)
        for (long long cap = fin; cap < n; cap *= 2) ++sure;
    const int max_live = (int)(total / (size_t)(fin + 1)) + T;
    const int grid_nodes = (max_live + kBlock - 1) / kBlock;
    int n_cur = n > fin ? T : 0;
    for (int level = 0; n_cur > 0; ++level) {
        // sixteen tiles per block while nodes are a million positions and more (levels 0..3 of the headline)
        const int tiles = (total >> level) / (size_t)T >= (size_t)kBlock * 256 ? 16 : 1;
        if (split_rule == EFANNA_SPLIT_VARIANCE)
            choose_dims_kernel<<<min(grid_nodes * (kBlock / EF_WAVE), 2048), kBlock, 0, st>>>(
                X, d, (int)n, perm_cur, nodes_cur, dims_cur, w.counters, level, seed);
        sum_kernel<<<(grid_pos + tiles - 1) / tiles, kBlock, 0, st>>>(w.xt, (int)n, perm_cur, node_cur, nodes_cur,
                                                                      dims_cur, w.val, total, w.counters, level, tiles, X, d);
        LeftPred pred{node_cur, nodes_cur, w.val, X, perm_cur, d};
        device_scan(pred, total, w.block_sums, w.lcount, w.left_bits, st);
        children_kernel<<<grid_nodes, kBlock, 0, st>>>(
            nodes_cur, level, nodes_nxt, dims_nxt, w.lcount, w.leaf_flag, S, fin, w.small, seed, (int)n, d,
            w.counters, w.rec, w.leaf_rec, split_rule);
        scatter_kernel<<<grid_pos, kBlock, 0, st>>>(perm_cur, perm_nxt, node_cur, node_nxt, nodes_cur,
                                                    w.left_bits, w.lcount, total);
        if (level + 1 >= sure) {
            EF_HIP_CHECK(hipMemcpyAsync(&host_c, w.counters, sizeof(Counters), hipMemcpyDeviceToHost, st));
            EF_HIP_CHECK(hipStreamSynchronize(st));
            n_cur = host_c.n_nodes[(level + 1) & 1];
        }
        int *tp = perm_cur; perm_cur = perm_nxt; perm_nxt = tp;
        int *tn = node_cur; node_cur = node_nxt; node_nxt = tn;
        Node *tq = nodes_cur; nodes_cur = nodes_nxt; nodes_nxt = tq;
        int *td = dims_cur; dims_cur = dims_nxt; dims_nxt = td;
    }
    // host_c.small_nodes is current: it was read after the last level (or after the roots)
    if (host_c.small_nodes > 0) {
        const size_t fin_lds = (size_t)(6 * kFinMax + 32) * 4 + 2 * (size_t)kFinNodes * sizeof(LNode) +
                               (split_rule == EFANNA_SPLIT_PROJECTION ? (size_t)kFinMax * 8 : 0);
        EF_HIP_CHECK(hipFuncSetAttribute((const void *)finish_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)fin_lds));
        finish_kernel<<<host_c.small_nodes, kFinThreads, fin_lds, st>>>(w.xt, d, perm_cur, w.small, w.leaf_flag,
                                                                  S, seed, (int)n, w.rec, w.leaf_rec,
                                                                  &w.counters->max_depth, X, split_rule);
    }
    if (perm_cur != perm)
        EF_HIP_CHECK(hipMemcpyAsync(perm, perm_cur, total * 4, hipMemcpyDeviceToDevice, st));

    FlagPred fp{w.leaf_flag};
    device_scan(fp, total, w.block_sums, w.lcount, (u64 *)nullptr, st);
    leaf_offsets_kernel<<<grid_pos, kBlock, 0, st>>>(w.leaf_flag, w.lcount, (int)n, T, max_leaves,
                                                     leaf_off, w.n_leaves_dev);
    if (nodes)
        export_nodes_kernel<<<grid_pos, kBlock, 0, st>>>(w.leaf_flag, w.lcount, w.rec, w.leaf_rec, (int)n, T,
                                                         max_leaves, nodes, leaf_up);
    EF_HIP_CHECK(hipMemcpyAsync(n_leaves, w.n_leaves_dev, (size_t)T * 4, hipMemcpyDeviceToHost, st));
    if (nodes) EF_HIP_CHECK(hipMemcpyAsync(&host_c, w.counters, sizeof(Counters), hipMemcpyDeviceToHost, st));
    EF_HIP_CHECK(hipStreamSynchronize(st));
    if (tree_depth) {
        *tree_depth = -1;      // no internal node anywhere: every tree is a single leaf
        for (int t = 0; t < T; ++t)
            if (nodes && n_leaves[t] > 1) *tree_depth = host_c.max_depth;
    }
    EF_HIP_CHECK(hipGetLastError());
    for (int t = 0; t < T; ++t)
        if (n_leaves[t] > max_leaves) return EFANNA_ECAPACITY;
    return EFANNA_OK;
}

extern "C" int efanna_build_trees(const float *X, int64_t n, int32_t d, int32_t n_trees,
                                  int32_t leaf_size, uint64_t seed, int32_t *perm,
                                  int32_t *leaf_off, int32_t max_leaves, int32_t *n_leaves,
                                  efanna_node *nodes, int32_t *leaf_up, int32_t *tree_depth,
                                  void *ws, size_t ws_bytes, void *stream)
{
    return efanna_build_trees_rule(X, n, d, n_trees, leaf_size, seed, EFANNA_SPLIT_UNIFORM, perm, leaf_off,
                                   max_leaves, n_leaves, nodes, leaf_up, tree_depth, ws, ws_bytes, stream);
}
