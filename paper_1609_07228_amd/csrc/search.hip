// Search with the finished index (Alg. 1) for gfx950: the trees give a query its first
// candidates, the kNN graph expands them (NN-expansion).
//
// One wave per query, queries grid-strided over persistent waves.
//   1. trees   lane t searches tree t for the N_node = P / S / T + 1 closest leaves, best
//              bin first: going down it takes the child on the query's side of the split and
//              puts the other aside with the priority of the branch it follows plus the
//              squared distance from the query's coordinate to the node's mean; after a leaf
//              it continues from the branch with the smallest (priority, link) put aside.
//              Priorities are float64, computed with the same operations as any other
//              implementation of this rule would use (one division, one fused multiply-add).
//   2. pool    the members of those leaves are checked 64 at a time (one lane per point: the
//              lane evaluates the library's fixed-order distance on its own, sixteen running
//              sums) and merged by rank into the pool, a sorted list in LDS of at most E keys.
//   3. expand  `iters` times: every pool member that has not been expanded yet hands in its
//              graph neighbours; those not checked before are evaluated and merged, the pool
//              keeping the P closest.
// "Checked" is a hash set in the wave's slice of the workspace; an entry carries the number of
// the query it belongs to, so the table is never cleared between queries.
#include "common.h"

namespace {

constexpr int kMaxPool = 1024;

struct Branch {
    double prio;
    int link;
    int pad;
};

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

struct SearchShape {
    int want;           // leaves per tree
    int heap_cap;       // branches one tree can have put aside
    int max_first;      // most points the trees can hand in
    int table;          // hash table entries per wave (power of two)
    int waves;          // persistent waves
    size_t heap_bytes, table_bytes, roots_bytes, bytes, lds;
};

SearchShape search_shape(int64_t nq, int d, int T, int S, int tree_depth, int Kg, int P, int iters)
{
    SearchShape sh;
    sh.want = P / S / T + 1;
    sh.heap_cap = sh.want * (tree_depth + 2) + 2;      // a descent puts aside one branch per level
    sh.max_first = sh.want * T * S;
    long most = (long)sh.max_first + (long)iters * P * Kg;
    sh.table = 64;
    while (sh.table < 2 * most) sh.table <<= 1;
    // persistent waves, six per SIMD (the kernel takes 71 vector registers; measured on 10^5 queries:
    // 2 per SIMD 4.0 M queries/s at P = 200, 4: 6.3 M, 6: 6.7 M, 8: 5.8 M)
    sh.waves = (int)(nq < 1024 * 6 ? nq : 1024 * 6);
    if (sh.waves < 1) sh.waves = 1;
    sh.heap_bytes = align_up((size_t)sh.waves * T * sh.heap_cap * sizeof(Branch));
    sh.table_bytes = align_up((size_t)sh.waves * sh.table * 8);
    sh.roots_bytes = align_up((size_t)2 * T * 4);      // roots and a device copy of the leaf counts
    sh.bytes = sh.heap_bytes + sh.table_bytes + sh.roots_bytes;
    // LDS: query, pool, batch keys, expansion list, first candidates, leaves found
    sh.lds = (size_t)((d + 15) & ~15) * 4 + (size_t)P * 8 + 64 * 8 + (size_t)P * 4 +
             (size_t)sh.max_first * 4 + (size_t)T * sh.want * 4 + (size_t)T * 4 + 64;
    return sh;
}

// root of every tree: the node without a parent (0 for a tree that is a single leaf)
__global__ void find_roots_kernel(const efanna_node *__restrict__ nodes, int max_leaves, int T,
                                  const int *__restrict__ n_leaves_dev, int *roots)
{
    const int t = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    if (j == 0 && n_leaves_dev[t] <= 1) roots[t] = 0;
    if (j >= 1 && j < n_leaves_dev[t] && nodes[(size_t)t * (max_leaves + 1) + j].parent < 0) roots[t] = j;
}

// id joins the wave's checked set; true if it was not in it.  Entries are tag << 32 | id.
__device__ inline bool checked_insert(u64 *table, int mask, u32 tag, int id)
{
    u32 h = (u32)(ef_mix64((u64)(u32)id) >> 40) & (u32)mask;
    const u64 mine = ((u64)tag << 32) | (u32)id;
    for (int probes = 0; probes <= mask; ++probes) {
        u64 v = table[h];
        while ((u32)(v >> 32) != tag) {      // free, or left over from another query
            const u64 old = atomicCAS(&table[h], v, mine);
            if (old == v) return true;
            v = old;
        }
        if (v == mine) return false;
        h = (h + 1) & (u32)mask;
    }
    return false;      // a full table cannot happen: it holds twice what a query can check
}

// The library's distance between the query (LDS) and the row of every lane's candidate (`id`, -1
// = none), by the whole wave: sixteen candidates at a time, four lanes each.  Lane (r, g) = lane
// r + 16 g loads the 16-byte pieces 16 s + 4 g of row r, so that four lanes fetch 64 contiguous
// bytes and every byte fetched is used (a lane reading a whole row alone touches 64 rows per
// load and finds their lines evicted before it comes back for the rest); it accumulates
// partial sums 4g..4g+3 of the fixed order, and the four lanes of a row add up 8 apart, 4
// apart, 2 apart, 1 apart.  The candidate of lane 16 g + r is handled in round g by column r,
// so the lane that owns it is among the four that end up with its distance.
// Requires d % 4 == 0 and a 16-byte aligned X; q holds the query padded with zeros to a multiple of 16.
__device__ inline float wave_distances(const float *q, const float *__restrict__ X, int d, int id)
{
    const int lane = ef_lane(), r16 = lane & 15, g = lane >> 4;
    float mine = 0.0f;
    for (int round = 0; round < 4; ++round) {
        const int rid = __shfl(id, 16 * round + r16, EF_WAVE);
        if (__ballot(rid >= 0) == 0) continue;
        const float *row = X + (size_t)max(rid, 0) * d + 4 * g;
        float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
        for (int c0 = 0; c0 < d; c0 += 128) {
            float4 v[8];
#pragma unroll
            for (int s = 0; s < 8; ++s)
                v[s] = rid >= 0 && c0 + 16 * s + 4 * g + 3 < d ? *reinterpret_cast<const float4 *>(row + c0 + 16 * s)
                                                               : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                if (c0 + 16 * s >= d) break;
                const float4 y = *reinterpret_cast<const float4 *>(q + c0 + 16 * s + 4 * g);
                const bool in = c0 + 16 * s + 4 * g + 3 < d;      // beyond d both sides count as zero
                const float d0 = in ? y.x - v[s].x : 0.f, d1 = in ? y.y - v[s].y : 0.f,
                            d2 = in ? y.z - v[s].z : 0.f, d3 = in ? y.w - v[s].w : 0.f;
                p0 = __builtin_fmaf(d0, d0, p0);
                p1 = __builtin_fmaf(d1, d1, p1);
                p2 = __builtin_fmaf(d2, d2, p2);
                p3 = __builtin_fmaf(d3, d3, p3);
            }
        }
        p0 += __shfl_xor(p0, 32, EF_WAVE);
        p1 += __shfl_xor(p1, 32, EF_WAVE);
        p2 += __shfl_xor(p2, 32, EF_WAVE);
        p3 += __shfl_xor(p3, 32, EF_WAVE);
        p0 += __shfl_xor(p0, 16, EF_WAVE);
        p1 += __shfl_xor(p1, 16, EF_WAVE);
        p2 += __shfl_xor(p2, 16, EF_WAVE);
        p3 += __shfl_xor(p3, 16, EF_WAVE);
        const float dist = (p0 + p2) + (p1 + p3);
        if (g == round) mine = dist;
    }
    return mine;
}

// Merge the wave's batch (one key per lane, ~0 = none) into the sorted pool (count keys, room for
// cap), in place.  Returns the new count.  Keys are distinct.
// The batch is packed to the front of `batch` first: usually only a few of its keys are there
// at all (the others were checked before or lie beyond a full pool).  Pool members below the
// smallest fresh key stay where they are; the others move up by the number of fresh keys below
// them, 64 at a time from the top (a chunk is read before it is written, and it only writes at
// or above its own places), and the fresh keys take the places left free.
__device__ inline int pool_merge(u64 *pool, int count, int cap, u64 key, u64 *batch)
{
    const int lane = ef_lane();
    const u64 there = __ballot(key != ~0ULL);
    const int fresh = __popcll(there);
    if (key != ~0ULL) batch[__popcll(there & ((1ULL << lane) - 1))] = key;
    __syncthreads();
    int lo = count, pos = 0;
    if (key != ~0ULL) {
        int hi = count;
        lo = 0;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (pool[mid] < key) lo = mid + 1;
            else hi = mid;
        }
        pos = lo;
        for (int o = 0; o < fresh; ++o) pos += batch[o] < key ? 1 : 0;
    }
    int first = lo;                  // the lowest place any fresh key takes
    for (int m = 32; m >= 1; m >>= 1) first = min(first, __shfl_xor(first, m, EF_WAVE));
    for (int top = count; top > first; top -= EF_WAVE) {
        const int j = top - EF_WAVE + lane;
        u64 e = 0;
        int up = 0;
        if (j >= first) {
            e = pool[j];
            for (int o = 0; o < fresh; ++o) up += batch[o] < e ? 1 : 0;
        }
        __syncthreads();             // the chunk is in registers before any of it is overwritten
        if (j >= first && j + up < cap) pool[j + up] = e;
    }
    if (key != ~0ULL && pos < cap) pool[pos] = key;
    __syncthreads();
    return min(cap, count + fresh);
}

__global__ void __launch_bounds__(EF_WAVE)
search_kernel(const float *__restrict__ X, int d, int n, const int *__restrict__ perm,
              const int *__restrict__ leaf_off, int max_leaves, const int *__restrict__ n_leaves_dev,
              const efanna_node *__restrict__ nodes, const int *__restrict__ roots, int T, int S,
              const int *__restrict__ graph_ids, int Kg, const float *__restrict__ queries, int nq,
              int K, int P, int E, int iters, int want, int heap_cap, int max_first, int table_size,
              Branch *heaps, u64 *tables, int *out_ids, float *out_dists, int *out_checked)
{
    extern __shared__ __align__(16) float smem[];
    const int dq = (d + 15) & ~15;
    float *q = smem;                                   // [dq]
    u64 *cur = (u64 *)(smem + dq);                     // [P] the pool, ascending
    u64 *batch = cur + P;                              // [64]
    int *expand = (int *)(batch + EF_WAVE);            // [P]
    int *first = expand + P;                           // [max_first] members of the leaves found
    int *leaves = first + max_first;                   // [T][want]
    int *n_found = leaves + T * want;                  // [T]
    const int lane = threadIdx.x;
    u64 *table = tables + (size_t)blockIdx.x * table_size;
    const int mask = table_size - 1;
    for (int qi = blockIdx.x; qi < nq; qi += gridDim.x) {
        const u32 tag = (u32)qi + 1u;
        __syncthreads();                  // the previous query's LDS reads are done
        for (int j = lane; j < dq; j += EF_WAVE) q[j] = j < d ? queries[(size_t)qi * d + j] : 0.0f;
        __syncthreads();
        // ---- 1. trees: lane t searches tree t -----------------------------------------------
        for (int t = lane; t < T; t += EF_WAVE) {
            const efanna_node *nd_t = nodes + (size_t)t * (max_leaves + 1);
            const int last = n_leaves_dev[t] - 1;
            Branch *heap = heaps + ((size_t)blockIdx.x * T + t) * heap_cap;
            int n_heap = 0, found = 0;
            int link = last <= 0 ? ~0 : roots[t];
            double prio = 0.0;
            while (found < want) {
                for (int steps = 0; link >= 0 && steps < 4096; ++steps) {      // down to a leaf
                    const efanna_node nd = nd_t[min(link, last)];
                    bool left = true;
                    double other = prio;
                    if (ef_has_test(nd.dim)) {
                        const long long diff = (long long)nd.cnt * ef_node_value([&](int j) { return q[j]; }, d, nd.dim) - nd.sum;
                        left = diff < 0;
                        const double gap = (double)diff / ((double)nd.cnt * 1048576.0);
                        other = __fma_rn(gap, gap, prio);
                    }
                    if (n_heap < heap_cap) {
                        heap[n_heap].prio = other;
                        heap[n_heap].link = nd.child[left ? 1 : 0];
                        ++n_heap;
                    }
                    link = nd.child[left ? 0 : 1];
                }
                leaves[t * want + found++] = link >= 0 ? 0 : min(~link, max(last, 0));
                if (n_heap == 0) break;
                int best = 0;
                double bp = heap[0].prio;
                int bl = heap[0].link;
                for (int h = 1; h < n_heap; ++h) {
                    const double hp = heap[h].prio;
                    const int hl = heap[h].link;
                    if (hp < bp || (hp == bp && hl < bl)) {
                        best = h;
                        bp = hp;
                        bl = hl;
                    }
                }
                prio = bp;
                link = bl;
                --n_heap;
                heap[best] = heap[n_heap];
            }
            n_found[t] = found;
        }
        __syncthreads();
        // ---- 2. first pool: the members of the leaves found, 64 at a time ---------------------
        int n_first = 0;
        for (int t = 0; t < T; ++t)
            for (int f = 0; f < n_found[t]; ++f) {
                const int leaf = leaves[t * want + f];
                const int b = leaf_off[(size_t)t * (max_leaves + 1) + leaf];
                const int s = min(leaf_off[(size_t)t * (max_leaves + 1) + leaf + 1] - b, S);
                for (int r = lane; r < s; r += EF_WAVE) first[n_first + r] = perm[(size_t)t * n + b + r];
                n_first += s;
            }
        __syncthreads();
        int count = 0, checked = 0;
        for (int c0 = 0; c0 < n_first; c0 += EF_WAVE) {
            u64 key = ~0ULL;
            int cand = -1;
            if (c0 + lane < n_first) {
                const int id = first[c0 + lane];
                if (id >= 0 && id < n && checked_insert(table, mask, tag, id)) cand = id;
            }
            const float dist = wave_distances(q, X, d, cand);
            if (cand >= 0) key = ef_pack(dist, cand, 1);
            checked += __popcll(__ballot(key != ~0ULL));
            if (count == E && key >= cur[E - 1]) key = ~0ULL;      // a full pool takes nothing beyond its last key
            if (__ballot(key != ~0ULL) == 0) continue;
            count = pool_merge(cur, count, E, key, batch);
        }
        // ---- 3. NN-expansion ---------------------------------------------------------------------
        for (int it = 0; it < iters; ++it) {
            // members not expanded yet (mark bit set) lose the mark and go to the list
            int n_exp = 0;
            for (int j0 = 0; j0 < count; j0 += EF_WAVE) {
                const int j = j0 + lane;
                const u64 e = j < count ? cur[j] : 0;
                const bool take = j < count && (e & 1);
                const u64 bal = __ballot(take);
                if (take) {
                    cur[j] = e & ~1ULL;
                    expand[n_exp + __popcll(bal & ((1ULL << lane) - 1))] = ef_id(e);
                }
                n_exp += __popcll(bal);
            }
            __syncthreads();
            if (n_exp == 0) break;
            const int total = n_exp * Kg;
            for (int f0 = 0; f0 < total; f0 += EF_WAVE) {
                u64 key = ~0ULL;
                int cand = -1;
                const int f = f0 + lane;
                if (f < total) {
                    const int src = expand[f / Kg];
                    const int id = graph_ids[(size_t)src * Kg + f % Kg];
                    if (id >= 0 && id < n && checked_insert(table, mask, tag, id)) cand = id;
                }
                const float dist = wave_distances(q, X, d, cand);
                if (cand >= 0) key = ef_pack(dist, cand, 1);
                checked += __popcll(__ballot(key != ~0ULL));
                if (count == P && key >= cur[P - 1]) key = ~0ULL;      // a full pool takes nothing beyond its last key
                if (__ballot(key != ~0ULL) == 0) continue;
                count = pool_merge(cur, count, P, key, batch);
            }
        }
        // ---- result: the K closest --------------------------------------------------------------
        for (int c = lane; c < K; c += EF_WAVE) {
            const bool live = c < count;
            out_ids[(size_t)qi * K + c] = live ? ef_id(cur[c]) : -1;
            out_dists[(size_t)qi * K + c] = live ? __uint_as_float(ef_dist_bits(cur[c])) : __uint_as_float(EF_INF_BITS);
        }
        if (out_checked && lane == 0) out_checked[qi] = checked;
    }
}

__global__ void zero_tables_kernel(u64 *p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

}  // namespace

extern "C" size_t efanna_search_workspace_bytes(int64_t nq, int32_t d, int32_t n_trees,
                                                int32_t leaf_size, int32_t tree_depth,
                                                int32_t graph_k, int32_t pool, int32_t iters)
{
    if (nq < 1 || d < 1 || n_trees < 1 || leaf_size < 1 || graph_k < 1 || pool < 1 || iters < 0 ||
        tree_depth < -1)
        return 0;
    return search_shape(nq, d, n_trees, leaf_size, tree_depth, graph_k, pool, iters).bytes;
}

extern "C" int efanna_search(const float *X, int64_t n, int32_t d, const int32_t *perm,
                             const int32_t *leaf_off, int32_t max_leaves, const int32_t *n_leaves,
                             const efanna_node *nodes, int32_t tree_depth, int32_t n_trees,
                             int32_t leaf_size, const int32_t *graph_ids, int32_t graph_k,
                             const float *queries, int64_t nq, int32_t k, int32_t pool,
                             int32_t expand, int32_t iters, int32_t *ids, float *dists,
                             int32_t *checked, void *ws, size_t ws_bytes, void *stream)
{
    if (!X || !perm || !leaf_off || !n_leaves || !nodes || !graph_ids || !queries || !ids || !dists)
        return EFANNA_EINVAL;
    if (n < 1 || d < 1 || n_trees < 1 || n_trees > EFANNA_MAX_TREES || leaf_size < 1 ||
        leaf_size > EFANNA_MAX_LEAF || max_leaves < 1 || graph_k < 1 || nq < 1 || k < 1 || pool < k ||
        expand < 1 || expand > pool || iters < 0 || tree_depth < -1 || n >= 2147483647LL - 256 ||
        nq >= 2147483647LL - 256)
        return EFANNA_EINVAL;
    for (int t = 0; t < n_trees; ++t)
        if (n_leaves[t] < 1 || n_leaves[t] > max_leaves) return EFANNA_EINVAL;
    if (pool > kMaxPool || (d & 3) || ((uintptr_t)X & 15) || ((uintptr_t)queries & 15) || tree_depth > 4000)
        return EFANNA_EUNSUPPORTED;
    const SearchShape sh = search_shape(nq, d, n_trees, leaf_size, tree_depth, graph_k, pool, iters);
    if (sh.lds > 160 * 1024) return EFANNA_EUNSUPPORTED;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < sh.bytes) return EFANNA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)ws;
    Branch *heaps = (Branch *)base;
    u64 *tables = (u64 *)(base + sh.heap_bytes);
    int *roots = (int *)(base + sh.heap_bytes + sh.table_bytes);
    int *n_leaves_dev = roots + n_trees;
    EF_HIP_CHECK(hipMemcpyAsync(n_leaves_dev, n_leaves, (size_t)n_trees * 4, hipMemcpyHostToDevice, st));
    zero_tables_kernel<<<1024, 256, 0, st>>>(tables, (size_t)sh.waves * sh.table);
    find_roots_kernel<<<dim3((unsigned)((max_leaves + 255) / 256), (unsigned)n_trees), 256, 0, st>>>(
        nodes, max_leaves, n_trees, n_leaves_dev, roots);
    EF_HIP_CHECK(hipFuncSetAttribute((const void *)search_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh.lds));
    search_kernel<<<sh.waves, EF_WAVE, sh.lds, st>>>(
        X, d, (int)n, perm, leaf_off, max_leaves, n_leaves_dev, nodes, roots, n_trees, leaf_size, graph_ids,
        graph_k, queries, (int)nq, k, pool, expand, iters, sh.want, sh.heap_cap, sh.max_first, sh.table,
        heaps, tables, ids, dists, checked);
    EF_HIP_CHECK(hipGetLastError());
    // the copy of n_leaves reads host memory the caller may reuse: wait for it
    EF_HIP_CHECK(hipStreamSynchronize(st));
    return EFANNA_OK;
}
