// Graph kernels for gfx950: leaf brute force (Alg. 3 at the leaves), NN-descent
// (Alg. 4) and packing / unpacking of graph rows.
//
// Distance blocks are computed by groups of 16 lanes.  Lane l of a group owns the
// partial sum of coordinates j = l mod 16, which is exactly the library's fixed
// order of operations; a group works on a 4x4 tile of pairs at a time (4 + 4 row
// values feed 16 fused multiply-adds per lane and step), and a transposed butterfly
// leaves the finished distance of pair l in lane l.  Each lane then offers its pair to
// the two rows concerned through the lock-free bounded insertion.
#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowPad = 4;   // floats appended to each LDS row

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// ---------------------------------------------------------------------------------------
// fills

__global__ void fill_graph_kernel(u64 *graph, size_t total, int K)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) graph[i] = ef_empty_entry((int)(i % (size_t)K));
}

__global__ void fill_u32_kernel(u32 *p, size_t total, u32 v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) p[i] = v;
}

// reverse lists: slot s of an empty list holds ~0 - s (above every real key)
__global__ void fill_reverse_kernel(u64 *a, u64 *b, size_t total, int L)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) {
        u64 v = ~0ULL - (u64)(i % (size_t)L);
        a[i] = v;
        b[i] = v;
    }
}

// ---------------------------------------------------------------------------------------
// one 4x4 tile of squared distances by a 16-lane group.
// rows: LDS, `stride` floats per row.  ra[r], rb[c]: row indices.  Returns in lane gl the
// distance of pair (ra[gl >> 2], rb[gl & 3]).
__device__ inline float tile_distance(const float *rows, int stride, int d, const int (&ra)[4],
                                      const int (&rb)[4], int gl)
{
    float acc[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = 0.0f;
    const float *pa0 = rows + ra[0] * stride, *pa1 = rows + ra[1] * stride,
                *pa2 = rows + ra[2] * stride, *pa3 = rows + ra[3] * stride;
    const float *pb0 = rows + rb[0] * stride, *pb1 = rows + rb[1] * stride,
                *pb2 = rows + rb[2] * stride, *pb3 = rows + rb[3] * stride;
    for (int j = gl; j < d; j += 16) {
        float a[4] = {pa0[j], pa1[j], pa2[j], pa3[j]};
        float b[4] = {pb0[j], pb1[j], pb2[j], pb3[j]};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float diff = a[r] - b[c];
                acc[r * 4 + c] = __builtin_fmaf(diff, diff, acc[r * 4 + c]);
            }
    }
    return ef_group_transpose_reduce16(acc, gl);
}

// offer entry (dist, other) to row `target`
__device__ inline int offer(u64 *graph, u32 *worst, int K, int target, int other, float dist,
                            u32 threshold_bits)
{
    if (__float_as_uint(dist) > threshold_bits) return 0;
    u64 new_max;
    if (!ef_bounded_insert(graph + (size_t)target * K, K, ef_pack(dist, other, 1), 1, &new_max))
        return 0;
    atomicMin(worst + target, ef_dist_bits(new_max));
    return 1;
}

// ---------------------------------------------------------------------------------------
// Alg. 3 at the leaves: one wave per (tree, leaf)

struct LeafBase {
    int v[EFANNA_MAX_TREES + 1];   // v[t] = number of leaves in trees 0..t-1
};

template <int NW>
__global__ void __launch_bounds__(NW * EF_WAVE)
init_leaf_kernel(const float *__restrict__ X, int n, int d, int stride, int S,
                 const int *__restrict__ perm, const int *__restrict__ leaf_off, int max_leaves,
                 LeafBase leaf_base, int total_leaves, int K, u64 *graph, u32 *worst)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x / EF_WAVE, lane = ef_lane();
    float *rows = smem + (size_t)wave * S * stride;
    int *ids = (int *)(smem + (size_t)NW * S * stride) + wave * EF_WAVE;
    const int g = blockIdx.x * NW + wave;
    int s = 0;
    if (g < total_leaves) {
        int t = 0;
        while (g >= leaf_base.v[t + 1]) ++t;
        const int l = g - leaf_base.v[t];
        const int *off = leaf_off + (size_t)t * (max_leaves + 1);
        const int b = off[l];
        s = min(off[l + 1] - b, S);   // a leaf larger than announced is truncated, never overrun
        ids[lane] = lane < s ? perm[(size_t)t * n + b + lane] : -1;
    }
    __syncthreads();
    for (int r = 0; r < s; ++r) {
        const float *src = X + (size_t)ids[r] * d;
        for (int j = lane; j < d; j += EF_WAVE) rows[r * stride + j] = src[j];
    }
    __syncthreads();
    const int nt = (s + 3) >> 2, n_tiles = nt * (nt + 1) / 2;
    const int grp = lane >> 4, gl = lane & 15;
    for (int q = grp; q < n_tiles; q += 4) {
        int ti = 0, rem = q;
        while (rem >= nt - ti) {
            rem -= nt - ti;
            ++ti;
        }
        const int tj = ti + rem;
        int ra[4], rb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            ra[r] = min(4 * ti + r, s - 1);
            rb[r] = min(4 * tj + r, s - 1);
        }
        const float dist = tile_distance(rows, stride, d, ra, rb, gl);
        const int ia = 4 * ti + (gl >> 2), ib = 4 * tj + (gl & 3);
        if (ia < ib && ib < s) {
            const int a = ids[ia], b = ids[ib];
            offer(graph, worst, K, a, b, dist, ef_load_coherent(worst + a));
            offer(graph, worst, K, b, a, dist, ef_load_coherent(worst + b));
        }
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 step 1+2: sample the new / old sets of every row, clear the sampled marks,
// refresh the row's threshold and push the row's id into the reverse lists of the
// sampled neighbours.  One wave per row, up to 128 entries (two per lane).

__global__ void __launch_bounds__(kBlock)
sample_kernel(u64 *graph, int n, int K, int L, u64 key_new, u64 key_old, int *__restrict__ nw,
              int *__restrict__ od, int *__restrict__ nw_c, int *__restrict__ od_c, u64 *rnew,
              u64 *rold, u32 *worst)
{
    __shared__ u64 keys_sh[kBlock / EF_WAVE][2 * EF_WAVE];
    __shared__ u64 stop_sh[kBlock / EF_WAVE];
    const int wave = threadIdx.x / EF_WAVE, lane = ef_lane();
    const int i = blockIdx.x * (kBlock / EF_WAVE) + wave;
    u64 *keys = keys_sh[wave];
    u64 e[2] = {~0ULL, ~0ULL};
    if (i < n) {
        if (lane < K) e[0] = graph[(size_t)i * K + lane];
        if (lane + EF_WAVE < K) e[1] = graph[(size_t)i * K + lane + EF_WAVE];
    }
    keys[lane] = e[0];
    keys[lane + EF_WAVE] = e[1];
    if (lane == 0) stop_sh[wave] = ~0ULL;
    __syncthreads();
    if (i >= n) return;     // whole wave leaves together; no block barrier follows
    // ranks among new-marked and among old entries
    int rn[2] = {0, 0}, ro[2] = {0, 0};
    for (int k = 0; k < K; ++k) {
        const u64 o = keys[k];
        const bool o_new = o & 1, o_old = !o_new && !ef_is_empty(o);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const bool less = o < e[h];
            rn[h] += (less && o_new) ? 1 : 0;
            ro[h] += (less && o_old) ? 1 : 0;
        }
    }
    bool valid[2], is_new[2], is_old[2], take_new[2];
    int total_new = 0;
    u32 wbits = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        valid[h] = lane + h * EF_WAVE < K;
        is_new[h] = valid[h] && (e[h] & 1);
        is_old[h] = valid[h] && !(e[h] & 1) && !ef_is_empty(e[h]);
        take_new[h] = is_new[h] && rn[h] < L;
        total_new += is_new[h] ? 1 : 0;
        if (valid[h]) wbits = max(wbits, ef_dist_bits(e[h]));
        if (take_new[h] && rn[h] == L - 1) stop_sh[wave] = e[h];   // the L-th new entry
    }
    total_new = ef_wave_sum_i32(total_new);
    for (int m = 32; m >= 1; m >>= 1) wbits = max(wbits, (u32)__shfl_xor((int)wbits, m, EF_WAVE));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    const u64 stop = stop_sh[wave];     // ~0 when fewer than L new entries exist
    int n_old = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot = lane + h * EF_WAVE;
        const int id = ef_id(e[h]);
        if (take_new[h]) {
            nw[(size_t)i * L + rn[h]] = id;
            graph[(size_t)i * K + slot] = e[h] & ~1ULL;
            u64 nm;
            u64 hk = (ef_mix64(key_new + (((u64)(u32)id << 32) | (u32)i)) >> 32 << 32) | (u32)i;
            ef_bounded_insert(rnew + (size_t)id * L, L, hk, 0, &nm);
        }
        const bool take_old = is_old[h] && e[h] < stop;
        if (take_old) {
            od[(size_t)i * K + ro[h]] = id;
            u64 nm;
            u64 hk = (ef_mix64(key_old + (((u64)(u32)id << 32) | (u32)i)) >> 32 << 32) | (u32)i;
            ef_bounded_insert(rold + (size_t)id * L, L, hk, 0, &nm);
        }
        n_old += take_old ? 1 : 0;
    }
    n_old = ef_wave_sum_i32(n_old);
    if (lane == 0) {
        nw_c[i] = min(total_new, L);
        od_c[i] = n_old;
        worst[i] = wbits;
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 step 3+4: local join of one point per block.

__global__ void join_kernel(const float *__restrict__ X, int n, int d, int stride, int K, int L,
                            const int *__restrict__ nw, const int *__restrict__ od,
                            const int *__restrict__ nw_c, const int *__restrict__ od_c,
                            const u64 *__restrict__ rnew, const u64 *__restrict__ rold,
                            u64 *graph, u32 *worst, int *__restrict__ cnt_evals,
                            int *__restrict__ cnt_upd, int *__restrict__ cnt_rows)
{
    extern __shared__ float smem[];
    const int max_new = 2 * L, max_old = K + L, max_rows = max_new + max_old;
    float *rows = smem;
    int *cand = (int *)(smem + (size_t)max_rows * stride);   // [max_rows] raw candidates
    int *uid = cand + max_rows;                               // [max_rows] U_new ++ U_old
    u32 *thr = (u32 *)(uid + max_rows);                       // [max_rows]
    int *meta = (int *)(thr + max_rows);                      // [0] m_new [1] m_old [2] updates
    const int i = blockIdx.x;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int c_new = nw_c[i], c_old = od_c[i];
    // raw candidates: [0, c_new) sampled new, [c_new, c_new+L) reverse new,
    // then at max_new: [0, c_old) sampled old, [c_old, c_old+L) reverse old
    for (int a = tid; a < c_new + L; a += nthr) {
        int id;
        if (a < c_new) id = nw[(size_t)i * L + a];
        else {
            u64 k = rnew[(size_t)i * L + (a - c_new)];
            id = (u32)k >= 0x80000000u ? -1 : (int)(u32)k;
        }
        cand[a] = id;
    }
    for (int a = tid; a < c_old + L; a += nthr) {
        int id;
        if (a < c_old) id = od[(size_t)i * K + a];
        else {
            u64 k = rold[(size_t)i * L + (a - c_old)];
            id = (u32)k >= 0x80000000u ? -1 : (int)(u32)k;
        }
        cand[max_new + a] = id;
    }
    if (tid == 0) meta[2] = 0;
    __syncthreads();
    // de-duplicate (first occurrence wins) and compact with wave 0
    if (tid < EF_WAVE) {
        int m = 0;
        const int tot_new = c_new + L, tot_old = c_old + L;
        for (int base = 0; base < tot_new; base += EF_WAVE) {
            const int a = base + tid;
            bool keep = false;
            int id = -1;
            if (a < tot_new) {
                id = cand[a];
                keep = id >= 0;
                for (int b = 0; b < a && keep; ++b) keep = cand[b] != id;
            }
            const u64 mask = __ballot(keep);
            if (keep) uid[m + __popcll(mask & ((1ULL << tid) - 1))] = id;
            m += __popcll(mask);
        }
        const int m_new = m;
        for (int base = 0; base < tot_old; base += EF_WAVE) {
            const int a = base + tid;
            bool keep = false;
            int id = -1;
            if (a < tot_old) {
                id = cand[max_new + a];
                keep = id >= 0;
                for (int b = 0; b < a && keep; ++b) keep = cand[max_new + b] != id;
                for (int b = 0; b < tot_new && keep; ++b) keep = cand[b] != id;
            }
            const u64 mask = __ballot(keep);
            if (keep) uid[m + __popcll(mask & ((1ULL << tid) - 1))] = id;
            m += __popcll(mask);
        }
        if (tid == 0) {
            meta[0] = m_new;
            meta[1] = m - m_new;
        }
    }
    __syncthreads();
    const int m_new = meta[0], m_old = meta[1], m = m_new + m_old;
    const bool idle = m_new == 0 || m < 2;
    if (tid == 0) {
        cnt_evals[i] = m_new * (m_new - 1) / 2 + m_new * m_old;
        cnt_rows[i] = idle ? 0 : m;
        if (idle) cnt_upd[i] = 0;
    }
    if (idle) return;
    // gather rows and thresholds
    const int wave = tid / EF_WAVE, lane = ef_lane(), n_waves = nthr / EF_WAVE;
    for (int r = wave; r < m; r += n_waves) {
        const float *src = X + (size_t)uid[r] * d;
        for (int j = lane; j < d; j += EF_WAVE) rows[r * stride + j] = src[j];
    }
    for (int r = tid; r < m; r += nthr) thr[r] = ef_load_coherent(worst + uid[r]);
    __syncthreads();
    // distance tiles: row tiles over U_new, column tiles over U_new ++ U_old, tj >= ti
    const int ntr = (m_new + 3) >> 2, ntc = (m + 3) >> 2;
    const int n_tiles = ntr * ntc - ntr * (ntr - 1) / 2;
    const int grp = tid >> 4, gl = tid & 15, n_grp = nthr >> 4;
    int updates = 0;
    for (int q = grp; q < n_tiles; q += n_grp) {
        int ti = 0, rem = q;
        while (rem >= ntc - ti) {
            rem -= ntc - ti;
            ++ti;
        }
        const int tj = ti + rem;
        int ra[4], rb[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            ra[r] = min(4 * ti + r, m - 1);
            rb[r] = min(4 * tj + r, m - 1);
        }
        const float dist = tile_distance(rows, stride, d, ra, rb, gl);
        const int ia = 4 * ti + (gl >> 2), ib = 4 * tj + (gl & 3);
        if (ia < ib && ia < m_new && ib < m) {
            const int a = uid[ia], b = uid[ib];
            updates += offer(graph, worst, K, a, b, dist, thr[ia]);
            updates += offer(graph, worst, K, b, a, dist, thr[ib]);
        }
    }
    if (updates) atomicAdd(&meta[2], updates);
    __syncthreads();
    if (tid == 0) cnt_upd[i] = meta[2];
}

__global__ void stats_kernel(const int *__restrict__ cnt_evals, const int *__restrict__ cnt_upd,
                             const int *__restrict__ cnt_rows, int n, u64 *stats)
{
    long long ev = 0, up = 0, rw = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        ev += cnt_evals[i];
        up += cnt_upd[i];
        rw += cnt_rows[i];
    }
    ev = ef_wave_sum_i64(ev);
    up = ef_wave_sum_i64(up);
    rw = ef_wave_sum_i64(rw);
    if (ef_lane() == 0) {
        atomicAdd(stats, (u64)ev);
        atomicAdd(stats + 1, (u64)up);
        atomicAdd(stats + 2, (u64)rw);
    }
}

__global__ void zero_u64_kernel(u64 *p, int count)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

// ---------------------------------------------------------------------------------------
// rows in and out

__global__ void __launch_bounds__(kBlock)
get_graph_kernel(const u64 *__restrict__ graph, int n, int K, int *__restrict__ ids,
                 float *__restrict__ dists, unsigned char *__restrict__ flags)
{
    __shared__ u64 keys_sh[kBlock / EF_WAVE][2 * EF_WAVE];
    const int wave = threadIdx.x / EF_WAVE, lane = ef_lane();
    const int i = blockIdx.x * (kBlock / EF_WAVE) + wave;
    u64 *keys = keys_sh[wave];
    u64 e[2] = {~0ULL, ~0ULL};
    if (i < n) {
        if (lane < K) e[0] = graph[(size_t)i * K + lane];
        if (lane + EF_WAVE < K) e[1] = graph[(size_t)i * K + lane + EF_WAVE];
    }
    keys[lane] = e[0];
    keys[lane + EF_WAVE] = e[1];
    __syncthreads();
    if (i >= n) return;
    int rank[2] = {0, 0};
    for (int k = 0; k < K; ++k) {
        const u64 o = keys[k];
        rank[0] += o < e[0] ? 1 : 0;
        rank[1] += o < e[1] ? 1 : 0;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (lane + h * EF_WAVE >= K) continue;
        const size_t dst = (size_t)i * K + rank[h];
        const bool empty = ef_is_empty(e[h]);
        ids[dst] = empty ? -1 : ef_id(e[h]);
        dists[dst] = empty ? __uint_as_float(EF_INF_BITS) : __uint_as_float(ef_dist_bits(e[h]));
        if (flags) flags[dst] = empty ? 0 : (unsigned char)(e[h] & 1);
    }
}

__global__ void set_graph_kernel(u64 *graph, size_t total, int n, int K, const int *__restrict__ ids,
                                 const float *__restrict__ dists,
                                 const unsigned char *__restrict__ flags)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int id = ids[i];
    graph[i] = (id < 0 || id >= n) ? ef_empty_entry((int)(i % (size_t)K))
                      : ef_pack(dists[i], id, flags ? flags[i] : 1);
}

__global__ void pair_distances_kernel(const float *__restrict__ X, int d,
                                      const int *__restrict__ a_ids, const int *__restrict__ b_ids,
                                      size_t m, float *__restrict__ out)
{
    const size_t g = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4;
    const int gl = threadIdx.x & 15;
    const size_t gc = g < m ? g : m - 1;   // keep every lane of a group active
    const float *a = X + (size_t)a_ids[gc] * d, *b = X + (size_t)b_ids[gc] * d;
    float acc = 0.0f;
    for (int j = gl; j < d; j += 16) {
        float diff = a[j] - b[j];
        acc = __builtin_fmaf(diff, diff, acc);
    }
    acc = ef_group_reduce16(acc);
    if (g < m && gl == 0) out[g] = acc;
}

struct NndWs {
    int *nw, *od, *nw_c, *od_c, *cnt_evals, *cnt_upd, *cnt_rows;
    u64 *rnew, *rold;
    u32 *worst;
    size_t bytes;
};

NndWs carve_nnd(void *ws, int64_t n, int K, int L)
{
    char *p = (char *)ws;
    size_t off = 0;
    NndWs w;
    auto take = [&](size_t bytes) {
        char *r = p ? p + off : nullptr;
        off += align_up(bytes);
        return r;
    };
    w.nw = (int *)take((size_t)n * L * 4);
    w.od = (int *)take((size_t)n * K * 4);
    w.nw_c = (int *)take((size_t)n * 4);
    w.od_c = (int *)take((size_t)n * 4);
    w.cnt_evals = (int *)take((size_t)n * 4);
    w.cnt_upd = (int *)take((size_t)n * 4);
    w.cnt_rows = (int *)take((size_t)n * 4);
    w.rnew = (u64 *)take((size_t)n * L * 8);
    w.rold = (u64 *)take((size_t)n * L * 8);
    w.worst = (u32 *)take((size_t)n * 4);
    w.bytes = off;
    return w;
}

constexpr size_t kLdsLimit = 160 * 1024;

inline int grid_for(size_t total, int block) { return (int)((total + block - 1) / block); }

}  // namespace

extern "C" const char *efanna_status_string(int status)
{
    switch (status) {
    case EFANNA_OK: return "ok";
    case EFANNA_EINVAL: return "invalid argument";
    case EFANNA_EWORKSPACE: return "workspace missing, misaligned or too small";
    case EFANNA_EINPUT: return "input holds a non-finite value or |x| >= 2^20";
    case EFANNA_EHIP: return "HIP runtime error";
    case EFANNA_ECAPACITY: return "more leaves than max_leaves";
    case EFANNA_EUNSUPPORTED: return "shape not supported by this build";
    default: return "unknown status";
    }
}

extern "C" size_t efanna_init_workspace_bytes(int64_t n, int32_t n_trees)
{
    if (n < 1 || n_trees < 1) return 0;
    return align_up((size_t)n * 4);
}

extern "C" int efanna_init_graph(const float *X, int64_t n, int32_t d, const int32_t *perm,
                                 const int32_t *leaf_off, int32_t max_leaves,
                                 const int32_t *n_leaves, int32_t n_trees, int32_t leaf_size,
                                 int32_t k, efanna_entry *graph_, void *ws, size_t ws_bytes,
                                 void *stream)
{
    if (!X || !perm || !leaf_off || !n_leaves || !graph_) return EFANNA_EINVAL;
    if (n < 2 || d < 1 || n_trees < 1 || n_trees > EFANNA_MAX_TREES || leaf_size < 1 ||
        leaf_size > EFANNA_MAX_LEAF || k < 1 || k > EFANNA_MAX_K || k >= n || max_leaves < 1 ||
        n >= 2147483647LL - 256)
        return EFANNA_EINVAL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < efanna_init_workspace_bytes(n, n_trees))
        return EFANNA_EWORKSPACE;
    LeafBase leaf_base;
    leaf_base.v[0] = 0;
    for (int t = 0; t < EFANNA_MAX_TREES; ++t) {
        if (t < n_trees && (n_leaves[t] < 1 || n_leaves[t] > max_leaves)) return EFANNA_EINVAL;
        leaf_base.v[t + 1] = leaf_base.v[t] + (t < n_trees ? n_leaves[t] : 0);
    }
    const int total_leaves = leaf_base.v[n_trees];
    hipStream_t st = (hipStream_t)stream;
    u64 *const graph = (u64 *)graph_;
    u32 *worst = (u32 *)ws;
    const int stride = d + kRowPad;
    const size_t per_leaf = (size_t)leaf_size * stride * 4 + EF_WAVE * 4;
    if (per_leaf > kLdsLimit) return EFANNA_EUNSUPPORTED;
    int nw = (int)(65536 / per_leaf);
    nw = nw >= 4 ? 4 : (nw >= 2 ? 2 : 1);

    fill_graph_kernel<<<grid_for((size_t)n * k, kBlock), kBlock, 0, st>>>(graph, (size_t)n * k, k);
    fill_u32_kernel<<<grid_for((size_t)n, kBlock), kBlock, 0, st>>>(worst, (size_t)n, EF_INF_BITS);
    const size_t lds = per_leaf * nw;
    const int grid = (total_leaves + nw - 1) / nw;
#define EF_LAUNCH_INIT(NW)                                                                      \
    do {                                                                                        \
        EF_HIP_CHECK(hipFuncSetAttribute((const void *)init_leaf_kernel<NW>,                    \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        init_leaf_kernel<NW><<<grid, NW * EF_WAVE, lds, st>>>(X, (int)n, d, stride, leaf_size,  \
            perm, leaf_off, max_leaves, leaf_base, total_leaves, k, graph, worst);              \
    } while (0)
    if (nw == 4) EF_LAUNCH_INIT(4);
    else if (nw == 2) EF_LAUNCH_INIT(2);
    else EF_LAUNCH_INIT(1);
#undef EF_LAUNCH_INIT
    EF_HIP_CHECK(hipGetLastError());
    return EFANNA_OK;
}

extern "C" size_t efanna_nndescent_workspace_bytes(int64_t n, int32_t k, int32_t sample_L)
{
    if (n < 1 || k < 1 || sample_L < 1) return 0;
    return carve_nnd(nullptr, n, k, sample_L).bytes;
}

extern "C" int efanna_nndescent(const float *X, int64_t n, int32_t d, int32_t k,
                                efanna_entry *graph_, int32_t iters, int32_t sample_L,
                                uint64_t seed, int32_t first_iter, uint64_t *stats_,
                                float *phase_ms, void *ws, size_t ws_bytes, void *stream)
{
    if (!X || !graph_) return EFANNA_EINVAL;
    u64 *const graph = (u64 *)graph_;
    u64 *const stats = (u64 *)stats_;
    if (n < 2 || d < 1 || k < 1 || k > EFANNA_MAX_K || k >= n || iters < 0 || sample_L < 1 ||
        sample_L > EFANNA_MAX_SAMPLE || first_iter < 0 || n >= 2147483647LL - 256)
        return EFANNA_EINVAL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < efanna_nndescent_workspace_bytes(n, k, sample_L))
        return EFANNA_EWORKSPACE;
    const int K = k, L = sample_L;
    const int stride = d + kRowPad;
    const int max_rows = 3 * L + K;
    const size_t lds = (size_t)max_rows * stride * 4 + (size_t)max_rows * 12 + 16;
    if (lds > kLdsLimit) return EFANNA_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    NndWs w = carve_nnd(ws, n, K, L);
    // threads per join block: enough 16-lane groups for the largest possible block of pairs
    const long max_pairs = (long)L * (2 * L - 1) + (long)2 * L * (K + L);
    int join_threads = max_pairs <= 1024 ? 64 : (max_pairs <= 4096 ? 128 : (max_pairs <= 12288 ? 256 : 512));
    EF_HIP_CHECK(hipFuncSetAttribute((const void *)join_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    if (stats) zero_u64_kernel<<<grid_for((size_t)iters * 4 + 1, kBlock), kBlock, 0, st>>>(stats, iters * 4);
    const int rows_per_block = kBlock / EF_WAVE;
    // optional phase timing: events around the sampling and the join of every iteration
    hipEvent_t *ev = nullptr;
    if (phase_ms && iters > 0) {
        ev = new hipEvent_t[(size_t)iters * 3];
        for (int e = 0; e < iters * 3; ++e) EF_HIP_CHECK(hipEventCreate(&ev[e]));
    }
    for (int it = 0; it < iters; ++it) {
        const int g = first_iter + it;
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[3 * it], st));
        fill_reverse_kernel<<<grid_for((size_t)n * L, kBlock), kBlock, 0, st>>>(w.rnew, w.rold,
                                                                              (size_t)n * L, L);
        sample_kernel<<<grid_for((size_t)n, rows_per_block), kBlock, 0, st>>>(
            graph, (int)n, K, L, ef_stream_key(seed, 2 * g), ef_stream_key(seed, 2 * g + 1), w.nw,
            w.od, w.nw_c, w.od_c, w.rnew, w.rold, w.worst);
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[3 * it + 1], st));
        join_kernel<<<(int)n, join_threads, lds, st>>>(X, (int)n, d, stride, K, L, w.nw, w.od, w.nw_c,
                                                       w.od_c, w.rnew, w.rold, graph, w.worst,
                                                       w.cnt_evals, w.cnt_upd, w.cnt_rows);
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[3 * it + 2], st));
        if (stats)
            stats_kernel<<<256, kBlock, 0, st>>>(w.cnt_evals, w.cnt_upd, w.cnt_rows, (int)n,
                                                 stats + 4 * it);
    }
    EF_HIP_CHECK(hipGetLastError());
    if (ev) {
        EF_HIP_CHECK(hipStreamSynchronize(st));
        for (int it = 0; it < iters; ++it) {
            EF_HIP_CHECK(hipEventElapsedTime(&phase_ms[2 * it], ev[3 * it], ev[3 * it + 1]));
            EF_HIP_CHECK(hipEventElapsedTime(&phase_ms[2 * it + 1], ev[3 * it + 1], ev[3 * it + 2]));
        }
        for (int e = 0; e < iters * 3; ++e) hipEventDestroy(ev[e]);
        delete[] ev;
    }
    return EFANNA_OK;
}

extern "C" int efanna_get_graph(const efanna_entry *graph_, int64_t n, int32_t k, int32_t *ids,
                                float *dists, uint8_t *flags, void *stream)
{
    const u64 *const graph = (const u64 *)graph_;
    if (!graph || !ids || !dists || n < 1 || k < 1 || k > EFANNA_MAX_K) return EFANNA_EINVAL;
    get_graph_kernel<<<grid_for((size_t)n, kBlock / EF_WAVE), kBlock, 0, (hipStream_t)stream>>>(
        graph, (int)n, k, ids, dists, flags);
    EF_HIP_CHECK(hipGetLastError());
    return EFANNA_OK;
}

extern "C" int efanna_set_graph(efanna_entry *graph_, int64_t n, int32_t k, const int32_t *ids,
                                const float *dists, const uint8_t *flags, void *stream)
{
    u64 *const graph = (u64 *)graph_;
    if (!graph || !ids || !dists || n < 1 || k < 1 || k > EFANNA_MAX_K) return EFANNA_EINVAL;
    set_graph_kernel<<<grid_for((size_t)n * k, kBlock), kBlock, 0, (hipStream_t)stream>>>(
        graph, (size_t)n * k, (int)n, k, ids, dists, flags);
    EF_HIP_CHECK(hipGetLastError());
    return EFANNA_OK;
}

extern "C" int efanna_pair_distances(const float *X, int64_t n, int32_t d, const int32_t *a_ids,
                                     const int32_t *b_ids, int64_t m, float *out, void *stream)
{
    if (!X || !a_ids || !b_ids || !out || n < 1 || d < 1 || m < 0) return EFANNA_EINVAL;
    if (m == 0) return EFANNA_OK;
    pair_distances_kernel<<<grid_for((size_t)m * 16, kBlock), kBlock, 0, (hipStream_t)stream>>>(
        X, d, a_ids, b_ids, (size_t)m, out);
    EF_HIP_CHECK(hipGetLastError());
    return EFANNA_OK;
}
