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
// LDS regions are laid out in units of floats; round to 16 bytes so that 8- and 16-byte
// accesses stay aligned
__host__ __device__ inline int align4(int x) { return (x + 3) & ~3; }

// ---------------------------------------------------------------------------------------
// fills

// reverse lists: slot s of an empty list holds ~0 - s (above every real key)
__global__ void fill_reverse_kernel(u64 *a, u64 *b, size_t total, int L, int *work_count)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 2) work_count[i] = 0;
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

// A proposal waiting in the block's LDS queue: entry `key` offered to row `target`.
struct Proposal {
    u64 key;
    int target;
    int pad;
};

// Coalesced gather of m rows of X into LDS.  Fast path (d multiple of 4): the block's
// threads walk the m*(d/4) 16-byte pieces, eight loads in flight per thread.
// q4_magic = ceil(2^32 / (d/4)) turns the piece index into (row, column) without a
// division (exact while pieces * (d/4) < 2^32).
__device__ inline void gather_rows(const float *__restrict__ X, int d, int stride, u32 q4_magic,
                                   const int *uid, int m, float *rows, int tid, int nthr)
{
    if ((d & 3) == 0 && ((uintptr_t)X & 15) == 0) {
        const int q4 = d >> 2, total = m * q4;
        for (int f0 = tid; f0 < total; f0 += nthr * 8) {
            float4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int f = min(f0 + k * nthr, total - 1);   // clamped: always a valid piece
                const int r = q4 == 1 ? f : (int)(((u64)(u32)f * q4_magic) >> 32), c = f - r * q4;
                v[k] = *reinterpret_cast<const float4 *>(X + (size_t)uid[r] * d + 4 * c);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int f = f0 + k * nthr;
                if (f < total) {
                    const int r = q4 == 1 ? f : (int)(((u64)(u32)f * q4_magic) >> 32), c = f - r * q4;
                    *reinterpret_cast<float4 *>(rows + r * stride + 4 * c) = v[k];
                }
            }
        }
    } else {
        const int total = m * d;
        for (int f = tid; f < total; f += nthr) {
            const int r = f / d, c = f - r * d;
            rows[r * stride + c] = X[(size_t)uid[r] * d + c];
        }
    }
}

// Drain the proposal queue: every thread applies whole proposals on its own, so all the
// row reads of up to blockDim proposals are in flight together.
__device__ inline int drain_queue(const Proposal *queue, int count, u64 *graph, u32 *worst, int K,
                                  int tid, int nthr)
{
    int updates = 0;
    for (int e = tid; e < count; e += nthr) {
        const Proposal p = queue[e];
        u64 new_max;
        if (ef_bounded_insert(graph + (size_t)p.target * K, K, p.key, 1, &new_max)) {
            atomicMin(worst + p.target, ef_dist_bits(new_max));
            ++updates;
        }
    }
    return updates;
}

// The local join of one set of rows held in LDS: rows [0, m_new) are joined with each
// other and with rows [m_new, m).  uid: global ids, thr: threshold bits per row.
// queue: LDS, capacity q_cap >= 4 * blockDim; q_count: LDS counter (zeroed by the caller
// before the preceding barrier).  Returns this thread's number of accepted insertions.
__device__ inline int join_rows(const float *rows, int stride, int d, const int *uid,
                                const u32 *thr, int m_new, int m, Proposal *queue, int *q_count,
                                int q_cap, u64 *graph, u32 *worst, int K)
{
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int ntr = (m_new + 3) >> 2, ntc = (m + 3) >> 2;
    const int n_tiles = ntr * ntc - ntr * (ntr - 1) / 2;
    const int grp = tid >> 4, gl = tid & 15, n_grp = nthr >> 4;
    int updates = 0;
    for (int q0 = 0; q0 < n_tiles; q0 += n_grp) {
        const int q = q0 + grp;
        if (q < n_tiles) {
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
                const u32 db = __float_as_uint(dist);
                const int a = uid[ia], b = uid[ib];
                if (db <= thr[ia]) {
                    const int slot = atomicAdd(q_count, 1);
                    queue[slot].key = ef_pack(dist, b, 1);
                    queue[slot].target = a;
                }
                if (db <= thr[ib]) {
                    const int slot = atomicAdd(q_count, 1);
                    queue[slot].key = ef_pack(dist, a, 1);
                    queue[slot].target = b;
                }
            }
        }
        __syncthreads();
        const int count = *q_count;
        const bool last = q0 + n_grp >= n_tiles;
        if (last || count + 2 * nthr > q_cap) {     // next round could overflow: drain now
            updates += drain_queue(queue, count, graph, worst, K, tid, nthr);
            __syncthreads();
            if (tid == 0) *q_count = 0;
            __syncthreads();
        }
    }
    return updates;
}

// ---------------------------------------------------------------------------------------
// Alg. 3 at the leaves, one tree per launch, one block (one wave) per leaf.  Within one
// tree every point lies in exactly one leaf, so a block owns the graph rows of its
// members for the duration of the launch: rows are merged in LDS without atomics and
// written back sorted.  Launches of successive trees are ordered by the stream.

__global__ void __launch_bounds__(EF_WAVE)
init_tree_kernel(const float *__restrict__ X, int d, int stride, u32 q4_magic, int S,
                 const int *__restrict__ perm_t, const int *__restrict__ leaf_off_t, int K,
                 u64 *graph, int first_tree)
{
    extern __shared__ float smem[];
    float *rows = smem;                                   // [S][stride]
    float *dmat = smem + align4(S * stride);              // [S][S] pairwise distances
    u64 *pools = (u64 *)(dmat + align4(S * S));           // [S][K] rows being merged, ascending
    int *uid = (int *)(pools + (size_t)S * K);            // [S]
    const int lane = threadIdx.x;
    const int b = leaf_off_t[blockIdx.x];
    const int s = min(leaf_off_t[blockIdx.x + 1] - b, S);   // never overrun the buffers
    if (lane < s) uid[lane] = perm_t[b + lane];
    __syncthreads();
    gather_rows(X, d, stride, q4_magic, uid, s, rows, lane, EF_WAVE);
    for (int e = lane; e < s * K; e += EF_WAVE) {
        const int r = e / K, c = e - r * K;
        pools[e] = first_tree ? ef_empty_entry(K - 1 - c) : graph[(size_t)uid[r] * K + c];
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
            dmat[ia * S + ib] = dist;
            dmat[ib * S + ia] = dist;
        }
    }
    __syncthreads();
    if (lane < s) {   // lane a merges the other members into row a (kept ascending)
        u64 *row = pools + (size_t)lane * K;
        for (int o = 0; o < s; ++o) {
            if (o == lane) continue;
            const u64 key = ef_pack(dmat[lane * S + o], uid[o], 1);
            if (key >= row[K - 1]) continue;
            int pos = K - 1;
            while (pos > 0 && row[pos - 1] > key) --pos;
            if (pos > 0 && row[pos - 1] == key) continue;   // already there from an earlier tree
            for (int c = K - 1; c > pos; --c) row[c] = row[c - 1];
            row[pos] = key;
        }
    }
    __syncthreads();
    for (int e = lane; e < s * K; e += EF_WAVE) {
        const int r = e / K, c = e - r * K;
        graph[(size_t)uid[r] * K + c] = pools[e];
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
    // unused tails of both lists read as -1, so the join needs no counts to parse them
    const int n_new = min(total_new, L);
    for (int s = n_new + lane; s < L; s += EF_WAVE) nw[(size_t)i * L + s] = -1;
    for (int s = n_old + lane; s < K; s += EF_WAVE) od[(size_t)i * K + s] = -1;
    if (lane == 0) {
        nw_c[i] = n_new;
        od_c[i] = n_old;
        worst[i] = wbits;
    }
}

// After sampling: sort the points that have something to join into two work lists by an
// upper bound of the number of vectors their join gathers, so that the common small joins
// run with a small LDS footprint (many waves per CU) and only the few large ones pay for
// the worst case.  Points with an empty new set are dropped here.
__global__ void classify_kernel(const int *__restrict__ nw_c, const int *__restrict__ od_c,
                                const u64 *__restrict__ rnew, const u64 *__restrict__ rold, int n,
                                int L, int small_rows, int *__restrict__ work_small,
                                int *__restrict__ work_large, int *__restrict__ work_count,
                                int *__restrict__ cnt_evals, int *__restrict__ cnt_upd,
                                int *__restrict__ cnt_rows)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    int cls = -1;
    if (i < n) {
        int rn = 0, ro = 0;
        for (int s = 0; s < L; ++s) {
            rn += (u32)rnew[(size_t)i * L + s] < 0x80000000u ? 1 : 0;
            ro += (u32)rold[(size_t)i * L + s] < 0x80000000u ? 1 : 0;
        }
        const int ub_new = nw_c[i] + rn, ub = ub_new + od_c[i] + ro;
        if (ub_new >= 1 && ub >= 2) cls = ub <= small_rows ? 0 : 1;
        else cnt_evals[i] = cnt_upd[i] = cnt_rows[i] = 0;
    }
    const int lane = ef_lane();
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const u64 mask = __ballot(cls == c);
        if (mask == 0) continue;
        int base = 0;
        const int leader = __ffsll((long long)mask) - 1;
        if (lane == leader) base = atomicAdd(&work_count[c], __popcll(mask));
        base = __shfl(base, leader, EF_WAVE);
        if (cls == c) (c == 0 ? work_small : work_large)[base + __popcll(mask & ((1ULL << lane) - 1))] = i;
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 step 3+4: local joins.  Each block walks a work list (grid-strided), one point
// at a time.  cap_rows: how many vectors the LDS row buffer of this launch holds.

__global__ void join_kernel(const float *__restrict__ X, int n, int d, int stride, u32 q4_magic,
                            int K, int L,
                            const int *__restrict__ work, const int *__restrict__ work_count,
                            int cap_rows, const int *__restrict__ nw, const int *__restrict__ od,
                            const u64 *__restrict__ rnew, const u64 *__restrict__ rold,
                            u64 *graph, u32 *worst, int *__restrict__ cnt_evals,
                            int *__restrict__ cnt_upd, int *__restrict__ cnt_rows, int q_cap)
{
    extern __shared__ float smem[];
    const int n_cand = 3 * L + K;
    float *rows = smem;
    int *cand = (int *)(smem + align4(cap_rows * stride));   // [3L+K] raw candidates
    int *uid = cand + n_cand;                                 // [cap_rows] U_new ++ U_old
    u32 *thr = (u32 *)(uid + cap_rows);                       // [cap_rows]
    int *meta = (int *)(smem + align4(cap_rows * stride) + align4(n_cand + 2 * cap_rows));
    Proposal *queue = (Proposal *)(meta + 4);   // meta: [0] m_new [1] m_old [2] updates [3] queue count
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int count = *work_count;
    for (int w = blockIdx.x; w < count; w += gridDim.x) {
        const int i = work[w];
        // raw candidates: [0,L) sampled new, [L,2L) reverse new, [2L,2L+K) sampled old,
        // [2L+K,3L+K) reverse old; -1 = nothing
        for (int a = tid; a < n_cand; a += nthr) {
            int id;
            if (a < L) id = nw[(size_t)i * L + a];
            else if (a < 2 * L) {
                const u64 k = rnew[(size_t)i * L + (a - L)];
                id = (u32)k >= 0x80000000u ? -1 : (int)(u32)k;
            } else if (a < 2 * L + K) id = od[(size_t)i * K + (a - 2 * L)];
            else {
                const u64 k = rold[(size_t)i * L + (a - 2 * L - K)];
                id = (u32)k >= 0x80000000u ? -1 : (int)(u32)k;
            }
            cand[a] = id;
        }
        if (tid == 0) {
            meta[2] = 0;
            meta[3] = 0;
        }
        __syncthreads();
        // de-duplicate (first occurrence wins) and compact with wave 0
        if (tid < EF_WAVE) {
            int m = 0, m_new = 0;
            for (int base = 0; base < n_cand; base += EF_WAVE) {
                const int a = base + tid;
                bool keep = false;
                int id = -1;
                if (a < n_cand) {
                    id = cand[a];
                    keep = id >= 0;
                    for (int b = 0; b < a && keep; ++b) keep = cand[b] != id;
                }
                const u64 mask = __ballot(keep);
                if (keep) uid[m + __popcll(mask & ((1ULL << tid) - 1))] = id;
                // candidates below 2L are the new ones; 2L need not be a multiple of 64
                const int lim = 2 * L - base;
                const u64 new_mask = lim >= EF_WAVE ? ~0ULL : (lim <= 0 ? 0ULL : ((1ULL << lim) - 1));
                m_new += __popcll(mask & new_mask);
                m += __popcll(mask);
            }
            if (tid == 0) {
                meta[0] = m_new;
                meta[1] = m - m_new;
            }
        }
        __syncthreads();
        const int m_new = meta[0], m_old = meta[1], m = m_new + m_old;
        if (tid == 0) {
            cnt_evals[i] = m_new * (m_new - 1) / 2 + m_new * m_old;
            cnt_rows[i] = m;
        }
        for (int r = tid; r < m; r += nthr) thr[r] = ef_load_coherent(worst + uid[r]);
        gather_rows(X, d, stride, q4_magic, uid, m, rows, tid, nthr);
        __syncthreads();
        const int updates = join_rows(rows, stride, d, uid, thr, m_new, m, queue, &meta[3], q_cap,
                                      graph, worst, K);
        if (updates) atomicAdd(&meta[2], updates);
        __syncthreads();
        if (tid == 0) cnt_upd[i] = meta[2];
        __syncthreads();
    }
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
    int *nw, *od, *nw_c, *od_c, *cnt_evals, *cnt_upd, *cnt_rows, *work_small, *work_large, *work_count;
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
    w.work_small = (int *)take((size_t)n * 4);
    w.work_large = (int *)take((size_t)n * 4);
    w.work_count = (int *)take(2 * 4);
    w.rnew = (u64 *)take((size_t)n * L * 8);
    w.rold = (u64 *)take((size_t)n * L * 8);
    w.worst = (u32 *)take((size_t)n * 4);
    w.bytes = off;
    return w;
}

constexpr size_t kLdsLimit = 160 * 1024;

inline u32 q4_magic_for(int d)
{
    const u64 q4 = (u64)(d >> 2 ? d >> 2 : 1);
    return q4 == 1 ? 0xFFFFFFFFu : (u32)(((1ULL << 32) + q4 - 1) / q4);
}

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
    return 256;   // nothing is needed at present; kept so that callers need not change
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
    if (n * (int64_t)k >= 2147483647LL) return EFANNA_EINVAL;   // LDS row indices are 32-bit
    for (int t = 0; t < n_trees; ++t)
        if (n_leaves[t] < 1 || n_leaves[t] > max_leaves) return EFANNA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *const graph = (u64 *)graph_;
    const int stride = d + kRowPad;
    const size_t lds = (size_t)(align4(leaf_size * stride) + align4(leaf_size * leaf_size)) * 4 +
                       (size_t)leaf_size * k * 8 + (size_t)leaf_size * 4;
    if (lds > kLdsLimit) return EFANNA_EUNSUPPORTED;
    EF_HIP_CHECK(hipFuncSetAttribute((const void *)init_tree_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    for (int t = 0; t < n_trees; ++t)
        init_tree_kernel<<<n_leaves[t], EF_WAVE, lds, st>>>(
            X, d, stride, q4_magic_for(d), leaf_size, perm + (size_t)t * n, leaf_off + (size_t)t * (max_leaves + 1), k,
            graph, t == 0);
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
    // two launch shapes: joins that gather at most small_rows vectors, and the rest
    const int small_rows = max_rows <= 16 ? max_rows : (max_rows * 2 / 5 < 16 ? 16 : align4(max_rows * 2 / 5));
    auto threads_for = [](long pairs) {
        return pairs <= 1024 ? 64 : (pairs <= 4096 ? 128 : (pairs <= 12288 ? 256 : 512));
    };
    auto lds_for = [&](int cap_rows, int threads) {
        return (size_t)(align4(cap_rows * stride) + align4(max_rows + 2 * cap_rows)) * 4 + 16 +
               (size_t)(4 * threads) * sizeof(Proposal);
    };
    const int thr_large = threads_for((long)L * (2 * L - 1) + (long)2 * L * (K + L));
    const int thr_small = threads_for((long)small_rows * small_rows / 2);
    const size_t lds_large = lds_for(max_rows, thr_large), lds_small = lds_for(small_rows, thr_small);
    if (lds_large > kLdsLimit) return EFANNA_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    NndWs w = carve_nnd(ws, n, K, L);
    EF_HIP_CHECK(hipFuncSetAttribute((const void *)join_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_large));
    // persistent grids: as many blocks as fit the 256 CUs at once (LDS- or wave-limited), twice over
    auto grid_for_lds = [](size_t lds, int threads) {
        long per_cu = (long)(kLdsLimit / lds);
        const long by_waves = 32 / (threads / EF_WAVE);
        if (per_cu > by_waves) per_cu = by_waves;
        if (per_cu < 1) per_cu = 1;
        return (int)(256 * per_cu * 2);
    };
    const int grid_small = grid_for_lds(lds_small, thr_small), grid_large = grid_for_lds(lds_large, thr_large);
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
        fill_reverse_kernel<<<grid_for((size_t)n * L, kBlock), kBlock, 0, st>>>(
            w.rnew, w.rold, (size_t)n * L, L, w.work_count);
        sample_kernel<<<grid_for((size_t)n, rows_per_block), kBlock, 0, st>>>(
            graph, (int)n, K, L, ef_stream_key(seed, 2 * g), ef_stream_key(seed, 2 * g + 1), w.nw,
            w.od, w.nw_c, w.od_c, w.rnew, w.rold, w.worst);
        classify_kernel<<<grid_for((size_t)n, kBlock), kBlock, 0, st>>>(
            w.nw_c, w.od_c, w.rnew, w.rold, (int)n, L, small_rows, w.work_small, w.work_large,
            w.work_count, w.cnt_evals, w.cnt_upd, w.cnt_rows);
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[3 * it + 1], st));
        join_kernel<<<grid_small, thr_small, lds_small, st>>>(
            X, (int)n, d, stride, q4_magic_for(d), K, L, w.work_small, w.work_count, small_rows, w.nw, w.od, w.rnew,
            w.rold, graph, w.worst, w.cnt_evals, w.cnt_upd, w.cnt_rows, 4 * thr_small);
        if (small_rows < max_rows)
            join_kernel<<<grid_large, thr_large, lds_large, st>>>(
                X, (int)n, d, stride, q4_magic_for(d), K, L, w.work_large, w.work_count + 1, max_rows, w.nw, w.od,
                w.rnew, w.rold, graph, w.worst, w.cnt_evals, w.cnt_upd, w.cnt_rows, 4 * thr_large);
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
        for (int e = 0; e < iters * 3; ++e) (void)hipEventDestroy(ev[e]);
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
