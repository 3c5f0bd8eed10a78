// Graph kernels for gfx950: leaf brute force (Alg. 3 at the leaves), NN-descent
// (Alg. 4) and packing / unpacking of graph rows.
//
// Distance blocks are computed by groups of 16 lanes.  Lane l of a group owns the
// partial sum of coordinates j = l mod 16, which is exactly the library's fixed
// order of operations; a group works on a 4x4 tile of pairs at a time (4 + 4 row
// values feed 16 fused multiply-adds per lane and step), and a transposed butterfly
// leaves the finished distance of pair l in lane l.  Each lane then offers its pair to
// the two rows concerned through the lock-free bounded insertion.
#include <atomic>
#include <type_traits>
#include <vector>

#include "common.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRegGrid = 256 * 128;    // blocks of the register-operand join kernels (grid-strided over the work list)
constexpr int kLeafGrid = 256 * 256;   // blocks of the register-operand leaf kernels (a leaf or two each: measured 1.55 ms
                                       // per headline graph against 1.74 ms with 256 * 32, where a block walks eleven)
constexpr int kMaxLargeGrid = 256 * 32 * 2;     // most blocks the LDS-row join kernel is launched with
constexpr int kRowPad = 4;   // floats appended to each LDS row
constexpr int kMaxClasses = 8;      // most work lists (size classes of joins)

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
// LDS regions are laid out in units of floats; round to 16 bytes so that 8- and 16-byte
// accesses stay aligned
__host__ __device__ inline int align4(int x) { return (x + 3) & ~3; }

// ---------------------------------------------------------------------------------------
// fills

// number of overflow queues of the reverse lists, and ints between their counters
constexpr int kOvfQueues = 256, kOvfCounterPitch = 16;

// per-iteration reset: reverse-list fill counts and bounds, work-list sizes, insertion
// counts of the join blocks.  The lists themselves need no reset: the first L arrivals
// overwrite slots 0..L-1 in some order, readers stop at min(count, L), and the bounded
// insertion only ever touches lists that are full.
__global__ void fill_reverse_kernel(int *a_count, int *b_count, u64 *list_max, size_t n,
                                    int *work_count, int *upd_block, int n_upd_block, int *ovf_count)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < kMaxClasses) work_count[i] = 0;     // the work lists
    for (size_t j = i; j < (size_t)kOvfQueues * kOvfCounterPitch; j += (size_t)gridDim.x * blockDim.x) ovf_count[j] = 0;
    // insertion counts of join blocks: kernels that are not launched leave theirs at zero
    for (size_t j = i; j < (size_t)n_upd_block; j += (size_t)gridDim.x * blockDim.x) upd_block[j] = 0;
    if (i < n) {
        a_count[i] = 0;
        b_count[i] = 0;
        list_max[i] = ~0ULL;
        list_max[n + i] = ~0ULL;
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

// Number of set bits of a ballot below the calling lane.
__device__ inline int lanes_below(u64 ballot)
{
    return (int)__builtin_amdgcn_mbcnt_hi((u32)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((u32)ballot, 0u));
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
template <bool WIDE = false, bool REFINE = false>
__device__ inline int drain_queue(const Proposal *queue, int count, u64 *graph, u32 *worst, int K,
                                  int tid, int nthr)
{
    int updates = 0;
    for (int e = tid; e < count; e += nthr) {
        const Proposal p = queue[e];
        u64 new_max;
        if (ef_bounded_insert_t<WIDE, REFINE>(graph + (size_t)p.target * K, K, p.key, 1, &new_max)) {
            atomicMin(worst + p.target, ef_dist_bits(new_max));
            ++updates;
        }
    }
    return updates;
}

// The same for long rows (even length, 16-byte aligned): a group of sixteen threads per
// proposal (nthr a multiple of 16; all threads of the block call this together).
// gid (or null): the mirror of the rows' ids (graph_ids_kernel), kept up to date with the insertions.
__device__ inline int drain_queue_g16(const Proposal *queue, int count, u64 *graph, u32 *worst, int K,
                                      int tid, int nthr, int *gid = nullptr)
{
    int updates = 0;
    const int gl = tid & 15;
    for (int e = tid >> 4; e < count; e += nthr >> 4) {
        const Proposal p = queue[e];
        u64 new_max;
        int slot = 0;
        if (ef_bounded_insert_g16(graph + (size_t)p.target * K, K, p.key, 1, &new_max, gl, &slot) && gl == 0) {
            atomicMin(worst + p.target, ef_dist_bits(new_max));
            // (a plain store: whatever order stores to a slot land in, the slot names an id that was in the row)
            if (gid) gid[(size_t)p.target * K + slot] = ef_id(p.key);
            ++updates;
        }
    }
    return updates;
}

// ---------------------------------------------------------------------------------------
// Alg. 3 at the leaves, one tree per launch, one block per leaf (256 threads per 16 leaf
// slots).  Within one tree every point lies in exactly one leaf, so a block owns the graph
// rows of its members for the duration of the launch and needs no atomics.  Launches of
// successive trees are ordered by the stream.
//
// Rows and the members' old graph rows (ascending) go to LDS; distances come in 4x4 tiles by
// 16-lane groups; then every (row a, mate o) pair becomes a candidate key and the rows are
// merged by rank: a candidate's rank is the number of old entries below it (binary search,
// which also finds it if an earlier tree put it there already) plus the number of candidates
// of its row below it, an old entry's rank is its index plus the number of candidates below
// it; ranks below K are stored straight to the row.  Every slot of a row is written exactly
// once (K old entries plus the fresh candidates are at least K keys, all distinct).

__global__ void __launch_bounds__(1024)
init_tree_kernel(const float *__restrict__ X, int d, int stride, u32 q4_magic, int S,
                 const int *__restrict__ perm_t, const int *__restrict__ leaf_off_t, int K,
                 u64 *graph, int first_tree)
{
    extern __shared__ __align__(16) float smem[];
    float *rows = smem;                                   // [S][stride]
    float *dmat = smem + align4(S * stride);              // [S][S] distances, then (as int) old entries below
    u64 *pools = (u64 *)(dmat + align4(S * S));           // [S][K] old rows, ascending
    u64 *cand = pools + (size_t)S * K;                    // [S][S + 1] candidate keys of each row
    int *uid = (int *)(cand + (size_t)S * (S + 1));       // [S]
    int *ncand = uid + S;                                 // [S] candidates of each row that may enter it
    int *below = (int *)dmat;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int b = leaf_off_t[blockIdx.x];
    const int s = min(leaf_off_t[blockIdx.x + 1] - b, S);   // never overrun the buffers
    if (tid < s) uid[tid] = perm_t[b + tid];
    __syncthreads();
    gather_rows(X, d, stride, q4_magic, uid, s, rows, tid, nthr);
    for (int e = tid; e < s * K; e += nthr) {
        const int r = e / K, c = e - r * K;
        pools[e] = first_tree ? ef_empty_entry(K - 1 - c) : graph[(size_t)uid[r] * K + c];
    }
    __syncthreads();
    const int nt = (s + 3) >> 2, n_tiles = nt * (nt + 1) / 2;
    const int grp = tid >> 4, gl = tid & 15, n_grp = nthr >> 4;
    for (int q = grp; q < n_tiles; q += n_grp) {
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
    // candidate keys; the distance's slot then holds the number of old entries below the key
    const int pitch = S + 1;
    for (int e = tid; e < s * s; e += nthr) {
        const int a = e / s, o = e - a * s;
        u64 key = ~0ULL;
        int lo = 0;
        if (o != a) {
            key = ef_pack(dmat[a * S + o], uid[o], 1);
            if (!first_tree) {
                const u64 *row = pools + (size_t)a * K;
                int hi = K;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (row[mid] < key) lo = mid + 1;
                    else hi = mid;
                }
                if (lo < K && row[lo] == key) key = ~0ULL;      // already there from an earlier tree
            }
        }
        // A key above all K old entries stays out of the row, and so does every candidate above
        // it: it counts for nobody.  (Rows are full after a tree or two; from then on this is what
        // happens to most candidates.)
        if (lo >= K) key = ~0ULL;
        cand[a * pitch + o] = key;
        below[a * S + o] = lo;
    }
    __syncthreads();
    // the candidates still in the race move to the front of their row (a wave per row: its
    // lanes read the row before any of them writes), their number to ncand
    for (int a = tid / EF_WAVE; a < s; a += nthr / EF_WAVE) {
        const int o = ef_lane();
        const u64 key = o < s ? cand[a * pitch + o] : ~0ULL;
        const int lo = o < s ? below[a * S + o] : 0;
        const u64 alive = __ballot(key != ~0ULL);
        if (key != ~0ULL) {
            const int pos = __popcll(alive & ((1ULL << o) - 1));
            cand[a * pitch + pos] = key;
            below[a * S + pos] = lo;
        }
        if (o == 0) ncand[a] = __popcll(alive);
    }
    __syncthreads();
    for (int e = tid; e < s * s; e += nthr) {      // the candidates' places
        const int a = e / s, o = e - a * s, nc = ncand[a];
        if (o >= nc) continue;
        const u64 key = cand[a * pitch + o];
        int rank = below[a * S + o];
        for (int k = 0; k < nc; ++k) rank += cand[a * pitch + k] < key ? 1 : 0;
        if (rank < K) graph[(size_t)uid[a] * K + rank] = key;
    }
    for (int e = tid; e < s * K; e += nthr) {      // the old entries' places (a row without candidates stays as it is)
        const int a = e / K, j = e - a * K, nc = ncand[a];
        if (nc == 0 && !first_tree) continue;
        const u64 en = pools[e];
        int rank = j;
        for (int k = 0; k < nc; ++k) rank += cand[a * pitch + k] < en ? 1 : 0;
        if (rank < K) graph[(size_t)uid[a] * K + rank] = en;
    }
}

// ---------------------------------------------------------------------------------------
// The same step for leaves of at most 16 points (d % 4 == 0, X 16-byte aligned), without a
// row buffer: persistent waves, one leaf at a time.
//
// Lane (r, g) = lane r + 16 g keeps, of member r of the leaf, the coordinates 16 s + 4 g + k
// (s = 0..7, k = 0..3) of the current 128-coordinate piece, i.e. terms of partial sums
// 4g..4g+3 of the library's fixed order.  Rotating the 16 lanes of a row by t (a DPP modifier, no memory traffic) puts
// member r opposite member r +- t, so eight rotations meet all pairs of the leaf; the four
// lanes of a column then add their partial sums in the fixed tree (8 apart, 4 apart, 2
// apart, 1 apart), transposed so that lane (r, g) ends up with the distances of rotations
// 2g+1 and 2g+2, and fetches the two that its mirror lanes computed towards r.
//
// Merge: the leaf owns its members' graph rows during the launch.  The old row (ascending,
// in LDS) and the row's up to 15 candidates are merged by rank: a candidate's rank is the
// number of old entries below it (binary search, which also finds it if it is already in
// the row) plus the number of candidates below it; an old entry's rank is its index plus
// the number of candidates below it.  Ranks below K are stored straight to the row.
#define EF_ROW_ROR(x, t) __builtin_amdgcn_update_dpp(0, (x), 0x120 | (t), 0xF, 0xF, false)

template <int T>
__device__ inline void init_round(const float4 (&va)[8], int n_pieces, float (&p)[4])
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s >= n_pieces) break;
        const float d0 = va[s].x - __int_as_float(EF_ROW_ROR(__float_as_int(va[s].x), T));
        const float d1 = va[s].y - __int_as_float(EF_ROW_ROR(__float_as_int(va[s].y), T));
        const float d2 = va[s].z - __int_as_float(EF_ROW_ROR(__float_as_int(va[s].z), T));
        const float d3 = va[s].w - __int_as_float(EF_ROW_ROR(__float_as_int(va[s].w), T));
        p[0] = __builtin_fmaf(d0, d0, p[0]);
        p[1] = __builtin_fmaf(d1, d1, p[1]);
        p[2] = __builtin_fmaf(d2, d2, p[2]);
        p[3] = __builtin_fmaf(d3, d3, p[3]);
    }
}

// the same for two sets of sixteen rows: row r of the first against row r + T (rotation) of the second
template <int T>
__device__ inline void cross_round(const float4 (&va)[8], const float4 (&vb)[8], int n_pieces, float (&p)[4])
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s >= n_pieces) break;
        float4 w = vb[s];
        if (T != 0) {      // (T ? T : 1: the rotation count is an immediate and 0 is not a valid one, used or not)
            w.x = __int_as_float(EF_ROW_ROR(__float_as_int(vb[s].x), T ? T : 1));
            w.y = __int_as_float(EF_ROW_ROR(__float_as_int(vb[s].y), T ? T : 1));
            w.z = __int_as_float(EF_ROW_ROR(__float_as_int(vb[s].z), T ? T : 1));
            w.w = __int_as_float(EF_ROW_ROR(__float_as_int(vb[s].w), T ? T : 1));
        }
        const float d0 = va[s].x - w.x, d1 = va[s].y - w.y, d2 = va[s].z - w.z, d3 = va[s].w - w.w;
        p[0] = __builtin_fmaf(d0, d0, p[0]);
        p[1] = __builtin_fmaf(d1, d1, p[1]);
        p[2] = __builtin_fmaf(d2, d2, p[2]);
        p[3] = __builtin_fmaf(d3, d3, p[3]);
    }
}

constexpr int kCandPitch = 17;      // u64 per row of the candidate table (odd: rows on different banks)

__global__ void __launch_bounds__(EF_WAVE) __attribute__((amdgpu_waves_per_eu(4)))
init_reg_kernel(const float *__restrict__ X, int d, const int *__restrict__ perm_t,
                const int *__restrict__ leaf_off_t, int n_leaves, int K, u64 *graph, int first_tree)
{
    extern __shared__ __align__(16) float smem[];
    u64 *pools = (u64 *)smem;                         // [16][K] old rows, ascending
    u64 *cand = pools + 16 * (size_t)K;               // [16][kCandPitch] candidates of each row
    int *uid = (int *)(cand + 16 * kCandPitch);       // [16]
    const int lane = threadIdx.x, r16 = lane & 15, g = lane >> 4;
    // which way the rotation moves data: lane r receives from lane r + dirn (mod 16)
    const int dirn = (EF_ROW_ROR(r16, 1) - r16) & 15;
    // leaf boundaries are fetched two leaves ahead and member ids one leaf ahead
    int leaf = blockIdx.x;
    int b0 = leaf < n_leaves ? leaf_off_t[leaf] : 0;
    int s0 = leaf < n_leaves ? min(leaf_off_t[leaf + 1] - b0, 16) : 0;
    int id_pre = r16 < s0 ? perm_t[b0 + r16] : -1;
    int leaf1 = leaf + (int)gridDim.x;
    int b1 = leaf1 < n_leaves ? leaf_off_t[leaf1] : 0;
    int s1 = leaf1 < n_leaves ? min(leaf_off_t[leaf1 + 1] - b1, 16) : 0;
    for (; leaf < n_leaves; leaf += gridDim.x) {
        const int s = s0, my_id = id_pre;
        __syncthreads();                  // the previous leaf's LDS reads are done
        if (g == 0) uid[r16] = my_id;
        // old rows of this leaf
        for (int c = g; c < K; c += 4)
            pools[r16 * K + c] = first_tree || r16 >= s ? ef_empty_entry(K - 1 - c)
                                                        : graph[(size_t)my_id * K + c];
        // prefetch for the leaves to come
        s0 = s1;
        b0 = b1;
        id_pre = r16 < s0 ? perm_t[b0 + r16] : -1;
        leaf1 += gridDim.x;
        b1 = leaf1 < n_leaves ? leaf_off_t[leaf1] : 0;
        s1 = leaf1 < n_leaves ? min(leaf_off_t[leaf1 + 1] - b1, 16) : 0;
        // ---- distances: rotations 1..8, 128 coordinates at a time ---------------------------
        float P[8][4];
#pragma unroll
        for (int t = 0; t < 8; ++t) P[t][0] = P[t][1] = P[t][2] = P[t][3] = 0.0f;
        const float *pa = X + (size_t)max(my_id, 0) * d + 4 * g;
        for (int c0 = 0; c0 < d; c0 += 128) {
            float4 va[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const bool in = r16 < s && c0 + 16 * q + 4 * g + 3 < d;   // d % 4 == 0: a piece is in or out
                va[q] = in ? *reinterpret_cast<const float4 *>(pa + c0 + 16 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            const int n_pieces = min(8, (d - c0 + 15) >> 4);
            init_round<1>(va, n_pieces, P[0]);
            init_round<2>(va, n_pieces, P[1]);
            init_round<3>(va, n_pieces, P[2]);
            init_round<4>(va, n_pieces, P[3]);
            init_round<5>(va, n_pieces, P[4]);
            init_round<6>(va, n_pieces, P[5]);
            init_round<7>(va, n_pieces, P[6]);
            init_round<8>(va, n_pieces, P[7]);
        }
        // partial sums l and l+8 live 2 lanes-of-g apart (xor 32), l and l+4 one apart (xor 16)
        const bool hi = g & 2, odd = g & 1;
        float Q[4][4], R[2][4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float keep = hi ? P[t + 4][k] : P[t][k], send = hi ? P[t][k] : P[t + 4][k];
                Q[t][k] = keep + __shfl_xor(send, 32, EF_WAVE);
            }
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float keep = odd ? Q[t + 2][k] : Q[t][k], send = odd ? Q[t][k] : Q[t + 2][k];
                R[t][k] = keep + __shfl_xor(send, 16, EF_WAVE);
            }
        __syncthreads();                  // uid, pools visible
        // ---- candidates of row r16: rotations 2g+1, 2g+2, forwards and from the mirror lane ---
        u64 key[4];
        int lt[4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const float dist = (R[t][0] + R[t][2]) + (R[t][1] + R[t][3]);
            const int rot = 2 * g + 1 + t;
            const int bf = (r16 + dirn * rot) & 15, br = (r16 - dirn * rot) & 15;
            const float dist_r = __shfl(dist, br + 16 * g, EF_WAVE);     // lane br met r16 at this rotation
            key[t] = r16 < s && bf < s ? ef_pack(dist, uid[bf], 1) : ~0ULL;
            key[2 + t] = r16 < s && br < s && rot != 8 ? ef_pack(dist_r, uid[br], 1) : ~0ULL;
        }
        const u64 *row = pools + r16 * K;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int lo = 0, hi_ = K;
            if (key[c] != ~0ULL && !first_tree) {
                while (lo < hi_) {
                    const int mid = (lo + hi_) >> 1;
                    if (row[mid] < key[c]) lo = mid + 1;
                    else hi_ = mid;
                }
                if (lo < K && row[lo] == key[c]) key[c] = ~0ULL;      // already there from an earlier tree
            }
            lt[c] = lo;
            cand[r16 * kCandPitch + 4 * g + c] = key[c];
        }
        __syncthreads();
        // ---- ranks ----------------------------------------------------------------------------
        u64 cs[16];
#pragma unroll
        for (int o = 0; o < 16; ++o) cs[o] = cand[r16 * kCandPitch + o];
        if (r16 < s) {
            u64 *out = graph + (size_t)my_id * K;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (key[c] == ~0ULL) continue;
                int rank = lt[c];
#pragma unroll
                for (int o = 0; o < 16; ++o) rank += cs[o] < key[c] ? 1 : 0;
                if (rank < K) out[rank] = key[c];
            }
            for (int j = g; j < K; j += 4) {
                const u64 e = row[j];
                int rank = j;
#pragma unroll
                for (int o = 0; o < 16; ++o) rank += cs[o] < e ? 1 : 0;
                if (rank < K) out[rank] = e;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 3 above the leaves: for every ancestor N of a point's leaf with depth >= dep, the point
// is sent down the subtree of N's other child by the split test of each node it meets, and the
// members of the leaf it reaches become candidates.  Runs after the leaf step of the same
// tree, in two kernels: classify_kernel finds the leaf reached for every point and level,
// conquer_kernel (one wave per home leaf, which owns its members' graph rows during the
// launch) evaluates the distances and merges.
//
// The members of a home leaf share their ancestors but land in different leaves of a sibling
// subtree more often than not, so every member is handled against its own leaf: lane (r, g)
// keeps its share of home member r as in init_reg_kernel and loads the same share of the
// members of the leaf that r reached, one after the other (members that reached the same leaf
// find those rows in the cache).  Eight such members give eight sets of partial sums, which
// the four lanes of a row add up in the fixed tree, transposed, as for rotations.  Rows are
// merged by rank in LDS after every level and stored at the end.
// Requires leaves of at most 16 points, d % 4 == 0 and a 16-byte aligned X.

// partial sums of one pair: lane (r, g) adds the terms of its coordinates
__device__ inline void accumulate_pair(const float4 (&va)[8], const float4 (&vb)[8], int n_pieces, float (&p)[4])
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (s >= n_pieces) break;
        const float d0 = va[s].x - vb[s].x, d1 = va[s].y - vb[s].y, d2 = va[s].z - vb[s].z,
                    d3 = va[s].w - vb[s].w;
        p[0] = __builtin_fmaf(d0, d0, p[0]);
        p[1] = __builtin_fmaf(d1, d1, p[1]);
        p[2] = __builtin_fmaf(d2, d2, p[2]);
        p[3] = __builtin_fmaf(d3, d3, p[3]);
    }
}

// eight partial-sum sets (one per pair) -> lane g keeps the finished distances of pairs 2g
// and 2g+1 of the eight; same adds, in the same tree, as the fixed order
__device__ inline void reduce_rotations(const float (&P)[8][4], int g, float (&out)[2])
{
    const bool hi = g & 2, odd = g & 1;
    float Q[4][4], R[2][4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float keep = hi ? P[t + 4][k] : P[t][k], send = hi ? P[t][k] : P[t + 4][k];
            Q[t][k] = keep + __shfl_xor(send, 32, EF_WAVE);
        }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float keep = odd ? Q[t + 2][k] : Q[t][k], send = odd ? Q[t][k] : Q[t + 2][k];
            R[t][k] = keep + __shfl_xor(send, 16, EF_WAVE);
        }
#pragma unroll
    for (int t = 0; t < 2; ++t) out[t] = (R[t][0] + R[t][2]) + (R[t][1] + R[t][3]);
}

// The same for four rotations (T0 + 1 .. T0 + 4 in P[0..3]): lane (r, g) ends up with the distance
// from row r to the row T0 + 1 + g places on.
__device__ inline float reduce_rotations4(const float (&P)[4][4], int g)
{
    const bool hi = g & 2, odd = g & 1;
    float Q[2][4], R[4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float keep = hi ? P[t + 2][k] : P[t][k], send = hi ? P[t][k] : P[t + 2][k];
            Q[t][k] = keep + __shfl_xor(send, 32, EF_WAVE);
        }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float keep = odd ? Q[1][k] : Q[0][k], send = odd ? Q[0][k] : Q[1][k];
        R[k] = keep + __shfl_xor(send, 16, EF_WAVE);
    }
    return (R[0] + R[2]) + (R[1] + R[3]);
}

// Which leaf of each sibling subtree every point reaches: etab[p * levels + k] for the point at
// position p of the tree's id array and the k-th ancestor of its leaf (k = 0: the leaf's
// parent), -1 where there is no such ancestor or its depth is below dep.  A wave takes one
// leaf at a time: all lanes climb the ancestors together (the links are the same for every
// member), then lane (member r, slot g) sends member r down the sibling subtrees of ancestors
// g, g+4, ...  Light on registers, so that many waves hide the chains of dependent loads.
// Node j is the right child of its parent pj iff j > pj, leaf l iff l >= pj (nodes are
// numbered by the leaf that starts their right part).  Links are clamped to the tables and
// walks are bounded, so tables that are not the tree builder's cannot lead out of them.
__global__ void __launch_bounds__(kBlock)
classify_kernel(const float *__restrict__ X, int d, const int *__restrict__ perm_t,
                const int *__restrict__ leaf_off_t, int n_leaves,
                const efanna_node *__restrict__ nodes_t, const int *__restrict__ leaf_up_t, int dep,
                int levels, int *__restrict__ etab)
{
    __shared__ int sib_sh[kBlock / EF_WAVE][64];      // sibling subtree of the k-th ancestor
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE, r16 = lane & 15, g = lane >> 4;
    const int last = n_leaves - 1;
    const int n_waves = gridDim.x * (kBlock / EF_WAVE);
    for (int leaf = blockIdx.x * (kBlock / EF_WAVE) + wave; leaf < n_leaves; leaf += n_waves) {
        const int b0 = leaf_off_t[leaf];
        const int s = min(leaf_off_t[leaf + 1] - b0, 16);
        const int my_id = r16 < s ? perm_t[b0 + r16] : -1;
        int n_lev = 0;
        int up = min(leaf_up_t[leaf], 2 * last + 1);
        while (up >= 0 && n_lev < levels && n_lev < 64) {
            const int j = up >> 1;
            const efanna_node anc = nodes_t[j];
            if (anc.depth < dep) break;
            if (lane == 0) sib_sh[wave][n_lev] = anc.child[1 - (up & 1)];
            ++n_lev;
            const int pj = min(anc.parent, last);
            up = pj < 0 ? -1 : pj * 2 + (j > pj ? 1 : 0);
        }
        // one wave: its LDS operations complete in program order; keep the compiler from moving
        // the reads below above the writes
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (r16 < s) {
            for (int k = g; k < levels; k += 4) {
                int e = -1;
                if (k < n_lev) {
                    int c = sib_sh[wave][k];
                    for (int steps = 0; c >= 0 && steps < 4096; ++steps) {
                        const efanna_node nd = nodes_t[min(c, last)];
                        const float *xi = X + (size_t)my_id * d;
                        const bool left = !ef_has_test(nd.dim) ||
                                          (long long)nd.cnt * ef_node_value([&](int j) { return xi[j]; }, d, nd.dim) < nd.sum;
                        c = nd.child[left ? 0 : 1];
                    }
                    e = c >= 0 ? 0 : min(~c, last);
                }
                etab[(size_t)(b0 + r16) * levels + k] = e;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ void __launch_bounds__(EF_WAVE)
conquer_kernel(const float *__restrict__ X, int d, const int *__restrict__ perm_t,
               const int *__restrict__ leaf_off_t, int n_leaves, const int *__restrict__ etab,
               int levels, int K, u64 *graph)
{
    extern __shared__ __align__(16) float smem[];
    u64 *pools_a = (u64 *)smem;                       // [16][K] rows being merged, ascending
    u64 *pools_b = pools_a + 16 * (size_t)K;          // [16][K] the other copy
    u64 *cand = pools_b + 16 * (size_t)K;             // [16][kCandPitch]
    int *uid_b = (int *)(cand + 16 * kCandPitch);     // [16][16] members of the leaf each row reached
    const int lane = threadIdx.x, r16 = lane & 15, g = lane >> 4;
    for (int leaf = blockIdx.x; leaf < n_leaves; leaf += gridDim.x) {
        const int b0 = leaf_off_t[leaf];
        const int s = min(leaf_off_t[leaf + 1] - b0, 16);
        // the ancestors are those of the leaf: a level exists for all members or for none
        int e = r16 < s ? etab[(size_t)(b0 + r16) * levels] : -1;
        if (__ballot(e >= 0) == 0) continue;      // nothing above this leaf to visit
        const int my_id = r16 < s ? perm_t[b0 + r16] : -1;
        const float *pa = X + (size_t)max(my_id, 0) * d + 4 * g;
        __syncthreads();                  // the previous leaf's LDS reads are done
        u64 *cur = pools_a, *nxt = pools_b;
        for (int c = g; c < K; c += 4)
            cur[r16 * K + c] = r16 < s ? graph[(size_t)my_id * K + c] : ef_empty_entry(K - 1 - c);
        for (int k = 0; k < levels; ++k) {
            if (k > 0) {
                e = r16 < s ? etab[(size_t)(b0 + r16) * levels + k] : -1;
                if (__ballot(e >= 0) == 0) break;
            }
            e = min(e, n_leaves - 1);
            {
                // ---- every member against the members of the leaf it reached ----------------------
                const bool target = e >= 0;
                const int bb = target ? leaf_off_t[e] : 0;
                const int sb = target ? min(leaf_off_t[e + 1] - bb, 16) : 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = 4 * g + q;
                    uid_b[r16 * 16 + j] = j < sb ? perm_t[bb + j] : -1;
                }
                __syncthreads();                  // uid_b and the current rows are visible
                float dist[4];      // members 2g, 2g+1, 8+2g, 8+2g+1 of that leaf
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    float P[8][4];
#pragma unroll
                    for (int t = 0; t < 8; ++t) P[t][0] = P[t][1] = P[t][2] = P[t][3] = 0.0f;
                    for (int c0 = 0; c0 < d; c0 += 128) {
                        float4 va[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const bool in = c0 + 16 * q + 4 * g + 3 < d;      // d % 4 == 0: a piece is in or out
                            va[q] = in && r16 < s ? *reinterpret_cast<const float4 *>(pa + c0 + 16 * q)
                                                  : make_float4(0.f, 0.f, 0.f, 0.f);
                        }
                        const int n_pieces = min(8, (d - c0 + 15) >> 4);
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const int id_b = uid_b[r16 * 16 + 8 * half + t];
                            const float *pb = X + (size_t)max(id_b, 0) * d + 4 * g + c0;
                            float4 vb[8];
#pragma unroll
                            for (int q = 0; q < 8; ++q) {
                                const bool in = c0 + 16 * q + 4 * g + 3 < d;
                                vb[q] = in && id_b >= 0 ? *reinterpret_cast<const float4 *>(pb + 16 * q)
                                                        : make_float4(0.f, 0.f, 0.f, 0.f);
                            }
                            accumulate_pair(va, vb, n_pieces, P[t]);
                        }
                    }
                    float two[2];
                    reduce_rotations(P, g, two);
                    dist[2 * half] = two[0];
                    dist[2 * half + 1] = two[1];
                }
                // ---- candidates of row r16 and their ranks ------------------------------------
                u64 key[4];
                int lt[4];
                const u64 *row = cur + r16 * K;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int bm = 8 * (c >> 1) + 2 * g + (c & 1);      // member of the leaf reached
                    key[c] = bm < sb ? ef_pack(dist[c], uid_b[r16 * 16 + bm], 1) : ~0ULL;
                    int lo = 0, hi_ = K;
                    if (key[c] != ~0ULL) {
                        while (lo < hi_) {
                            const int mid = (lo + hi_) >> 1;
                            if (row[mid] < key[c]) lo = mid + 1;
                            else hi_ = mid;
                        }
                        if (lo < K && row[lo] == key[c]) key[c] = ~0ULL;      // already in the row
                    }
                    lt[c] = lo;
                    cand[r16 * kCandPitch + 4 * g + c] = key[c];
                }
                __syncthreads();
                u64 cs[16];
#pragma unroll
                for (int o = 0; o < 16; ++o) cs[o] = cand[r16 * kCandPitch + o];
                u64 *out = nxt + r16 * K;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (key[c] == ~0ULL) continue;
                    int rank = lt[c];
#pragma unroll
                    for (int o = 0; o < 16; ++o) rank += cs[o] < key[c] ? 1 : 0;
                    if (rank < K) out[rank] = key[c];
                }
                for (int j = g; j < K; j += 4) {
                    const u64 en = row[j];
                    int rank = j;
#pragma unroll
                    for (int o = 0; o < 16; ++o) rank += cs[o] < en ? 1 : 0;
                    if (rank < K) out[rank] = en;
                }
                __syncthreads();                  // merged rows complete before they are read again
                u64 *tmp = cur;
                cur = nxt;
                nxt = tmp;
            }
        }
        if (r16 < s)
            for (int c = g; c < K; c += 4) graph[(size_t)my_id * K + c] = cur[r16 * K + c];
    }
}

// ---------------------------------------------------------------------------------------
// The same step for any leaf size up to 64 and any dimension (the kernels above want leaves of at
// most 16 points and d % 4 == 0).  classify_any_kernel: one wave per leaf, lane r sends member r
// down the sibling subtree of every ancestor in range.  conquer_any_kernel: one wave per member
// (the waves of a block take the members of one home leaf, which owns its members' rows during
// the launch); per level the wave evaluates its member against the members of the leaf reached,
// one pair per group of sixteen lanes in the library's fixed order, and merges by rank in LDS.
__global__ void __launch_bounds__(kBlock)
classify_any_kernel(const float *__restrict__ X, int d, const int *__restrict__ perm_t,
                    const int *__restrict__ leaf_off_t, int n_leaves,
                    const efanna_node *__restrict__ nodes_t, const int *__restrict__ leaf_up_t, int dep,
                    int levels, int *__restrict__ etab)
{
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE;
    const int last = n_leaves - 1;
    const int n_waves = gridDim.x * (kBlock / EF_WAVE);
    for (int leaf = blockIdx.x * (kBlock / EF_WAVE) + wave; leaf < n_leaves; leaf += n_waves) {
        const int b0 = leaf_off_t[leaf];
        const int s = min(leaf_off_t[leaf + 1] - b0, EF_WAVE);
        if (lane >= s) continue;
        const int my_id = perm_t[b0 + lane];
        int up = min(leaf_up_t[leaf], 2 * last + 1);
        for (int k = 0; k < levels; ++k) {
            int e = -1;
            if (up >= 0) {
                const int j = up >> 1;
                const efanna_node anc = nodes_t[j];
                if (anc.depth >= dep) {
                    int c = anc.child[1 - (up & 1)];
                    for (int steps = 0; c >= 0 && steps < 4096; ++steps) {      // (bounded: foreign tables cannot hold it)
                        const efanna_node nd = nodes_t[min(c, last)];
                        const float *xi = X + (size_t)my_id * d;
                        const bool left = !ef_has_test(nd.dim) ||
                                          (long long)nd.cnt * ef_node_value([&](int j) { return xi[j]; }, d, nd.dim) < nd.sum;
                        c = nd.child[left ? 0 : 1];
                    }
                    e = c >= 0 ? 0 : min(~c, last);
                    const int pj = min(anc.parent, last);
                    up = pj < 0 ? -1 : pj * 2 + (j > pj ? 1 : 0);
                } else {
                    up = -1;
                }
            }
            etab[(size_t)(b0 + lane) * levels + k] = e;
        }
    }
}

__global__ void __launch_bounds__(kBlock)
conquer_any_kernel(const float *__restrict__ X, int d, const int *__restrict__ perm_t,
                   const int *__restrict__ leaf_off_t, int n_leaves, const int *__restrict__ etab,
                   int levels, int K, u64 *graph)
{
    extern __shared__ __align__(16) float smem[];
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE, n_waves = kBlock / EF_WAVE;
    const int grp = lane >> 4, gl = lane & 15;
    u64 *row_a = (u64 *)smem + (size_t)wave * (2 * K + EF_WAVE);      // [K] the row being merged, ascending
    u64 *row_b = row_a + K;                                           // [K] the other copy
    u64 *cand = row_b + K;                                            // [64] candidates of the level in hand
    auto wave_sync = [&]() {      // one wave: its LDS operations complete in program order
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    for (int leaf = blockIdx.x; leaf < n_leaves; leaf += gridDim.x) {
        const int b0 = leaf_off_t[leaf];
        const int s = min(leaf_off_t[leaf + 1] - b0, EF_WAVE);
        for (int r = wave; r < s; r += n_waves) {
            if (levels < 1 || etab[(size_t)(b0 + r) * levels] < 0) continue;      // nothing above this leaf to visit
            const int my_id = perm_t[b0 + r];
            const float *xa = X + (size_t)my_id * d;
            u64 *cur = row_a, *nxt = row_b;
            wave_sync();
            for (int c = lane; c < K; c += EF_WAVE) cur[c] = graph[(size_t)my_id * K + c];
            for (int k = 0; k < levels; ++k) {
                const int e = etab[(size_t)(b0 + r) * levels + k];
                if (e < 0) break;      // the ancestors in range are the first ones
                const int bb = leaf_off_t[min(e, n_leaves - 1)];
                const int sb = min(leaf_off_t[min(e, n_leaves - 1) + 1] - bb, EF_WAVE);
                // ---- distances to the members of the leaf reached, four pairs at a time -----------
                for (int j0 = 0; j0 < sb; j0 += 4) {
                    const int j = min(j0 + grp, sb - 1);      // (whole groups stay busy)
                    const int id_b = perm_t[bb + j];
                    const float *xb = X + (size_t)id_b * d;
                    float acc = 0.0f;
                    for (int t = gl; t < d; t += 16) {
                        const float diff = xa[t] - xb[t];
                        acc = __builtin_fmaf(diff, diff, acc);
                    }
                    acc = ef_group_reduce16(acc);
                    if (gl == 0 && j0 + grp < sb) cand[j0 + grp] = id_b != my_id ? ef_pack(acc, id_b, 1) : ~0ULL;
                }
                wave_sync();
                // ---- merge by rank: K old entries and sb candidates, the K smallest stay ------------
                u64 key = ~0ULL;
                int below = 0;      // old entries below the candidate
                if (lane < sb) {
                    key = cand[lane];
                    int lo = 0, hi = K;
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (cur[mid] < key) lo = mid + 1;
                        else hi = mid;
                    }
                    if (lo < K && cur[lo] == key) key = ~0ULL;      // already in the row
                    below = lo;
                }
                wave_sync();
                cand[lane] = key;      // (dropped candidates become the largest key: they count for nobody)
                wave_sync();
                if (key != ~0ULL) {
                    int rank = below;
                    for (int o = 0; o < sb; ++o) rank += cand[o] < key ? 1 : 0;
                    if (rank < K) nxt[rank] = key;
                }
                for (int c = lane; c < K; c += EF_WAVE) {
                    const u64 en = cur[c];
                    int rank = c;
                    for (int o = 0; o < sb; ++o) rank += cand[o] < en ? 1 : 0;
                    if (rank < K) nxt[rank] = en;
                }
                wave_sync();
                u64 *tmp = cur;
                cur = nxt;
                nxt = tmp;
            }
            for (int c = lane; c < K; c += EF_WAVE) graph[(size_t)my_id * K + c] = cur[c];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 step 1+2: sample the new / old sets of every row, clear the sampled marks,
// refresh the row's threshold and enter the row's id into the reverse lists of the
// sampled neighbours.
//
// A row is handled by a group of G lanes holding E entries each (G*E >= K); ranks among
// the marked and the unmarked entries come from broadcasting every entry to the group.
//
// Reverse lists keep the L members with the smallest (hash, source) key.  Most lists
// never overflow, so the first L arrivals of a list just take the next free slot (one
// counter bump); later arrivals are parked in an overflow queue and settled by
// reverse_overflow_kernel, after this kernel has finished, with the bounded insertion.
// Whatever the arrival order, a list ends up with the L smallest keys offered to it.

struct Overflow {
    u64 key;      // hash << 32 | source
    int target;   // list owner
    int which;    // 0: reverse-new, 1: reverse-old
};

// Parked keys go to kOvfQueues dense queues, block b of the sampling kernels to queue
// b % kOvfQueues: a wave bumps its queue's counter once for all the keys it parks (bumps of one
// address serialise, so the counters are many and a cache line apart), and
// reverse_overflow_kernel gets one thread per parked key instead of a sweep over all rows.
// A row parks at most K keys, so a queue holds at most (blocks per queue) x (rows per block) x K.

__host__ __device__ inline int sample_group_for(int K) { return K <= 16 ? 16 : (K <= 32 ? 32 : 64); }

__host__ __device__ inline size_t ovf_region_for(int64_t n, int K)
{
    const int G = sample_group_for(K);
    const size_t blocks = ((size_t)n * G + kBlock - 1) / kBlock;
    return (blocks + kOvfQueues - 1) / kOvfQueues * (size_t)(kBlock / G) * K;
}

// All lanes of the wave call this together; lanes with `parked` set file `o`.
__device__ inline void park_keys(bool parked, const Overflow &o, Overflow *overflow, size_t region,
                                 int *ovf_count)
{
    const u64 mask = __ballot(parked);
    if (mask == 0) return;
    const int q = blockIdx.x % kOvfQueues, leader = __ffsll((unsigned long long)mask) - 1;
    int base = 0;
    if (ef_lane() == leader) base = atomicAdd(ovf_count + q * kOvfCounterPitch, __popcll(mask));
    base = __shfl(base, leader, EF_WAVE);
    if (parked) overflow[(size_t)q * region + base + lanes_below(mask)] = o;
}

// Offer `key` to reverse list v.  Returns true if the list had no free slot: the caller
// parks the key for reverse_overflow_kernel.  Every offer bumps the list's counter, full or
// not: a read beforehand to spare full lists the bump costs more transactions than it saves
// (bumps of one counter serialise at about 11 ns each, so a point that is the neighbour of
// c others costs c * 11 ns at worst).
__device__ inline bool reverse_offer(u64 *lists, int *counts, int L, int v, u64 key)
{
    const int pos = atomicAdd(&counts[v], 1);
    if (pos >= L) return true;
    lists[(size_t)v * L + pos] = key;
    return false;
}

// Entry gl + h * G of row i for lane gl of the row's group (the largest key where there is none).
template <int G, int E>
__device__ inline void sample_load(const u64 *graph, int i, bool row_ok, int K, u64 (&e)[E])
{
    const int gl = threadIdx.x & (G - 1);
#pragma unroll
    for (int h = 0; h < E; ++h) {
        const int slot = gl + h * G;
        e[h] = row_ok && slot < K ? graph[(size_t)i * K + slot] : ~0ULL;
    }
}

// The sampling of row i by its group of G lanes, which hold the row's entries e as sample_load
// delivers them (all lanes of the wave call this together, rows past the end with row_ok false).
// offer(take, id): called by every lane once per entry it holds; lanes with `take` set offer
// row i to the reverse-new list of point id.
template <int G, int E, class Offer>
__device__ inline void sample_row(u64 *graph, const u64 (&e)[E], int i, bool row_ok, int K, int L,
                                  int *__restrict__ nw, int *__restrict__ od, int *__restrict__ nw_c,
                                  int *__restrict__ od_c, u32 *worst, Offer &&offer)
{
    const int gl = threadIdx.x & (G - 1);
    int rn[E], ro[E];
    const bool all_sampled = K <= L;
    if (all_sampled) {
        // Rows no longer than the sample: every marked entry is sampled and every other entry is
        // old, whatever their ranks.  The two lists are sets (their order decides nothing), so
        // the places in them are handed out by compaction: a ballot instead of K broadcasts.
        const int lane = ef_lane();
        const u64 group = (G == 64 ? ~0ULL : ((1ULL << (G & 63)) - 1)) << (lane & ~(G - 1));
        const u64 below = group & ((1ULL << lane) - 1);
        int base_n = 0, base_o = 0;
#pragma unroll
        for (int h = 0; h < E; ++h) {
            const bool valid = gl + h * G < K;
            const u64 bn = __ballot(valid && (e[h] & 1)) & group;
            const u64 bo = __ballot(valid && !(e[h] & 1) && !ef_is_empty(e[h])) & group;
            rn[h] = base_n + __popcll(bn & below);
            ro[h] = base_o + __popcll(bo & below);
            base_n += __popcll(bn);
            base_o += __popcll(bo);
        }
    } else {
        // ranks among new-marked and among old entries (all lanes of the group take part)
#pragma unroll
        for (int h = 0; h < E; ++h) rn[h] = ro[h] = 0;
#pragma unroll
        for (int part = 0; part < E; ++part) {
            const int k_end = min(K - part * G, G);
            for (int k = 0; k < k_end; ++k) {
                const u64 o = __shfl(e[part], k, G);
                const bool o_new = o & 1, o_old = !o_new && !ef_is_empty(o);
#pragma unroll
                for (int h = 0; h < E; ++h) {
                    const bool less = o < e[h];
                    rn[h] += (less && o_new) ? 1 : 0;
                    ro[h] += (less && o_old) ? 1 : 0;
                }
            }
        }
    }
    bool is_new[E], is_old[E], take_new[E];
    int total_new = 0;
    u32 wbits = 0;
    u64 stop = ~0ULL;      // key of the L-th new entry, if there is one
#pragma unroll
    for (int h = 0; h < E; ++h) {
        const bool valid = gl + h * G < K;
        is_new[h] = valid && (e[h] & 1);
        is_old[h] = valid && !(e[h] & 1) && !ef_is_empty(e[h]);
        take_new[h] = is_new[h] && rn[h] < L;
        total_new += is_new[h] ? 1 : 0;
        if (valid) wbits = max(wbits, ef_dist_bits(e[h]));
        if (!all_sampled && take_new[h] && rn[h] == L - 1) stop = e[h];
    }
    for (int m = G / 2; m >= 1; m >>= 1) {
        total_new += __shfl_xor(total_new, m, G);
        wbits = max(wbits, (u32)__shfl_xor((int)wbits, m, G));
        const u64 other = __shfl_xor(stop, m, G);
        stop = other < stop ? other : stop;
    }
    // sampled new entries lose their mark, go to the new list and are offered to the reverse-new
    // list of the neighbour; old entries only go to the old list here (reverse_old_kernel offers
    // them once it is known which points take part in a join at all)
    int n_old = 0;
#pragma unroll
    for (int h = 0; h < E; ++h) {
        const int slot = gl + h * G;
        const int id = ef_id(e[h]);
        if (row_ok && is_old[h] && e[h] < stop) {
            od[(size_t)i * K + ro[h]] = id;
            ++n_old;
        }
        const bool take = row_ok && take_new[h];
        if (take) {
            nw[(size_t)i * L + rn[h]] = id;
            graph[(size_t)i * K + slot] = e[h] & ~1ULL;
        }
        offer(take, id);
    }
    for (int m = G / 2; m >= 1; m >>= 1) n_old += __shfl_xor(n_old, m, G);
    if (!row_ok) return;
    // unused tails of both lists read as -1, so the join needs no counts to parse them
    const int n_new = min(total_new, L);
    for (int s = n_new + gl; s < L; s += G) nw[(size_t)i * L + s] = -1;
    for (int s = n_old + gl; s < K; s += G) od[(size_t)i * K + s] = -1;
    if (gl == 0) {
        nw_c[i] = n_new;
        od_c[i] = n_old;
        worst[i] = wbits;
    }
}

// The key under which `source` competes for a place in a reverse list of `target`.
__device__ inline u64 reverse_key(u64 stream_key, int target, int source)
{
    return (ef_mix64(stream_key + (((u64)(u32)target << 32) | (u32)source)) >> 32 << 32) | (u32)source;
}

template <int G, int E>
__global__ void __launch_bounds__(kBlock)
sample_kernel(u64 *graph, int n, int K, int L, u64 key_new, int *__restrict__ nw,
              int *__restrict__ od, int *__restrict__ nw_c, int *__restrict__ od_c, u64 *rnew,
              int *rnew_c, Overflow *overflow, size_t ovf_region, int *ovf_count, u32 *worst)
{
    const int i = (int)(((size_t)blockIdx.x * kBlock + threadIdx.x) / G);
    u64 e[E];
    sample_load<G, E>(graph, i, i < n, K, e);
    sample_row<G, E>(graph, e, i, i < n, K, L, nw, od, nw_c, od_c, worst, [&](bool take, int id) {
        bool parked = false;
        u64 hk = 0;
        if (take) {
            hk = reverse_key(key_new, id, i);
            parked = reverse_offer(rnew, rnew_c, L, id, hk);
        }
        park_keys(parked, Overflow{hk, id, 0}, overflow, ovf_region, ovf_count);
    });
}

// Bit i of `active` says whether point i has a non-empty U_new (a sampled new neighbour or a
// reverse-new member), i.e. whether it joins anything in this iteration.  One bit per point:
// the map of a million points is 128 KB and stays in L2 for the random look-ups that follow.
__global__ void __launch_bounds__(kBlock)
active_kernel(const int *__restrict__ nw_c, const int *__restrict__ rnew_c, int n, u64 *__restrict__ active)
{
    const int i = blockIdx.x * kBlock + threadIdx.x;
    const u64 mask = __ballot(i < n && (nw_c[i] > 0 || rnew_c[i] > 0));
    if (ef_lane() == 0 && (i & ~(EF_WAVE - 1)) < n) active[i / EF_WAVE] = mask;
}

// Reverse-old lists, after sampling: row i offers itself to the reverse-old list of each of its
// sampled old neighbours -- but only to those that join something; the list of a point whose
// U_new is empty is never read (Alg. 4 pairs U_old only with U_new), so it stays empty.
// One lane per slot of the old list, a group of G lanes per row as in sample_kernel; parked keys
// go behind the ones sample_kernel parked for the row.
template <int G>
__global__ void __launch_bounds__(kBlock)
reverse_old_kernel(const int *__restrict__ od, int n, int K, int L, u64 key_old,
                   const u64 *__restrict__ active, u64 *rold, int *rold_c, Overflow *overflow,
                   size_t ovf_region, int *ovf_count)
{
    const int gl = threadIdx.x & (G - 1);
    const int i = (int)(((size_t)blockIdx.x * kBlock + threadIdx.x) / G);
    const bool row_ok = i < n;
    for (int s0 = 0; s0 < K; s0 += G) {
        const int slot = s0 + gl;
        const int id = row_ok && slot < K ? od[(size_t)i * K + slot] : -1;
        bool parked = false;
        u64 hk = 0;
        if (id >= 0 && ((active[id / EF_WAVE] >> (id % EF_WAVE)) & 1)) {
            hk = reverse_key(key_old, id, i);
            parked = reverse_offer(rold, rold_c, L, id, hk);
        }
        park_keys(parked, Overflow{hk, id, 1}, overflow, ovf_region, ovf_count);
    }
}

// One thread per parked key (queue blockIdx.y, blocks of a queue stride over its keys).
// list_max[which][v] is an upper bound of the largest key of (full) list v, lowered after
// every successful insertion: the many keys offered to a popular point are turned away after
// one read instead of a scan of the list.
constexpr int kOvfBlocksPerQueue = 16;

// WIDE: lists of fifty keys or more are read fifty keys at a time.
template <bool WIDE>
__global__ void __launch_bounds__(kBlock)
reverse_overflow_kernel(const Overflow *__restrict__ overflow, size_t ovf_region,
                        const int *__restrict__ ovf_count, size_t n, u64 *rnew, u64 *rold,
                        u64 *list_max, int L)
{
    const int q = blockIdx.y, parked = ovf_count[q * kOvfCounterPitch];
    for (int e = blockIdx.x * kBlock + threadIdx.x; e < parked; e += kOvfBlocksPerQueue * kBlock) {
        const Overflow ov = overflow[(size_t)q * ovf_region + e];
        u64 *bound = list_max + (size_t)ov.which * n + ov.target;
        if (ov.key >= ef_load_coherent(bound)) continue;
        u64 nm;
        if (ef_bounded_insert_t<WIDE, true>((ov.which ? rold : rnew) + (size_t)ov.target * L, L, ov.key, 0, &nm))
            atomicMin(bound, nm);
    }
}

// ---------------------------------------------------------------------------------------
// Reverse lists without device-wide atomics, for short rows and lists (K, L <= 32) of at most
// 2^21 points (2^20 if L > 16).  A counter bump per offer is bound by the rate of atomics on random addresses;
// here the offers are sorted by target range instead, and the lists of a range are built in LDS:
//   1. an offer block (1024 threads) handles kBktRows consecutive source rows, keeps their
//      offers (one word: target << 10 | source row inside the block) in LDS, counts them per
//      bucket (a range of 1024 targets, of 512 if L > 16: the lists of a range have to fit the
//      LDS), and writes them to its own part of the offer array, bucket after bucket;
//      table[bucket][block] = start << 16 | count of that run;
//   2. a list block (one per bucket) walks the runs of its bucket, one thread per offer, and
//      enters every key into the target's list in LDS with the bounded insertion; lists and
//      counts (filled slots) go out in one contiguous piece.
// Whatever the order of the offers, a list ends up with the L smallest keys offered to it.

constexpr int kBktRows = 1024;        // source rows per offer block
constexpr int kBktThreads = 1024;
constexpr int kBktMaxRuns = 2 * kBktThreads;    // buckets and offer blocks a block-wide scan of two per thread takes
static_assert(kBktRows == 1024, "an offer word keeps the source row in ten bits");

// log2 of the targets per bucket
__host__ __device__ inline int bucket_shift(int L) { return L <= 16 ? 10 : 9; }

__host__ __device__ inline size_t bucket_lists_lds(int L, int n_blocks);

__host__ __device__ inline bool bucketed_lists(int64_t n, int K, int L)
{
    if (K > 32 || L > 32 || n > (1 << 21)) return false;      // (targets fit 21 bits of an offer word)
    const int64_t n_blocks = (n + kBktRows - 1) / kBktRows, n_buckets = ((n - 1) >> bucket_shift(L)) + 1;
    return n_blocks <= kBktMaxRuns && n_buckets <= kBktMaxRuns &&
           bucket_lists_lds(L, (int)n_blocks) <= 160 * 1024 - 256;
}

// All lanes of the wave call this together; lanes with `take` set append `offer`.
__device__ inline void offer_append(bool take, u32 offer, int shift, u32 *offers, int *hist, int *fill)
{
    const u64 mask = __ballot(take);
    if (mask == 0) return;
    const int leader = __ffsll((unsigned long long)mask) - 1;
    int base = 0;
    if (ef_lane() == leader) base = atomicAdd(fill, __popcll(mask));
    base = __shfl(base, leader, EF_WAVE);
    if (take) {
        offers[base + lanes_below(mask)] = offer;
        atomicAdd(&hist[offer >> (10 + shift)], 1);
    }
}

// End of an offer block: runs per bucket in `out` (this block's part of the offer array) and
// the block's column of the table.  hist, cursor: [n_buckets] in LDS, n_buckets <= kBktMaxRuns.
__device__ inline void offers_flush(const u32 *offers, const int *hist, int *cursor, int n_buckets, int shift,
                                    int total, u32 *__restrict__ out, u32 *__restrict__ table)
{
    __shared__ int wave_tot[kBktThreads / EF_WAVE];
    const int t = threadIdx.x, b0 = 2 * t;
    const int c0 = b0 < n_buckets ? hist[b0] : 0, c1 = b0 + 1 < n_buckets ? hist[b0 + 1] : 0;
    const int incl = ef_wave_scan_i32(c0 + c1);
    if (ef_lane() == EF_WAVE - 1) wave_tot[t / EF_WAVE] = incl;
    __syncthreads();
    int off = incl - (c0 + c1);
    for (int v = 0; v < t / EF_WAVE; ++v) off += wave_tot[v];
    if (b0 < n_buckets) {
        cursor[b0] = off;
        table[(size_t)b0 * gridDim.x + blockIdx.x] = (u32)off << 16 | (u32)c0;
    }
    if (b0 + 1 < n_buckets) {
        cursor[b0 + 1] = off + c0;
        table[(size_t)(b0 + 1) * gridDim.x + blockIdx.x] = (u32)(off + c0) << 16 | (u32)c1;
    }
    __syncthreads();
    for (int e = t; e < total; e += kBktThreads) {
        const u32 o = offers[e];
        out[atomicAdd(&cursor[o >> (10 + shift)], 1)] = o;
    }
}

// Alg. 4 step 1+2 for short rows: sample_row for kBktRows rows, the reverse-new offers to the
// block's runs.  LDS: offers [kBktRows * L] words, hist and cursor [n_buckets] int each.
// E: entries per lane of a row's eight lanes (8 E >= K).
template <int E>
__global__ void __launch_bounds__(kBktThreads)
sample_bucket_kernel(u64 *graph, int n, int K, int L, int *__restrict__ nw, int *__restrict__ od,
                     int *__restrict__ nw_c, int *__restrict__ od_c, u32 *worst, int n_buckets, int shift,
                     u32 *__restrict__ offer_runs, u32 *__restrict__ table)
{
    extern __shared__ __align__(16) u32 offer_sm[];
    u32 *offers = offer_sm;
    int *hist = (int *)(offers + (size_t)kBktRows * L), *cursor = hist + n_buckets;
    __shared__ int fill;
    for (int b = threadIdx.x; b < n_buckets; b += kBktThreads) hist[b] = 0;
    if (threadIdx.x == 0) fill = 0;
    __syncthreads();
    // (loading the entries of several of a thread's rows ahead of time gains nothing measurable,
    // and beyond 64 registers the second block of a CU is lost)
    // eight lanes with two entries each per row: a wave ranks eight rows with the broadcasts that
    // four rows of sixteen lanes would take (147 -> 93 us on the headline; four or two lanes
    // per row: the same again)
    constexpr int G = 8, kRowsPerPass = kBktThreads / G;
    for (int pass = 0; pass < kBktRows / kRowsPerPass; ++pass) {
        const int i = blockIdx.x * kBktRows + pass * kRowsPerPass + (int)(threadIdx.x / G);
        u64 e[E];
        sample_load<G, E>(graph, i, i < n, K, e);
        sample_row<G, E>(graph, e, i, i < n, K, L, nw, od, nw_c, od_c, worst, [&](bool take, int id) {
            // (an id outside the data, from a graph the library did not write, is not offered:
            // it would index the bucket counters out of bounds)
            offer_append(take && (unsigned)id < (unsigned)n, ((u32)id << 10) | (u32)(i & (kBktRows - 1)), shift, offers,
                         hist, &fill);
        });
    }
    __syncthreads();
    offers_flush(offers, hist, cursor, n_buckets, shift, fill, offer_runs + (size_t)blockIdx.x * kBktRows * L, table);
}

// Reverse-old offers of kBktRows rows (to points that join something, as in reverse_old_kernel).
// LDS: offers [kBktRows * K] words, hist and cursor [n_buckets] int each.
__global__ void __launch_bounds__(kBktThreads)
reverse_old_bucket_kernel(const int *__restrict__ od, int n, int K, const u64 *__restrict__ active,
                          int n_buckets, int shift, u32 *__restrict__ offer_runs, u32 *__restrict__ table)
{
    extern __shared__ __align__(16) u32 offer_sm[];
    u32 *offers = offer_sm;
    int *hist = (int *)(offers + (size_t)kBktRows * K), *cursor = hist + n_buckets;
    __shared__ int fill;
    for (int b = threadIdx.x; b < n_buckets; b += kBktThreads) hist[b] = 0;
    if (threadIdx.x == 0) fill = 0;
    __syncthreads();
    const int first = blockIdx.x * kBktRows, rows_here = min(kBktRows, n - first);
    for (int f0 = 0; f0 < rows_here * K; f0 += kBktThreads) {      // all threads take every round
        const int f = f0 + (int)threadIdx.x;
        const int id = f < rows_here * K ? od[(size_t)first * K + f] : -1;
        const bool take = id >= 0 && id < n && ((active[id / EF_WAVE] >> (id % EF_WAVE)) & 1);
        offer_append(take, ((u32)id << 10) | (u32)(f / K), shift, offers, hist, &fill);
    }
    __syncthreads();
    offers_flush(offers, hist, cursor, n_buckets, shift, fill, offer_runs + (size_t)blockIdx.x * kBktRows * K, table);
}

// The lists of one bucket.  run_cap: offers per part of an offer block (kBktRows * L or * K).
// Every key goes through the bounded insertion; all slots start as the largest key, so a list
// fills from slot 0 up and then keeps its L smallest keys.
// LDS: lists [bucket's targets * L] u64, scan [n_blocks + 1] and start [n_blocks] int;
// n_blocks <= kBktMaxRuns.
// What the time is made of (headline workload, 82 us per launch on average, 170 us for the
// ten million offers of the first iteration): 18 us fixed, about 5 ns per thousand offers to
// find and load them, the rest the insertions; by the counters the SIMDs issue an instruction
// in 70 to 85 % of their clocks (500 to 600 instructions per 64 offers), the LDS is active a third
// of the time.  Variants that were no faster or slower: a thread walking consecutive offers
// instead of a search per offer; offers loaded eight ahead; list reads issued in groups; the
// first L offers of a list placed by a counter and the others entered behind a per-list bound,
// or smallest first in rounds between barriers; a per-list bound on the hash in front of the
// scan; offers to popular points thinned out by a hash threshold first; the keys sorted by
// target in LDS (count, prefix sum, scatter) and one thread per target selecting its L smallest
// alone, without atomics (175 us: the popular points' threads run long, and the offers are
// found twice).
__host__ __device__ inline size_t bucket_lists_lds(int L, int n_blocks)
{
    return ((size_t)L << bucket_shift(L)) * 8 + ((size_t)2 * n_blocks + 2) * 4;
}

template <int SHIFT, int LT>      // log2 of the bucket's targets; the list length if fixed at compile time, else 0
__global__ void __launch_bounds__(kBktThreads)
bucket_lists_kernel(const u32 *__restrict__ offer_runs, const u32 *__restrict__ table, int n_blocks,
                    int run_cap, u64 stream_key, int n, int L_, u32 *__restrict__ lists,
                    int *__restrict__ counts)
{
    const int L = LT ? LT : L_;
    extern __shared__ __align__(16) u64 list_sm[];
    u64 *ll = list_sm;
    constexpr int targets = 1 << SHIFT;
    int *scan = (int *)(ll + (size_t)targets * L), *start = scan + n_blocks + 1;
    __shared__ int wave_tot[kBktThreads / EF_WAVE];
    const int t = threadIdx.x, first = blockIdx.x * targets, rows_here = min(targets, n - first);
    for (int f = t; f < targets * L; f += kBktThreads) ll[f] = ~0ULL;
    const u32 *runs = table + (size_t)blockIdx.x * n_blocks;
    {
        const int k0 = 2 * t;
        const u32 r0 = k0 < n_blocks ? runs[k0] : 0u, r1 = k0 + 1 < n_blocks ? runs[k0 + 1] : 0u;
        const int c0 = (int)(r0 & 0xffffu), c1 = (int)(r1 & 0xffffu);
        const int incl = ef_wave_scan_i32(c0 + c1);
        if (ef_lane() == EF_WAVE - 1) wave_tot[t / EF_WAVE] = incl;
        __syncthreads();
        int off = incl - (c0 + c1);
        for (int v = 0; v < t / EF_WAVE; ++v) off += wave_tot[v];
        if (k0 < n_blocks) {
            scan[k0] = off;
            start[k0] = (int)(r0 >> 16);
        }
        if (k0 + 1 < n_blocks) {
            scan[k0 + 1] = off + c0;
            start[k0 + 1] = (int)(r1 >> 16);
        }
        if (t == kBktThreads - 1) scan[n_blocks] = off + c0 + c1;      // everything before it, and its own
    }
    __syncthreads();
    const int total = scan[n_blocks];
    for (int j = t; j < total; j += kBktThreads) {      // neighbouring threads take neighbouring offers
        int lo = 0, hi = n_blocks;      // scan[lo] <= j < scan[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (scan[mid] <= j) lo = mid;
            else hi = mid;
        }
        const u32 o = offer_runs[(size_t)lo * run_cap + start[lo] + (j - scan[lo])];
        const int target = (int)(o >> 10), source = lo * kBktRows + (int)(o & (kBktRows - 1));
        const int row = target - first;
        if ((unsigned)row >= (unsigned)rows_here) continue;      // cannot happen: runs are filed by bucket
        const u64 key = reverse_key(stream_key, target, source);
        unsigned long long *list = (unsigned long long *)(ll + row * L);
        for (;;) {
            u64 mx = 0;
            int ms = 0;
            for (int a = 0; a < L; ++a) {
                const u64 v = __hip_atomic_load(list + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (v > mx) {      // the first of equal (empty) slots: lists fill from slot 0 up
                    mx = v;
                    ms = a;
                }
            }
            if (key >= mx) break;
            // slots only ever fall: if slot ms still holds mx, it still is the largest
            if (atomicCAS(list + ms, (unsigned long long)mx, (unsigned long long)key) == mx) break;
        }
    }
    __syncthreads();
    // only the sources are wanted from here on (the keys decided who is in the list)
    for (int f = t; f < rows_here * L; f += kBktThreads) lists[(size_t)first * L + f] = (u32)ll[f];
    if (t < rows_here) {
        int c = 0;
        for (int a = 0; a < L; ++a) c += ll[t * L + a] != ~0ULL ? 1 : 0;
        counts[first + t] = c;
    }
}

// Work lists by the number of vectors a join gathers: list c takes the joins of at most
// bound[c] vectors that no earlier list takes (bounds ascending; a bound of 0: no such list).
// Lists 0 and 1 are the register-operand joins (16 and 32 vectors), the others the size classes
// of the LDS-row join: a launch per class with a row buffer of that size, so that small joins
// do not occupy the LDS of the largest one and several blocks fit a CU.
struct JoinClasses {
    int n;
    int bound[kMaxClasses];
};

// the size classes for joins of up to max_rows vectors; reg_ok: lists 0 and 1 are in use
inline JoinClasses join_classes(int max_rows, bool reg_ok)
{
    JoinClasses jc;
    jc.n = 2;
    jc.bound[0] = reg_ok ? 16 : 0;
    jc.bound[1] = reg_ok ? 32 : 0;
    for (int c : {48, 64, 96, 128, 160})
        if (c < max_rows && c > jc.bound[1]) jc.bound[jc.n++] = c;
    jc.bound[jc.n++] = max_rows;
    for (int c = jc.n; c < kMaxClasses; ++c) jc.bound[c] = 0;
    return jc;
}

// After sampling and the reverse lists: one thread per point merges its four id lists
// into U_new ++ U_old (Alg. 4: G_new U G_rnew, G_old U G_rold), without duplicates and
// with everything already in U_new left out of U_old, and files the point under one of
// the work lists by the number of vectors its join gathers.
// Points with an empty U_new are dropped.  A thread compares only what can collide:
// ids inside one sampled list are distinct, and so are the sources inside one reverse
// list.  ulist: [n][cap] (written through LDS so that the stores coalesce), ucount: [n]
// (m_new, m); work: [jc.n][n], work_count: [kMaxClasses].
template <bool IDS32>      // reverse lists hold 32-bit sources (bucket scheme), not 64-bit keys
__global__ void prepare_kernel(const int *__restrict__ nw, const int *__restrict__ od,
                               const int *__restrict__ nw_c, const int *__restrict__ od_c,
                               const u64 *__restrict__ rnew, const u64 *__restrict__ rold,
                               const int *__restrict__ rnew_c, const int *__restrict__ rold_c,
                               int n, int K, int L, int cap, u32 cap_magic, JoinClasses jc,
                               int *__restrict__ ulist, int2 *__restrict__ ucount,
                               int *__restrict__ work, int *__restrict__ work_count,
                               long long *__restrict__ part)
{
    extern __shared__ int ids_sh[];
    const int pitch = cap | 1;                      // odd: threads hit different banks
    int *mine = ids_sh + threadIdx.x * pitch;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    int cls = -1, m = 0;
    int evals = 0, rows = 0;      // this point's share of the iteration's work counters
    if (i < n) {
        const int c_new = nw_c[i];
        int c_old = od_c[i];
        const int rn = min(rnew_c[i], L), ro = min(rold_c[i], L);
        if (c_new + rn == 0) c_old = 0;      // empty U_new: no join, nothing to list
        for (int a = 0; a < c_new; ++a) mine[m++] = nw[(size_t)i * L + a];
        for (int a = 0; a < rn; ++a) {
            const int id = IDS32 ? (int)((const u32 *)rnew)[(size_t)i * L + a] : (int)(u32)rnew[(size_t)i * L + a];
            bool dup = false;
            for (int k = 0; k < c_new; ++k) dup |= mine[k] == id;
            if (!dup) mine[m++] = id;
        }
        const int m_new = m;
        for (int a = 0; a < c_old; ++a) {
            const int id = od[(size_t)i * K + a];
            bool dup = false;
            for (int k = c_new; k < m_new; ++k) dup |= mine[k] == id;      // only reverse-new can collide
            if (!dup) mine[m++] = id;
        }
        const int m_mid = m;
        for (int a = 0; a < ro; ++a) {
            const int id = IDS32 ? (int)((const u32 *)rold)[(size_t)i * L + a] : (int)(u32)rold[(size_t)i * L + a];
            bool dup = false;
            for (int k = 0; k < m_mid; ++k) dup |= mine[k] == id;
            if (!dup) mine[m++] = id;
        }
        ucount[i] = make_int2(m_new, m);
        if (m_new >= 1 && m >= 2) {
            cls = 0;
            while (cls < jc.n - 1 && m > jc.bound[cls]) ++cls;
            evals = m_new * (m_new - 1) / 2 + m_new * (m - m_new);
            rows = m;
        }
    }
    for (int k = m; k < cap; ++k) mine[k] = -1;
    __syncthreads();
    // coalesced write-out of the block's lists
    const int first = blockIdx.x * blockDim.x, rows_here = min((int)blockDim.x, n - first);
    for (int f = threadIdx.x; f < rows_here * cap; f += blockDim.x) {
        const int r = (int)(((u64)(u32)f * cap_magic) >> 32), c = f - r * cap;
        ulist[(size_t)first * cap + f] = ids_sh[r * pitch + c];
    }
    // append to the work lists: ranks inside the block first, then one counter bump per
    // list and block (bumps of one address serialise at about 11 ns each)
    __shared__ int wave_cnt[kMaxClasses][kBlock / EF_WAVE], block_base[kMaxClasses];
    __shared__ int wave_sum[3][kBlock / EF_WAVE];
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE, n_waves = blockDim.x / EF_WAVE;
    int rank = 0;
    for (int c = 0; c < jc.n; ++c) {
        const u64 mask = __ballot(cls == c);
        if (cls == c) rank = __popcll(mask & ((1ULL << lane) - 1));
        if (lane == 0) wave_cnt[c][wave] = __popcll(mask);
    }
    // the block's share of the counters: pairs evaluated, vectors gathered, vectors gathered by
    // joins of at most rows0 vectors (a block's totals fit 32 bits)
    const int s_ev = ef_wave_sum_i32(evals), s_rw = ef_wave_sum_i32(rows),
              s_r0 = ef_wave_sum_i32(cls == 0 ? rows : 0);
    if (lane == 0) {
        wave_sum[0][wave] = s_ev;
        wave_sum[1][wave] = s_rw;
        wave_sum[2][wave] = s_r0;
    }
    __syncthreads();
    if ((int)threadIdx.x < jc.n) {
        int tot = 0;
        for (int v = 0; v < n_waves; ++v) tot += wave_cnt[threadIdx.x][v];
        block_base[threadIdx.x] = tot ? atomicAdd(&work_count[threadIdx.x], tot) : 0;
    }
    if (threadIdx.x < 3) {
        long long sum = 0;
        for (int v = 0; v < n_waves; ++v) sum += wave_sum[threadIdx.x][v];
        part[(size_t)blockIdx.x * 3 + threadIdx.x] = sum;
    }
    __syncthreads();
    if (cls >= 0) {
        int off = block_base[cls] + rank;
        for (int v = 0; v < wave; ++v) off += wave_cnt[cls][v];
        work[(size_t)cls * n + off] = i;
    }
}

// ---------------------------------------------------------------------------------------
// Alg. 4 step 3+4: local joins.
//
// Each block walks a work list (grid-strided), one point at a time:
//   0. candidates: the four id lists are merged and de-duplicated through a small LDS
//      hash table into U_new ++ U_old;
//   1. gather: their rows, thresholds and squared norms go to LDS;
//   2. filter: 16x16 blocks of the Gram matrix U_new x U are formed with fp32 MFMA
//      (v_mfma_f32_16x16x4f32); a pair survives if |a|^2 + |b|^2 - 2ab, lowered by a
//      bound on the rounding error of that expression, is not above the larger of
//      the two rows' thresholds.  The bound is conservative, so no pair that the exact
//      test would accept is dropped; most pairs are, at a quarter of the VALU cost;
//   3. survivors get the library's fixed-order distance (one 16-lane group per pair),
//      the exact threshold test, and go to the proposal queue;
//   4. the queue is drained into the graph rows with the lock-free insertion.
// cap_rows: how many vectors the LDS row buffer of this launch holds.

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));

// Eight coordinates of a vector, times a power of two, as half-precision numbers rounded towards
// zero: an operand of the 16x16x32 matrix instruction.  Both operands of a Gram block are packed
// the same way, so the order of the coordinates inside the operand does not matter.
template <bool SCALED>
__device__ inline f16x8 ef_pack_f16(const float4 &lo, const float4 &hi, float s)
{
    union {
        fp16x2 h[4];
        f16x8 v;
    } u;
    if (SCALED) {
        u.h[0] = __builtin_amdgcn_cvt_pkrtz(lo.x * s, lo.y * s);
        u.h[1] = __builtin_amdgcn_cvt_pkrtz(lo.z * s, lo.w * s);
        u.h[2] = __builtin_amdgcn_cvt_pkrtz(hi.x * s, hi.y * s);
        u.h[3] = __builtin_amdgcn_cvt_pkrtz(hi.z * s, hi.w * s);
    } else {
        u.h[0] = __builtin_amdgcn_cvt_pkrtz(lo.x, lo.y);
        u.h[1] = __builtin_amdgcn_cvt_pkrtz(lo.z, lo.w);
        u.h[2] = __builtin_amdgcn_cvt_pkrtz(hi.x, hi.y);
        u.h[3] = __builtin_amdgcn_cvt_pkrtz(hi.z, hi.w);
    }
    return u.v;
}

struct JoinLds {
    float *rows;      // [cap_rows][stride], columns d..dpad-1 zero
    int *uid;         // [cap_rows] U_new ++ U_old
    u32 *thr;         // [cap_rows] threshold bits
    float *nrm;       // [cap_rows] squared norms (float32, any order: filter only)
    int *meta;        // [2] updates [3] queue count [4] survivor count
    u32 *surv;        // [s_cap] a | b << 16
    u32 *known;       // [cap_rows][known_words(cap_rows)] bit c of row r: uid[c] is (or was) in the graph row of uid[r]
    int *hkey, *hidx; // [known_slots(cap_rows)] each: open-addressing table id -> place in uid
    Proposal *queue;  // [q_cap]
};

// words per row of the `known` bit table, slots of the id table (a power of two, at most half full)
__host__ __device__ inline int known_words(int cap_rows) { return (cap_rows + 31) >> 5; }
__host__ __device__ inline int known_slots(int cap_rows)
{
    int s = 64;
    while (s < 2 * cap_rows) s <<= 1;
    return s;
}

__host__ __device__ inline size_t join_lds_floats(int cap_rows, int stride, int s_cap)
{
    return (size_t)align4(cap_rows * stride) + align4(3 * cap_rows) + 8 + align4(s_cap) +
           align4(cap_rows * known_words(cap_rows)) + 2 * known_slots(cap_rows);
}

__device__ inline JoinLds join_lds_carve(float *smem, int cap_rows, int stride, int s_cap)
{
    JoinLds l;
    l.rows = smem;
    l.uid = (int *)(smem + align4(cap_rows * stride));
    l.thr = (u32 *)(l.uid + cap_rows);
    l.nrm = (float *)(l.thr + cap_rows);
    l.meta = l.uid + align4(3 * cap_rows);
    l.surv = (u32 *)(l.meta + 8);
    l.known = l.surv + align4(s_cap);
    l.hkey = (int *)(l.known + align4(cap_rows * known_words(cap_rows)));
    l.hidx = l.hkey + known_slots(cap_rows);
    l.queue = (Proposal *)(l.hidx + known_slots(cap_rows));
    return l;
}

template <bool WIDE>      // WIDE: graph rows of fifty entries or more are read fifty entries at a time
__global__ void __launch_bounds__(512) join_kernel(const float *__restrict__ X, const float *__restrict__ norms, int d,
                            int dpad, int stride, u32 q4_magic, int K, u32 k_magic,
                            const int *__restrict__ work, const int *__restrict__ work_count,
                            int cap_rows, int s_cap, int q_cap, float margin_rel, float thr_scale,
                            const int *__restrict__ ulist, const int2 *__restrict__ ucount,
                            int ucap, u64 *graph, u32 *worst, int *__restrict__ upd_block, int mode)
{
    extern __shared__ __align__(16) float smem[];
    const JoinLds lds = join_lds_carve(smem, cap_rows, stride, s_cap);
    const int mark = mode != 2;      // (modes: see join_reg_kernel)
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & (EF_WAVE - 1), wave = tid / EF_WAVE, n_waves = nthr / EF_WAVE;
    const int grp = tid >> 4, gl = tid & 15, n_grp = nthr >> 4;
    const int count = *work_count;
    const int kw = known_words(cap_rows), hslots = known_slots(cap_rows), hshift = 32 - (31 - __clz(hslots));
    int block_updates = 0;      // thread 0: insertions made by this block
    for (int w = blockIdx.x; w < count; w += gridDim.x) {
        const int i = work[w];
        // ---- 0. the point's U_new ++ U_old ------------------------------------------------
        const int2 mc = ucount[i];
        const int m_new = mc.x, m = mc.y;
        for (int r = tid; r < m; r += nthr) lds.uid[r] = ulist[(size_t)i * ucap + r];
        if (tid < 8) lds.meta[tid] = 0;
        for (int f = tid; f < m * kw; f += nthr) lds.known[f] = 0u;
        for (int f = tid; f < hslots; f += nthr) lds.hkey[f] = -1;
        __syncthreads();
        // ---- 1. gather -------------------------------------------------------------------
        for (int r = tid; r < m; r += nthr) {
            const int id = lds.uid[r];
            lds.thr[r] = ef_load_coherent(worst + id);
            lds.nrm[r] = norms[id];
            // the members' places by id (ids of a list are distinct: every one finds a free slot)
            int h = (int)(((u32)id * 0x9E3779B1u) >> hshift);
            while (atomicCAS(&lds.hkey[h], -1, id) != -1) h = (h + 1) & (hslots - 1);
            lds.hidx[h] = r;
        }
        gather_rows(X, d, stride, q4_magic, lds.uid, m, lds.rows, tid, nthr);
        __syncthreads();      // the id table is complete
        // Which members already know which: the graph rows of all members are read once (plain
        // loads: a row as it was some time ago will do) and every entry that is itself a member
        // sets a bit.  An entry that is or ever was in a row never needs to be offered to that row
        // again (rows only improve: what has left a row cannot come back), so such pairs are
        // neither evaluated exactly nor queued; with rows of a hundred entries they are nearly all
        // of the pairs inside the thresholds, and each would otherwise cost a scan of the row.
        for (int f0 = tid; f0 < m * K; f0 += 8 * nthr) {      // eight entries in flight per thread
            u64 en[8];
            int rr[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int f = f0 + q * nthr;
                rr[q] = K == 1 ? min(f, m * K - 1) : (int)(((u64)(u32)min(f, m * K - 1) * k_magic) >> 32);
                en[q] = f < m * K ? graph[(size_t)lds.uid[rr[q]] * K + (f - rr[q] * K)] : ~0ULL;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (ef_is_empty(en[q])) continue;
                const int id = ef_id(en[q]);
                int h = (int)(((u32)id * 0x9E3779B1u) >> hshift);
                for (int k = lds.hkey[h]; k != -1; k = lds.hkey[h]) {
                    if (k == id) {
                        const int c = lds.hidx[h];
                        atomicOr(&lds.known[rr[q] * kw + (c >> 5)], 1u << (c & 31));
                        break;
                    }
                    h = (h + 1) & (hslots - 1);
                }
            }
        }
        if (dpad > d)
            for (int f = tid; f < m * (dpad - d); f += nthr) {
                const int r = f / (dpad - d), c = f - r * (dpad - d);
                lds.rows[r * stride + d + c] = 0.0f;
            }
        __syncthreads();
        // ---- 2..4: blocks of 16x16 pairs, in rounds of one block per wave -----------------
        const int nbr = (m_new + 15) >> 4, nbc = (m + 15) >> 4;
        const int n_blocks = nbr * nbc - nbr * (nbr - 1) / 2;     // block row <= block column
        int updates = 0;
        for (int q0 = 0; q0 < n_blocks; q0 += n_waves) {
            const int q = q0 + wave;
            if (q < n_blocks) {
                int bi = 0, rem = q;
                while (rem >= nbc - bi) {
                    rem -= nbc - bi;
                    ++bi;
                }
                const int bj = bi + rem;
                const int r16 = lane & 15, g = lane >> 4;
                const float *pa = lds.rows + min(16 * bi + r16, m - 1) * stride + 4 * g;
                const float *pb = lds.rows + min(16 * bj + r16, m - 1) * stride + 4 * g;
                floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
                for (int c = 0; c < dpad; c += 16) {
                    const float4 va = *reinterpret_cast<const float4 *>(pa + c);
                    const float4 vb = *reinterpret_cast<const float4 *>(pb + c);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(va.x, vb.x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(va.y, vb.y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(va.z, vb.z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(va.w, vb.w, acc1, 0, 0, 0);
                }
                // lane holds G[a = 16 bi + 4 g + k][b = 16 bj + r16], k = 0..3
                const int b = 16 * bj + r16;
                const float nb = lds.nrm[min(b, m - 1)];
                const float tb = __uint_as_float(lds.thr[min(b, m - 1)]);
                // what row b already knows of rows 16 bi .. 16 bi + 15 (one half of a word)
                const u32 known_b = lds.known[min(b, m - 1) * kw + (bi >> 1)] >> (16 * (bi & 1));
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int a = 16 * bi + 4 * g + k;
                    if (a < b && a < m_new && b < m && (mode == 0 || (mode == 1) == (b < m_new))) {
                        const float na = lds.nrm[a];
                        const float ta = __uint_as_float(lds.thr[a]);
                        const float sum = na + nb;
                        const float low = sum - 2.0f * (acc0[k] + acc1[k]) - margin_rel * sum;
                        // the pair is wanted by a row that may still accept it and does not know it yet
                        const bool for_a = low <= ta * thr_scale && !((lds.known[a * kw + (b >> 5)] >> (b & 31)) & 1u);
                        const bool for_b = low <= tb * thr_scale && !((known_b >> (4 * g + k)) & 1u);
                        if (for_a || for_b) lds.surv[atomicAdd(&lds.meta[4], 1)] = (u32)a | ((u32)b << 16);
                    }
                }
            }
            __syncthreads();
            const int n_surv = lds.meta[4];
            const bool last = q0 + n_waves >= n_blocks;
            if (last || n_surv + 256 * n_waves > s_cap) {
                // ---- 3. exact distances of the survivors, one 16-lane group per pair,
                //         in chunks whose proposals (two per pair at most) fit the queue -------
                for (int c0 = 0; c0 < n_surv; c0 += q_cap / 2) {
                    const int c1 = min(n_surv, c0 + q_cap / 2);
                    for (int p0 = c0; p0 < c1; p0 += n_grp) {
                        const int p = min(p0 + grp, c1 - 1);      // keep whole groups busy
                        const u32 ab = lds.surv[p];
                        const int a = ab & 0xFFFF, b = ab >> 16;
                        const float *ra = lds.rows + a * stride, *rb = lds.rows + b * stride;
                        float acc = 0.0f;
                        for (int j = gl; j < dpad; j += 16) {      // padding columns are 0 in both rows
                            const float diff = ra[j] - rb[j];
                            acc = __builtin_fmaf(diff, diff, acc);
                        }
                        const float dist = ef_group_reduce16(acc);
                        if (gl == 0 && p0 + grp < c1) {
                            const u32 db = __float_as_uint(dist);
                            if (db <= lds.thr[a] && !((lds.known[a * kw + (b >> 5)] >> (b & 31)) & 1u)) {
                                const int slot = atomicAdd(&lds.meta[3], 1);
                                lds.queue[slot].key = ef_pack(dist, lds.uid[b], mark);
                                lds.queue[slot].target = lds.uid[a];
                            }
                            if (db <= lds.thr[b] && !((lds.known[b * kw + (a >> 5)] >> (a & 31)) & 1u)) {
                                const int slot = atomicAdd(&lds.meta[3], 1);
                                lds.queue[slot].key = ef_pack(dist, lds.uid[a], mark);
                                lds.queue[slot].target = lds.uid[b];
                            }
                        }
                    }
                    __syncthreads();
                    // ---- 4. drain -----------------------------------------------------------
                    updates += WIDE && (K & 1) == 0 && ((uintptr_t)graph & 15) == 0
                                   ? drain_queue_g16(lds.queue, lds.meta[3], graph, worst, K, tid, nthr)
                                   : drain_queue<WIDE>(lds.queue, lds.meta[3], graph, worst, K, tid, nthr);
                    __syncthreads();
                    if (tid == 0) lds.meta[3] = 0;
                    __syncthreads();
                }
                if (tid == 0) lds.meta[4] = 0;
                __syncthreads();
            }
        }
        if (updates) atomicAdd(&lds.meta[2], updates);
        __syncthreads();
        if (tid == 0) block_updates += lds.meta[2];
        __syncthreads();
    }
    if (tid == 0) upd_block[blockIdx.x] += block_updates;      // (zeroed once per iteration; passes add up)
}

// ---------------------------------------------------------------------------------------
// The same for long lists (some hundred ids per point): a thread per point would compare every
// id with every other and leaves room for a wave or three per CU next to its lists.  Here a
// wave takes a point: the four lists are read 64 ids at a time, an id is new to the join if
// its insertion into a hash table in LDS (open addressing, cleared per point) finds it absent,
// and a ballot gives the fresh ids their places.  A block of four waves takes 256 consecutive
// points per round and appends them to the work lists together (one counter bump per list and
// round).  Same lists as prepare_kernel up to the order of the ids inside U_new and U_old,
// which nothing depends on.  part: one triple per block.
template <bool IDS32>
__global__ void __launch_bounds__(kBlock)
prepare_wave_kernel(const int *__restrict__ nw, const int *__restrict__ od,
                    const int *__restrict__ nw_c, const int *__restrict__ od_c,
                    const u64 *__restrict__ rnew, const u64 *__restrict__ rold,
                    const int *__restrict__ rnew_c, const int *__restrict__ rold_c,
                    int n, int K, int L, int cap, int hash_slots, JoinClasses jc,
                    int *__restrict__ ulist, int2 *__restrict__ ucount,
                    int *__restrict__ work, int *__restrict__ work_count,
                    long long *__restrict__ part)
{
    extern __shared__ int prep_sh[];
    constexpr int n_waves = kBlock / EF_WAVE;
    const int lane = ef_lane(), wave = threadIdx.x / EF_WAVE;
    int *hash = prep_sh + wave * (hash_slots + cap + EF_WAVE);      // [hash_slots]
    int *out = hash + hash_slots;                                  // [cap]
    int *cls_of = out + cap;                                       // [64] class of each point of the round
    __shared__ int wave_cnt[kMaxClasses][n_waves], block_base[kMaxClasses];
    __shared__ long long wave_sum[3][n_waves];
    const int hshift = 32 - (31 - __clz(hash_slots));
    auto wave_sync = [&]() {      // one wave: its LDS operations complete in program order
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    long long evals = 0, rows = 0, rows0 = 0;      // lane 0: this wave's share of the iteration's work counters
    for (int i0 = blockIdx.x * kBlock; i0 < n; i0 += gridDim.x * kBlock) {      // (uniform over the block)
        const int w0 = i0 + wave * EF_WAVE;
        for (int p = 0; p < EF_WAVE; ++p) {
            const int i = w0 + p;
            if (i >= n) break;
            const int c_new = nw_c[i], rn = min(rnew_c[i], L);
            int m = 0, m_new = 0, cls = -1;
            if (c_new + rn > 0) {
                const int c_old = od_c[i], ro = min(rold_c[i], L);
                for (int f = lane; f < hash_slots; f += EF_WAVE) hash[f] = -1;
                wave_sync();
                auto add = [&](int id, bool have) {      // all lanes call; have: this lane offers id
                    bool fresh = false;
                    if (have) {
                        int h = (int)(((u32)id * 0x9E3779B1u) >> hshift);
                        for (;;) {
                            const int prev = atomicCAS(&hash[h], -1, id);
                            if (prev == -1) {
                                fresh = true;
                                break;
                            }
                            if (prev == id) break;
                            h = (h + 1) & (hash_slots - 1);
                        }
                    }
                    const u64 mask = __ballot(fresh);
                    if (fresh) out[m + __popcll(mask & ((1ULL << lane) - 1))] = id;
                    m += __popcll(mask);
                };
                for (int a0 = 0; a0 < c_new; a0 += EF_WAVE) {
                    const int a = a0 + lane;
                    add(a < c_new ? nw[(size_t)i * L + a] : -1, a < c_new);
                }
                for (int a0 = 0; a0 < rn; a0 += EF_WAVE) {
                    const int a = a0 + lane;
                    const int id = a < rn ? (IDS32 ? (int)((const u32 *)rnew)[(size_t)i * L + a] : (int)(u32)rnew[(size_t)i * L + a]) : -1;
                    add(id, a < rn);
                }
                m_new = m;
                for (int a0 = 0; a0 < c_old; a0 += EF_WAVE) {
                    const int a = a0 + lane;
                    add(a < c_old ? od[(size_t)i * K + a] : -1, a < c_old);
                }
                for (int a0 = 0; a0 < ro; a0 += EF_WAVE) {
                    const int a = a0 + lane;
                    const int id = a < ro ? (IDS32 ? (int)((const u32 *)rold)[(size_t)i * L + a] : (int)(u32)rold[(size_t)i * L + a]) : -1;
                    add(id, a < ro);
                }
                wave_sync();
                if (m_new >= 1 && m >= 2) {
                    cls = 0;
                    while (cls < jc.n - 1 && m > jc.bound[cls]) ++cls;
                    evals += (long long)m_new * (m_new - 1) / 2 + (long long)m_new * (m - m_new);
                    rows += m;
                    if (cls == 0) rows0 += m;
                }
            }
            for (int f = lane; f < cap; f += EF_WAVE) ulist[(size_t)i * cap + f] = f < m ? out[f] : -1;
            if (lane == 0) {
                ucount[i] = make_int2(m_new, m);
                cls_of[p] = cls;
            }
            wave_sync();      // out is free for the next point
        }
        // append the round's points to the work lists
        const int mine = w0 + lane < n ? cls_of[lane] : -1;
        int rank = 0;
        for (int c = 0; c < jc.n; ++c) {
            const u64 mask = __ballot(mine == c);
            if (mine == c) rank = __popcll(mask & ((1ULL << lane) - 1));
            if (lane == 0) wave_cnt[c][wave] = __popcll(mask);
        }
        __syncthreads();
        if ((int)threadIdx.x < jc.n) {
            int tot = 0;
            for (int v = 0; v < n_waves; ++v) tot += wave_cnt[threadIdx.x][v];
            block_base[threadIdx.x] = tot ? atomicAdd(&work_count[threadIdx.x], tot) : 0;
        }
        __syncthreads();
        if (mine >= 0) {
            int off = block_base[mine] + rank;
            for (int v = 0; v < wave; ++v) off += wave_cnt[mine][v];
            work[(size_t)mine * n + off] = w0 + lane;
        }
        __syncthreads();      // wave_cnt and block_base are free for the next round
    }
    if (lane == 0) {
        wave_sum[0][wave] = evals;
        wave_sum[1][wave] = rows;
        wave_sum[2][wave] = rows0;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        long long sum = 0;
        for (int v = 0; v < n_waves; ++v) sum += wave_sum[threadIdx.x][v];
        part[(size_t)blockIdx.x * 3 + threadIdx.x] = sum;
    }
}

// ---------------------------------------------------------------------------------------
// The same local join for points whose join gathers at most 16 * NB vectors (NB = 1, 2),
// which is nearly all of them.  One wave per point and no row buffer in LDS: lane
// (r, g) = (lane % 16, lane / 16) loads 16-byte pieces of vector r (and 16 + r) straight
// from memory into the registers the MFMA reads, 128 coordinates at a time, so a block
// needs a few KB of LDS and many more waves fit a CU to hide the memory round trips.
// Survivors of the filter (few) get their exact distance from the same registers when
// the vectors fit them in one piece (ONE: d <= 128): lane (a, g) fetches the matching
// pieces of row b from lane (b, g) with cross-lane reads, accumulates the four partial
// sums it owns (coordinates = 4g..4g+3 mod 16, ascending) and the 16 partial sums are
// added in the fixed tree across the four lanes of row a.  Longer vectors are re-read
// from memory (they are still in L2) by one 16-lane group per pair.
// Requires d % 4 == 0 and a 16-byte aligned X.

// where the survivors of Gram blocks (0,0), (0,1), (1,1) start in the LDS survivor buffer
__device__ constexpr int kSurvBase[3] = {0, 120, 376};
// d > 128: up to this many surviving pairs of a Gram block (per 16 rows) are read pair by pair
constexpr int kFewPairs = 4;
// d <= 128: more survivors than this inside one set of sixteen rows and all its pairs are evaluated by row rotations
constexpr int kDenseSurvivors = 24;

// One surviving pair (rows a, b of the point's list) per lane with `mine` set: its distance is
// offered to row a and to row b where it passes their thresholds.  All lanes of the wave call
// this together; `fill` is the wave-uniform number of proposals queued, the new one is returned.
__device__ inline int propose_pair(Proposal *queue, int fill, bool mine, float dist, int a, int b,
                                   const u32 *thr, const int *uid, int mark)
{
    const u32 db = __float_as_uint(dist);
    const int ua = uid[a], ub = uid[b];
    const bool to_a = mine && db <= thr[a], to_b = mine && db <= thr[b];
    const u64 mask_a = __ballot(to_a), mask_b = __ballot(to_b);
    if (to_a) {
        Proposal &p = queue[fill + lanes_below(mask_a)];
        p.key = ef_pack(dist, ub, mark);
        p.target = ua;
    }
    fill += __popcll(mask_a);
    if (to_b) {
        Proposal &p = queue[fill + lanes_below(mask_b)];
        p.key = ef_pack(dist, ua, mark);
        p.target = ub;
    }
    return fill + __popcll(mask_b);
}

template <int NB, bool ONE, int KT>      // KT: the row length if fixed at compile time (the row scans unroll), else 0
__global__ void __launch_bounds__(EF_WAVE) __attribute__((amdgpu_waves_per_eu(NB > 1 ? 3 : 4)))
join_reg_kernel(const float *__restrict__ X, int d, int K_,
                const int *__restrict__ work, const int *__restrict__ work_count, int q_cap,
                float margin_rel, float thr_scale, float u_rel, float rho0, const int *__restrict__ ulist,
                const int2 *__restrict__ ucount, int ucap, u64 *graph, u32 *worst,
                int *__restrict__ upd_block, int mode, int dense_min, const u32 *__restrict__ xmax)
{
    // mode 0: every pair of the join, fresh entries marked new.  1: only pairs of two new members.
    // 2: only pairs of a new and an old member, fresh entries marked old (the literal marking of
    // Alg. 4's second inner loop runs the joins twice, mode 1 before mode 2).  Rows 0 .. m_new - 1
    // of a list are its new members, so a pair (a, b), a < b, a new, is of two new members iff b is.
    const int mark = mode != 2;
    const int K = KT ? KT : K_;
    constexpr int R = 16 * NB;                    // rows
    constexpr int S_CAP = R * (R - 1) / 2 + 8;    // every pair may survive
    extern __shared__ __align__(16) float smem[];
    int *uid = (int *)smem;                       // [R]
    u32 *thr = (u32 *)(uid + R);                  // [R] threshold bits (exact test)
    float *nf = (float *)(thr + R);               // [R] |x|^2 (1 - margin)   } the filter's
    float *tf = nf + R;                           // [R] threshold * scale    } operands (in the
    float *sq = tf + R;                           // [R] its square root      } scaled units of
    float *rr = sq + R;                           // [R] rounding radius      } the operands)
    u32 *surv = (u32 *)(rr + R);                  // [S_CAP] surviving pairs
    Proposal *queue = (Proposal *)(surv + align4(S_CAP));   // [q_cap]
    const int lane = threadIdx.x, r16 = lane & 15, g = lane >> 4, gl = r16, grp = g;
    const int dirn = (EF_ROW_ROR(r16, 1) - r16) & 15;      // a rotation by t brings row r + t * dirn to row r
    const int count = *work_count;
    // The filter works on the vectors times a power of two that brings the largest coordinate of
    // the data below 2^15 (1 for all data below that already): half precision then never overflows.
    const int x_exp = (int)(*xmax >> 23) - 127;
    const float scale = x_exp >= 15 ? __uint_as_float((u32)(127 + 14 - x_exp) << 23) : 1.0f;
    const float t_scale = thr_scale * scale * scale;
    // The id list and the sizes of a point are fetched one point ahead, and the thresholds of
    // its vectors as soon as those ids are there, so that they travel while the point before
    // is being worked on: the row loads are the only latency a point waits for.
    // (Thresholds only ever fall: one that is a point old lets a few more pairs through the
    // filter, nothing else.)
    int w = blockIdx.x;
    int i = w < count ? work[w] : -1;
    int u_pre = i >= 0 && lane < R ? ulist[(size_t)i * ucap + min(lane, ucap - 1)] : -1;
    int2 c_pre = i >= 0 ? ucount[i] : make_int2(0, 0);
    int i_next = w + (int)gridDim.x < count ? work[w + gridDim.x] : -1;
    u32 t_pre = u_pre >= 0 ? worst[u_pre] : 0u;
    // Proposals wait in the queue across points and are applied when about half of it is
    // full (and at the end): late iterations accept well under one proposal per point, and
    // a drain costs two memory round trips whatever its size.
    // The block is one wave: the fill of the queue and of the survivor lists are wave-uniform
    // registers, and a lane finds its slot from a ballot (no LDS counters, no round trips).
    int updates = 0, q_fill = 0;
    auto drain = [&](const Proposal *from, int cnt) {
        return drain_queue<false, NB == 1>(from, cnt, graph, worst, K, lane, EF_WAVE);
    };
    auto drain_mid = drain;
    for (; i >= 0; w += gridDim.x) {
        // ---- 0. the point's U_new ++ U_old (the loop ends with a barrier: LDS is free) -------
        const int m_new = c_pre.x, m = c_pre.y;
        auto mode_ok = [&](int b) { return mode == 0 || (mode == 1) == (b < m_new); };      // b: the pair's larger row
        const int u_cur = u_pre;
        if (lane < R) {
            uid[lane] = u_cur;
            thr[lane] = t_pre;
            const float t = __uint_as_float(t_pre) * t_scale;
            tf[lane] = t;
            sq[lane] = __builtin_sqrtf(t) * 1.000001f;
        }
        i = i_next;
        u_pre = i >= 0 && lane < R ? ulist[(size_t)i * ucap + min(lane, ucap - 1)] : -1;
        c_pre = i >= 0 ? ucount[i] : make_int2(0, 0);
        i_next = w + 2 * (int)gridDim.x < count ? work[w + 2 * gridDim.x] : -1;
        // ---- 1+2. Gram blocks from register operands ---------------------------------------
        const float *pa = X + (size_t)__shfl(u_cur, min(r16, m - 1), EF_WAVE) * d + 4 * g;
        const float *pb = NB > 1 ? X + (size_t)__shfl(u_cur, min(16 + r16, m - 1), EF_WAVE) * d + 4 * g : pa;
        const bool need11 = NB > 1 && m_new > 16;      // block (1,1) only if new rows reach it
        constexpr int NQ = NB > 1 ? 3 : 1;      // Gram blocks (0,0), (0,1), (1,1)
        floatx4 acc[NQ][2];
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h) acc[q][h] = (floatx4){0.f, 0.f, 0.f, 0.f};
        float4 va[8], vb[NB > 1 ? 8 : 1];
        // Long vectors (d > 128): with the filter the rows would have to be streamed again for the
        // pairs that pass it, once per 128 of them.  Instead every pair gets its fixed-order
        // distance straight away, as in init_reg_kernel: row rotations per 128-coordinate piece
        // meet the pairs (vector instructions that hide under the gather: 512 per 8 KB of rows),
        // the four lanes of a column add their partial sums in the fixed tree, and lane (r, g)
        // holds the distances from row r to the rows 2g+1 and 2g+2 places on.  No Gram block, no
        // filter.  At most 16 rows: one pass, eight rotations.  17..32 rows: a first pass for the
        // pairs inside rows 0..15 and inside rows 16..31, a second one for rows 0..15 against
        // rotations 0..15 of rows 16..31.
        constexpr bool rotated = !ONE;
        float two[2] = {0.f, 0.f}, two_b[2] = {0.f, 0.f};
        if (rotated) {
            float P[8][4], PB[NB > 1 ? 8 : 1][4];
#pragma unroll
            for (int t = 0; t < 8; ++t) P[t][0] = P[t][1] = P[t][2] = P[t][3] = 0.0f;
            if (NB > 1) {
#pragma unroll
                for (int t = 0; t < 8; ++t) PB[NB > 1 ? t : 0][0] = PB[NB > 1 ? t : 0][1] = PB[NB > 1 ? t : 0][2] = PB[NB > 1 ? t : 0][3] = 0.0f;
            }
            for (int c0 = 0; c0 < d; c0 += 128) {
                const int n_pieces = min(8, (d - c0 + 15) >> 4);
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bool in = c0 + 16 * s + 4 * g + 3 < d;      // d % 4 == 0: a piece is in or out
                    va[s] = in ? *reinterpret_cast<const float4 *>(pa + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
                init_round<1>(va, n_pieces, P[0]);
                init_round<2>(va, n_pieces, P[1]);
                init_round<3>(va, n_pieces, P[2]);
                init_round<4>(va, n_pieces, P[3]);
                init_round<5>(va, n_pieces, P[4]);
                init_round<6>(va, n_pieces, P[5]);
                init_round<7>(va, n_pieces, P[6]);
                init_round<8>(va, n_pieces, P[7]);
                if (NB > 1 && need11) {      // pairs inside rows 16..31 are wanted only if new rows reach them
                    float4 (&wb)[8] = reinterpret_cast<float4 (&)[8]>(vb);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const bool in = c0 + 16 * s + 4 * g + 3 < d;
                        wb[s] = in ? *reinterpret_cast<const float4 *>(pb + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                    init_round<1>(wb, n_pieces, PB[0]);
                    init_round<2>(wb, n_pieces, PB[NB > 1 ? 1 : 0]);
                    init_round<3>(wb, n_pieces, PB[NB > 1 ? 2 : 0]);
                    init_round<4>(wb, n_pieces, PB[NB > 1 ? 3 : 0]);
                    init_round<5>(wb, n_pieces, PB[NB > 1 ? 4 : 0]);
                    init_round<6>(wb, n_pieces, PB[NB > 1 ? 5 : 0]);
                    init_round<7>(wb, n_pieces, PB[NB > 1 ? 6 : 0]);
                    init_round<8>(wb, n_pieces, PB[NB > 1 ? 7 : 0]);
                }
            }
            reduce_rotations(P, g, two);
            if (NB > 1) reduce_rotations(reinterpret_cast<const float (&)[8][4]>(PB), g, two_b);
        }
        for (int c0 = 0; c0 < d && !rotated; c0 += 128) {
            if (c0 + 128 <= d) {     // a whole 128-coordinate piece: no per-load bounds test
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    va[s] = *reinterpret_cast<const float4 *>(pa + c0 + 16 * s);
                    if (NB > 1) vb[NB > 1 ? s : 0] = *reinterpret_cast<const float4 *>(pb + c0 + 16 * s);
                }
            } else {
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const int j = c0 + 16 * s + 4 * g;
                    const bool in = j + 3 < d;                 // d % 4 == 0: a piece is in or out
                    va[s] = in ? *reinterpret_cast<const float4 *>(pa + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                    if (NB > 1)
                        vb[NB > 1 ? s : 0] = in ? *reinterpret_cast<const float4 *>(pb + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            auto gram = [&](auto scaled) {
#pragma unroll
                for (int s = 0; s < 8; s += 2) {
                    if (c0 + 16 * s >= d) break;      // (pieces beyond d were loaded as zeros)
                    const f16x8 oa = ef_pack_f16<decltype(scaled)::value>(va[s], va[s + 1], scale);
                    acc[0][(s >> 1) & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(oa, oa, acc[0][(s >> 1) & 1], 0, 0, 0);
                    if (NB > 1) {
                        constexpr int Q1 = NB > 1 ? 1 : 0, Q2 = NB > 1 ? 2 : 0;
                        const f16x8 ob = ef_pack_f16<decltype(scaled)::value>(vb[NB > 1 ? s : 0], vb[NB > 1 ? s + 1 : 0], scale);
                        acc[Q1][(s >> 1) & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(oa, ob, acc[Q1][(s >> 1) & 1], 0, 0, 0);
                        acc[Q2][(s >> 1) & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ob, ob, acc[Q2][(s >> 1) & 1], 0, 0, 0);
                    }
                }
            };
            if (scale != 1.0f) gram(std::true_type{});
            else gram(std::false_type{});
        }
        if (!rotated) {
            // The filter's squared norms are those of the rounded vectors: the diagonals of Gram
            // blocks (0,0) and (1,1) (lane (r16, g) holds G[4 g + k][r16]).  rr: how far rounding may
            // have moved the vector, u |x'| + r0.
            if ((r16 >> 2) == g) {
                const int kd = r16 & 3;
                const float dg = kd == 0 ? acc[0][0][0] + acc[0][1][0]
                               : kd == 1 ? acc[0][0][1] + acc[0][1][1]
                               : kd == 2 ? acc[0][0][2] + acc[0][1][2] : acc[0][0][3] + acc[0][1][3];
                nf[r16] = dg * (1.0f - margin_rel);
                rr[r16] = __builtin_fmaf(u_rel, __builtin_sqrtf(dg), rho0);
                if (NB > 1) {
                    constexpr int Q2 = NB > 1 ? 2 : 0;
                    const float dh = kd == 0 ? acc[Q2][0][0] + acc[Q2][1][0]
                                   : kd == 1 ? acc[Q2][0][1] + acc[Q2][1][1]
                                   : kd == 2 ? acc[Q2][0][2] + acc[Q2][1][2] : acc[Q2][0][3] + acc[Q2][1][3];
                    nf[16 + r16] = dh * (1.0f - margin_rel);
                    rr[16 + r16] = __builtin_fmaf(u_rel, __builtin_sqrtf(dh), rho0);
                }
            }
        }
        __syncthreads();      // uid, thr, nf, tf, sq, rr visible
        t_pre = u_pre >= 0 ? worst[u_pre] : 0u;      // the next point's; its ids have arrived by now
        // ---- filter: lane holds G[a = 16 bi + 4 g + k][b = 16 bj + r16] of block q -----------
        // With D' the distance of the rounded vectors, r = rr[a] + rr[b] and T the larger threshold:
        // |D' - D| <= r, so D^2 <= T implies D'^2 <= T + r (2 sqrt(T) + r).  Pair (a, b) survives
        // unless (|a'|^2 + |b'|^2)(1 - margin) - 2 a'.b' is above that (the margin covers the three
        // accumulations; a comparison with a NaN - an infinite threshold times a zero radius -
        // keeps the pair).
        int n_surv[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) n_surv[q] = 0;
#pragma unroll
        for (int q = 0; q < (NB > 1 ? 3 : 1); ++q) {
            if (rotated) break;
            const int bi = q == 2 ? 1 : 0, bj = q == 0 ? 0 : 1;
            const int b = 16 * bj + r16, a0 = 16 * bi + 4 * g;
            // valid pairs: a < lim
            const int lim = b >= m ? 0 : mode == 0 ? min(m_new, b) : mode == 1 ? (b < m_new ? b : 0) : (b >= m_new ? m_new : 0);
            const float nfb = nf[b], tfb = tf[b], sqb = sq[b], rrb = rr[b];      // junk beyond m, masked by lim
            const float4 nfa = *reinterpret_cast<const float4 *>(nf + a0);
            const float4 tfa = *reinterpret_cast<const float4 *>(tf + a0);
            const float4 sqa = *reinterpret_cast<const float4 *>(sq + a0);
            const float4 rra = *reinterpret_cast<const float4 *>(rr + a0);
            const float nfa_k[4] = {nfa.x, nfa.y, nfa.z, nfa.w}, tfa_k[4] = {tfa.x, tfa.y, tfa.z, tfa.w};
            const float sqa_k[4] = {sqa.x, sqa.y, sqa.z, sqa.w}, rra_k[4] = {rra.x, rra.y, rra.z, rra.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float lhs = __builtin_fmaf(-2.0f, acc[q][0][k] + acc[q][1][k], nfa_k[k] + nfb);
                const float rad = rra_k[k] + rrb;
                const float rhs = __builtin_fmaf(rad, __builtin_fmaf(2.0f, fmaxf(sqa_k[k], sqb), rad), fmaxf(tfa_k[k], tfb));
                // one list per Gram block, entries are rows local to the block
                const bool keep = a0 + k < lim && !(lhs > rhs);
                const u64 kept = __ballot(keep);
                if (keep) surv[kSurvBase[q] + n_surv[q] + lanes_below(kept)] = (u32)((a0 + k) & 15) | ((u32)(b & 15) << 8);
                n_surv[q] += __popcll(kept);
            }
        }
        __syncthreads();
        if (rotated) {
            auto room = [&]() {      // a step adds at most two proposals per lane
                if (q_fill + 2 * EF_WAVE > q_cap) {
                    updates += drain_mid(queue, q_fill);
                    q_fill = 0;
                    __syncthreads();
                }
            };
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int rot = 2 * g + 1 + t, b = (r16 + dirn * rot) & 15;
                // rotation 8 meets every pair from both ends: the lower row keeps it
                const bool once = rot != 8 || r16 < b;
                room();
                q_fill = propose_pair(queue, q_fill,
                                      once && r16 < m && b < m && min(r16, b) < m_new && mode_ok(max(r16, b)), two[t],
                                      r16, b, thr, uid, mark);
                __syncthreads();
                if (NB > 1 && need11) {
                    room();
                    q_fill = propose_pair(queue, q_fill,
                                          once && 16 + r16 < m && 16 + b < m && 16 + min(r16, b) < m_new &&
                                              mode_ok(16 + max(r16, b)),
                                          two_b[t], 16 + r16, 16 + b, thr, uid, mark);
                    __syncthreads();
                }
            }
            if (NB > 1) {
                // second pass: row r of rows 0..15 against rows 16 + (r + T) of rows 16..31, T = 0..15
                float PX[2][8][4];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int t = 0; t < 8; ++t) PX[h][t][0] = PX[h][t][1] = PX[h][t][2] = PX[h][t][3] = 0.0f;
                float4 (&wb)[8] = reinterpret_cast<float4 (&)[8]>(vb);
                for (int c0 = 0; c0 < d; c0 += 128) {
                    const int n_pieces = min(8, (d - c0 + 15) >> 4);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const bool in = c0 + 16 * s + 4 * g + 3 < d;
                        va[s] = in ? *reinterpret_cast<const float4 *>(pa + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                        wb[s] = in ? *reinterpret_cast<const float4 *>(pb + c0 + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                    cross_round<0>(va, wb, n_pieces, PX[0][0]);
                    cross_round<1>(va, wb, n_pieces, PX[0][1]);
                    cross_round<2>(va, wb, n_pieces, PX[0][2]);
                    cross_round<3>(va, wb, n_pieces, PX[0][3]);
                    cross_round<4>(va, wb, n_pieces, PX[0][4]);
                    cross_round<5>(va, wb, n_pieces, PX[0][5]);
                    cross_round<6>(va, wb, n_pieces, PX[0][6]);
                    cross_round<7>(va, wb, n_pieces, PX[0][7]);
                    cross_round<8>(va, wb, n_pieces, PX[1][0]);
                    cross_round<9>(va, wb, n_pieces, PX[1][1]);
                    cross_round<10>(va, wb, n_pieces, PX[1][2]);
                    cross_round<11>(va, wb, n_pieces, PX[1][3]);
                    cross_round<12>(va, wb, n_pieces, PX[1][4]);
                    cross_round<13>(va, wb, n_pieces, PX[1][5]);
                    cross_round<14>(va, wb, n_pieces, PX[1][6]);
                    cross_round<15>(va, wb, n_pieces, PX[1][7]);
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float cross[2];
                    reduce_rotations(PX[h], g, cross);      // rotations 8h + 2g and 8h + 2g + 1
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int rot = 8 * h + 2 * g + t, b = 16 + ((r16 + dirn * rot) & 15);
                        room();
                        q_fill = propose_pair(queue, q_fill, b < m && r16 < m_new && mode_ok(b), cross[t], r16, b, thr,
                                              uid, mark);
                        __syncthreads();
                    }
                }
            }
        }
        // ---- 3a. survivors from registers, sixteen pairs per round --------------------------
        // The four lanes r16 + 16 g (g = 0..3) of column r16 take pair p0 + r16: lane g
        // fetches the pieces it needs of rows a and b from lanes a + 16 g and b + 16 g,
        // which hold the coordinates = 4g..4g+3 (mod 16) of those rows.
        if (ONE) {
#pragma unroll
            for (int q = 0; q < (NB > 1 ? 3 : 1); ++q) {
                const int bi = q == 2 ? 1 : 0, bj = q == 0 ? 0 : 1;
                const int n_q = n_surv[q];
                // Many survivors inside one set of sixteen rows (early iterations: most pairs
                // pass): all 120 pairs by row rotations, as for long vectors, cost what two rounds
                // of sixteen survivors cost.  The filter never drops a pair that would pass a
                // threshold, so which way a pair takes makes no difference to what is proposed.
                // (only with the row length compiled in: the other variants would spill registers)
                if (NB == 1 && KT != 0 && n_q > dense_min) {
                    const float4 (&rows)[8] = reinterpret_cast<const float4 (&)[8]>(*(q == 0 ? va : vb));
                    const int n_pieces = (d + 15) >> 4, base = 16 * bi;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {      // rotations 1..4, then 5..8
                        float P[4][4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) P[t][0] = P[t][1] = P[t][2] = P[t][3] = 0.0f;
                        if (half == 0) {
                            init_round<1>(rows, n_pieces, P[0]);
                            init_round<2>(rows, n_pieces, P[1]);
                            init_round<3>(rows, n_pieces, P[2]);
                            init_round<4>(rows, n_pieces, P[3]);
                        } else {
                            init_round<5>(rows, n_pieces, P[0]);
                            init_round<6>(rows, n_pieces, P[1]);
                            init_round<7>(rows, n_pieces, P[2]);
                            init_round<8>(rows, n_pieces, P[3]);
                        }
                        const float dist = reduce_rotations4(P, g);
                        const int rot = 4 * half + 1 + g, b = (r16 + dirn * rot) & 15;
                        const bool once = rot != 8 || r16 < b;      // rotation 8 meets every pair from both ends
                        if (NB > 1 && q_fill + 2 * EF_WAVE > q_cap) {
                            updates += drain_mid(queue, q_fill);
                            q_fill = 0;
                            __syncthreads();
                        }
                        q_fill = propose_pair(queue, q_fill,
                                              once && base + r16 < m && base + b < m && base + min(r16, b) < m_new &&
                                                  mode_ok(base + max(r16, b)),
                                              dist, base + r16, base + b, thr, uid, mark);
                        __syncthreads();
                    }
                    continue;
                }
                for (int p0 = 0; p0 < n_q; p0 += 16) {
                    const bool has = p0 + r16 < n_q;
                    const u32 ent = surv[kSurvBase[q] + min(p0 + r16, n_q - 1)];
                    const int al = ent & 15, bl = (ent >> 8) & 15;
                    const int src_a = al + 16 * g, src_b = bl + 16 * g;
                    float p0s = 0.f, p1s = 0.f, p2s = 0.f, p3s = 0.f;
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        if (16 * s >= d) break;
                        const float4 own = bi == 0 ? va[s] : vb[NB > 1 ? s : 0];
                        const float4 oth = bj == 0 ? va[s] : vb[NB > 1 ? s : 0];
                        const float d0 = __shfl(own.x, src_a, EF_WAVE) - __shfl(oth.x, src_b, EF_WAVE);
                        const float d1 = __shfl(own.y, src_a, EF_WAVE) - __shfl(oth.y, src_b, EF_WAVE);
                        const float d2 = __shfl(own.z, src_a, EF_WAVE) - __shfl(oth.z, src_b, EF_WAVE);
                        const float d3 = __shfl(own.w, src_a, EF_WAVE) - __shfl(oth.w, src_b, EF_WAVE);
                        p0s = __builtin_fmaf(d0, d0, p0s);
                        p1s = __builtin_fmaf(d1, d1, p1s);
                        p2s = __builtin_fmaf(d2, d2, p2s);
                        p3s = __builtin_fmaf(d3, d3, p3s);
                    }
                    // partial sum l lives in lane g = l / 4, slot l % 4: l += l+8, l += l+4 across
                    // lanes, l += l+2, l += l+1 inside lane g = 0
                    p0s += __shfl_xor(p0s, 32, EF_WAVE);
                    p1s += __shfl_xor(p1s, 32, EF_WAVE);
                    p2s += __shfl_xor(p2s, 32, EF_WAVE);
                    p3s += __shfl_xor(p3s, 32, EF_WAVE);
                    p0s += __shfl_xor(p0s, 16, EF_WAVE);
                    p1s += __shfl_xor(p1s, 16, EF_WAVE);
                    p2s += __shfl_xor(p2s, 16, EF_WAVE);
                    p3s += __shfl_xor(p3s, 16, EF_WAVE);
                    const float dist = (p0s + p2s) + (p1s + p3s);
                    q_fill = propose_pair(queue, q_fill, has && g == 0, dist, 16 * bi + al, 16 * bj + bl, thr, uid, mark);
                    __syncthreads();
                    // NB = 1: the queue is sized so that a point's proposals always fit (at most 240
                    // on top of fewer than q_cap / 2): no drain while the operands are live
                    if (NB > 1 && q_fill + 32 > q_cap) {      // a round adds at most two proposals per pair
                        updates += drain_mid(queue, q_fill);
                        q_fill = 0;
                        __syncthreads();
                    }
                }
            }
        }
        if (q_fill >= q_cap / 2) {
            // whole passes of 64 only, from the end of the queue: what is left waits for the next
            // drain (a pass costs its two round trips however few lanes it fills)
            const int rest = q_fill & (EF_WAVE - 1);
            updates += drain(queue + rest, q_fill - rest);
            q_fill = rest;
        }
        __syncthreads();
    }
    __syncthreads();
    updates += drain(queue, q_fill);
    updates = ef_wave_sum_i32(updates);
    if (lane == 0) upd_block[blockIdx.x] += updates;      // (zeroed once per iteration; passes add up)
}

// ---------------------------------------------------------------------------------------
// The local join for points whose join gathers more than 32 vectors of at most 128 coordinates
// (d % 4 == 0, X 16-byte aligned), without a row buffer: one wave per point, the vectors pass
// through registers sixteen at a time.  For every tile of sixteen new rows (A) and every tile of
// sixteen rows from it onwards (B) the wave loads both tiles as join_reg_kernel does - lane
// (r, g) the 16-byte pieces 16 s + 4 g of row r - forms their Gram block with fp32 MFMA, filters,
// and evaluates the surviving pairs exactly from the same registers.  B tiles are read once per
// A tile: the rows of a join (some tens of KB) come from the caches after the first time.  What
// a block keeps in LDS is small (ids, thresholds, the table of pairs already known, queues: a few
// KB against the tens of KB of a row buffer), its waves never wait for one another, and a dozen
// joins are in flight on a CU instead of one or two.
struct TileLds {
    int *uid;          // [cap] U_new ++ U_old
    u32 *thr;          // [cap] threshold bits (exact test)
    float *nf, *tf;    // [cap] |x|^2 (1 - margin), threshold * scale (filter)
    u32 *known;        // [cap][known_words(cap)]
    int2 *hslot;       // [tile_slots(cap)] (id, its place in uid) in buckets of two slots, id -1 = free
    u32 *surv;         // [256] surviving pairs of the tile pair in hand
    Proposal *queue;   // [q_cap]
};
// The table that maps an id to its place in the list: buckets of two slots, a quarter full at
// most, so that nearly every look-up is one 16-byte read of the id's own bucket (ten thousand
// look-ups per join: a probe loop whose length differs from lane to lane was most of a join).
// An id goes to the first free slot of its bucket, else of the buckets after it; a look-up
// therefore ends at the first bucket with a free slot.
__host__ __device__ inline int tile_slots(int cap)
{
    int s = 128;
    while (s < 4 * cap) s <<= 1;
    return s;
}
__host__ __device__ inline size_t tile_lds_bytes(int cap, int q_cap)
{
    return (size_t)(align4(cap) * 4 + align4(cap * known_words(cap)) + 2 * tile_slots(cap) + 256) * 4 +
           (size_t)q_cap * sizeof(Proposal);
}
__device__ inline TileLds tile_lds_carve(float *smem, int cap)
{
    TileLds l;
    const int c4 = align4(cap);
    l.uid = (int *)smem;
    l.thr = (u32 *)(l.uid + c4);
    l.nf = (float *)(l.thr + c4);
    l.tf = l.nf + c4;
    l.known = (u32 *)(l.tf + c4);
    l.hslot = (int2 *)(l.known + align4(cap * known_words(cap)));
    l.surv = (u32 *)(l.hslot + tile_slots(cap));
    l.queue = (Proposal *)(l.surv + 256);
    return l;
}

constexpr int kTileWaves = 3;      // waves per SIMD the tile join is compiled for (four would spill)
template <bool LONG_ROWS>      // graph rows of even length, 16-byte aligned, more than 16 entries: sixteen lanes per proposal
__global__ void __launch_bounds__(EF_WAVE) __attribute__((amdgpu_waves_per_eu(kTileWaves)))
join_tile_kernel(const float *__restrict__ X, const float *__restrict__ norms, int d, int K, u32 k_magic,
                 u32 kq_magic, int *gid, const int *__restrict__ work, const int *__restrict__ work_count, int cap, int q_cap,
                 float margin_rel, float thr_scale, const int *__restrict__ ulist,
                 const int2 *__restrict__ ucount, int ucap, u64 *graph, u32 *worst,
                 int *__restrict__ upd_block, int mode)
{
    extern __shared__ __align__(16) float smem[];
    const TileLds lds = tile_lds_carve(smem, cap);
    const int mark = mode != 2;      // (modes: see join_reg_kernel)
    const int lane = threadIdx.x, r16 = lane & 15, g = lane >> 4;
    const int kw = known_words(cap), hslots = tile_slots(cap), n_buckets = hslots >> 1;
    const int hshift = 32 - (31 - __clz(n_buckets));      // id * odd constant >> hshift: the id's bucket
    const int count = *work_count;
    const int n_pieces = (d + 15) >> 4;      // 16-coordinate pieces of a vector (at most 8)
    int updates = 0, q_fill = 0;
    auto drain = [&]() {
        updates += LONG_ROWS ? drain_queue_g16(lds.queue, q_fill, graph, worst, K, lane, EF_WAVE, gid)
                             : drain_queue<false, false>(lds.queue, q_fill, graph, worst, K, lane, EF_WAVE);
        q_fill = 0;
        __syncthreads();
    };
    // The table of known pairs is kept by column: bit r of the words of member c says that row r
    // holds (or held) c.  The lanes of a wave scan the same row or two at a time, and the ids of a
    // row are distinct: their hits then fall into different words (by row, they would all be
    // or-ed into the same few words, one after the other).
    auto is_known = [&](int row, int col) { return (lds.known[col * kw + (row >> 5)] >> (row & 31)) & 1u; };
    for (int w = blockIdx.x; w < count; w += gridDim.x) {
        const int i = work[w];
        const int2 mc = ucount[i];
        const int m_new = mc.x, m = min(mc.y, cap);
        // ---- 0. ids, thresholds, norms; the members' places by id ---------------------------
        for (int f = lane; f < m * kw; f += EF_WAVE) lds.known[f] = 0u;
        for (int f = lane; f < hslots; f += EF_WAVE) lds.hslot[f].x = -1;
        __syncthreads();
        for (int r = lane; r < m; r += EF_WAVE) {
            const int id = ulist[(size_t)i * ucap + r];
            const u32 t = ef_load_coherent(worst + id);
            lds.uid[r] = id;
            lds.thr[r] = t;
            lds.tf[r] = __uint_as_float(t) * thr_scale;
            lds.nf[r] = norms[id] * (1.0f - margin_rel);
            int h = 2 * (int)(((u32)id * 0x9E3779B1u) >> hshift);      // ids of a list are distinct: every one finds a slot
            while (atomicCAS(&lds.hslot[h].x, -1, id) != -1) h = (h + 1) & (hslots - 1);
            lds.hslot[h].y = r;
        }
        __syncthreads();
        // ---- 1. which members already know which (see join_kernel): the members' rows of ids, sixteen
        //         loads in flight per lane, four ids per load where rows allow it -----------------
        // `two`: the id's own bucket, read beforehand (several look-ups are issued together: one
        // after the other, each would wait out its own LDS round trips)
        auto note = [&](int row, int id, int4 two) {
            if (id < 0) return;
            int c = two.x == id ? two.y : (two.z == id ? two.w : -1);
            if (c < 0 && two.x != -1 && two.z != -1) {      // a full bucket without the id: it may have moved on (rare)
                int b = (int)(((u32)id * 0x9E3779B1u) >> hshift);
                do {
                    b = (b + 1) & (n_buckets - 1);
                    two = *reinterpret_cast<const int4 *>(lds.hslot + 2 * b);
                    c = two.x == id ? two.y : (two.z == id ? two.w : -1);
                } while (c < 0 && two.x != -1 && two.z != -1);
            }
            if (c >= 0) atomicOr(&lds.known[c * kw + (row >> 5)], 1u << (row & 31));
        };
        auto bucket_of = [&](int id) {      // (an id of -1 reads some bucket and is dropped afterwards)
            return *reinterpret_cast<const int4 *>(lds.hslot + 2 * (int)(((u32)id * 0x9E3779B1u) >> hshift));
        };
        if ((K & 3) == 0 && ((uintptr_t)gid & 15) == 0) {
            const int kq = K >> 2, total = m * kq;
            for (int f0 = lane; f0 < total; f0 += 16 * EF_WAVE) {
                int4 four[16];
                int rr[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int f = f0 + q * EF_WAVE;
                    rr[q] = kq == 1 ? min(f, total - 1) : (int)(((u64)(u32)min(f, total - 1) * kq_magic) >> 32);
                    four[q] = f < total ? *reinterpret_cast<const int4 *>(gid + (size_t)lds.uid[rr[q]] * K + 4 * (f - rr[q] * kq))
                                        : make_int4(-1, -1, -1, -1);
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int id4[4] = {four[q].x, four[q].y, four[q].z, four[q].w};
                    int4 bk[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) bk[t] = bucket_of(id4[t]);
#pragma unroll
                    for (int t = 0; t < 4; ++t) note(rr[q], id4[t], bk[t]);
                }
            }
        } else {
            for (int f0 = lane; f0 < m * K; f0 += 8 * EF_WAVE) {
                int one[8], rr[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int f = f0 + q * EF_WAVE;
                    rr[q] = K == 1 ? min(f, m * K - 1) : (int)(((u64)(u32)min(f, m * K - 1) * k_magic) >> 32);
                    one[q] = f < m * K ? gid[(size_t)lds.uid[rr[q]] * K + (f - rr[q] * K)] : -1;
                }
#pragma unroll
                for (int q0 = 0; q0 < 8; q0 += 4) {
                    int4 bk[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) bk[t] = bucket_of(one[q0 + t]);
#pragma unroll
                    for (int t = 0; t < 4; ++t) note(rr[q0 + t], one[q0 + t], bk[t]);
                }
            }
        }
        __syncthreads();
        // ---- 2. tile pairs ---------------------------------------------------------------------
        const int nbr = (m_new + 15) >> 4, nbc = (m + 15) >> 4;
        for (int bi = 0; bi < nbr; ++bi) {
            float4 va[8];
            {
                const float *pa = X + (size_t)lds.uid[min(16 * bi + r16, m - 1)] * d + 4 * g;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bool in = 16 * s + 4 * g + 3 < d;      // d % 4 == 0: a piece is in or out
                    va[s] = in ? *reinterpret_cast<const float4 *>(pa + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            for (int bj = bi; bj < nbc; ++bj) {
                float4 vb[8];
                if (bj == bi) {
#pragma unroll
                    for (int s = 0; s < 8; ++s) vb[s] = va[s];
                } else {
                    const float *pb = X + (size_t)lds.uid[min(16 * bj + r16, m - 1)] * d + 4 * g;
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const bool in = 16 * s + 4 * g + 3 < d;
                        vb[s] = in ? *reinterpret_cast<const float4 *>(pb + 16 * s) : make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                }
                floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    if (s >= n_pieces) break;
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(va[s].x, vb[s].x, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(va[s].y, vb[s].y, acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(va[s].z, vb[s].z, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(va[s].w, vb[s].w, acc1, 0, 0, 0);
                }
                // ---- filter: the lane holds G[a = 16 bi + 4 g + k][b = 16 bj + r16] ---------------
                const int b = 16 * bj + r16, bc = min(b, m - 1);
                const float nfb = lds.nf[bc], tfb = lds.tf[bc];
                const u32 knows_b = lds.known[bc * kw + (bi >> 1)] >> (16 * (bi & 1));      // which of rows 16 bi .. know b
                int n_surv = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int a = 16 * bi + 4 * g + k, ac = min(a, m - 1);
                    const float low = __builtin_fmaf(-2.0f, acc0[k] + acc1[k], lds.nf[ac] + nfb);
                    const bool valid = a < m_new && b < m && a < b && (mode == 0 || (mode == 1) == (b < m_new));
                    // wanted by a row that may still accept the pair and does not know it yet
                    const bool keep = valid && ((low <= lds.tf[ac] && !((knows_b >> (4 * g + k)) & 1u)) ||
                                                (low <= tfb && !is_known(bc, ac)));
                    const u64 kept = __ballot(keep);
                    if (keep) lds.surv[n_surv + lanes_below(kept)] = (u32)(4 * g + k) | ((u32)r16 << 8);
                    n_surv += __popcll(kept);
                }
                __syncthreads();
                // ---- survivors from registers, sixteen pairs per round (see join_reg_kernel) ------
                for (int p0 = 0; p0 < n_surv; p0 += 16) {
                    const bool has = p0 + r16 < n_surv;
                    const u32 ent = lds.surv[min(p0 + r16, n_surv - 1)];
                    const int al = ent & 15, bl = (ent >> 8) & 15;
                    const int src_a = al + 16 * g, src_b = bl + 16 * g;
                    float p0s = 0.f, p1s = 0.f, p2s = 0.f, p3s = 0.f;
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        if (s >= n_pieces) break;
                        const float d0 = __shfl(va[s].x, src_a, EF_WAVE) - __shfl(vb[s].x, src_b, EF_WAVE);
                        const float d1 = __shfl(va[s].y, src_a, EF_WAVE) - __shfl(vb[s].y, src_b, EF_WAVE);
                        const float d2 = __shfl(va[s].z, src_a, EF_WAVE) - __shfl(vb[s].z, src_b, EF_WAVE);
                        const float d3 = __shfl(va[s].w, src_a, EF_WAVE) - __shfl(vb[s].w, src_b, EF_WAVE);
                        p0s = __builtin_fmaf(d0, d0, p0s);
                        p1s = __builtin_fmaf(d1, d1, p1s);
                        p2s = __builtin_fmaf(d2, d2, p2s);
                        p3s = __builtin_fmaf(d3, d3, p3s);
                    }
                    p0s += __shfl_xor(p0s, 32, EF_WAVE);
                    p1s += __shfl_xor(p1s, 32, EF_WAVE);
                    p2s += __shfl_xor(p2s, 32, EF_WAVE);
                    p3s += __shfl_xor(p3s, 32, EF_WAVE);
                    p0s += __shfl_xor(p0s, 16, EF_WAVE);
                    p1s += __shfl_xor(p1s, 16, EF_WAVE);
                    p2s += __shfl_xor(p2s, 16, EF_WAVE);
                    p3s += __shfl_xor(p3s, 16, EF_WAVE);
                    const float dist = (p0s + p2s) + (p1s + p3s);
                    const int a = 16 * bi + al, bb = 16 * bj + bl;
                    const u32 db = __float_as_uint(dist);
                    const bool mine = has && g == 0;
                    const bool to_a = mine && db <= lds.thr[a] && !is_known(a, bb);
                    const bool to_b = mine && db <= lds.thr[bb] && !is_known(bb, a);
                    const u64 mask_a = __ballot(to_a), mask_b = __ballot(to_b);
                    if (to_a) {
                        Proposal &pr = lds.queue[q_fill + lanes_below(mask_a)];
                        pr.key = ef_pack(dist, lds.uid[bb], mark);
                        pr.target = lds.uid[a];
                    }
                    q_fill += __popcll(mask_a);
                    if (to_b) {
                        Proposal &pr = lds.queue[q_fill + lanes_below(mask_b)];
                        pr.key = ef_pack(dist, lds.uid[a], mark);
                        pr.target = lds.uid[bb];
                    }
                    q_fill += __popcll(mask_b);
                    __syncthreads();
                    if (q_fill + 32 > q_cap) drain();      // a round adds at most two proposals per pair
                }
                __syncthreads();      // the survivor list is free again
            }
        }
        if (q_fill >= q_cap / 2) drain();
        __syncthreads();
    }
    drain();
    updates = ef_wave_sum_i32(updates);
    if (lane == 0) upd_block[blockIdx.x] += updates;      // (zeroed once per iteration; passes add up)
}

// The ids of all graph entries (-1 for an empty slot), written once per iteration after the
// sampling: the tile join looks for pairs that already know each other in these, at half the
// bytes of the entries themselves, and notes the ids it inserts there as well.  An id that is or
// was in a row is all the table of known pairs asks for: the mirror may lag behind the rows.
__global__ void __launch_bounds__(kBlock) graph_ids_kernel(const u64 *__restrict__ graph, size_t total, int *__restrict__ gid)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (size_t)gridDim.x * kBlock) {
        const u64 e = graph[i];
        gid[i] = ef_is_empty(e) ? -1 : ef_id(e);
    }
}

// squared norms in float32 (only the join's filter uses them; any summation order will do) and
// the largest |coordinate| of the data (its bits, which order like the values; *xmax starts at 0).
// A group of sixteen lanes per point, points strided over the grid: one atomic per block.
__global__ void __launch_bounds__(kBlock)
norms_kernel(const float *__restrict__ X, int n, int d, float *__restrict__ norms, u32 *xmax)
{
    __shared__ u32 wave_max[kBlock / EF_WAVE];
    const int gl = threadIdx.x & 15;
    const size_t n_groups = (size_t)gridDim.x * (kBlock / 16);
    float mx = 0.0f;
    for (size_t g = ((size_t)blockIdx.x * kBlock + threadIdx.x) >> 4; g < (size_t)n; g += n_groups) {
        const float *a = X + g * d;
        float acc = 0.0f;
        for (int j = gl; j < d; j += 16) {
            const float v = a[j];
            acc = __builtin_fmaf(v, v, acc);
            mx = fmaxf(mx, fabsf(v));
        }
        acc = ef_group_reduce16(acc);
        if (gl == 0) norms[g] = acc;
    }
    for (int o = EF_WAVE / 2; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, EF_WAVE));
    if (ef_lane() == 0) wave_max[threadIdx.x / EF_WAVE] = __float_as_uint(mx);
    __syncthreads();
    if (threadIdx.x == 0) {
        u32 m = 0;
        for (int w = 0; w < kBlock / EF_WAVE; ++w) m = max(m, wave_max[w]);
        if (m) atomicMax(xmax, m);
    }
}

// per-iteration counters from the per-block partial sums: part[b] = (pairs evaluated, vectors
// gathered, vectors gathered by the smallest join class) of prepare block b; upd_block: insertions
// per join block
__global__ void stats_kernel(const long long *__restrict__ part, int n_part,
                             const int *__restrict__ upd_block, int n_upd_block, u64 *stats)
{
    long long ev = 0, up = 0, rw = 0, r0 = 0;
    const int t = blockIdx.x * blockDim.x + threadIdx.x, nt = gridDim.x * blockDim.x;
    for (int b = t; b < n_part; b += nt) {
        ev += part[(size_t)b * 3];
        rw += part[(size_t)b * 3 + 1];
        r0 += part[(size_t)b * 3 + 2];
    }
    for (int b = t; b < n_upd_block; b += nt) up += upd_block[b];
    ev = ef_wave_sum_i64(ev);
    up = ef_wave_sum_i64(up);
    rw = ef_wave_sum_i64(rw);
    r0 = ef_wave_sum_i64(r0);
    if (ef_lane() == 0) {
        atomicAdd(stats, (u64)ev);
        atomicAdd(stats + 1, (u64)up);
        atomicAdd(stats + 2, (u64)rw);
        atomicAdd(stats + 3, (u64)r0);
    }
}

// number of graph entries carrying the new mark (early termination)
__global__ void __launch_bounds__(kBlock) count_new_kernel(const u64 *__restrict__ graph, size_t total, u64 *out)
{
    __shared__ int wave_cnt[kBlock / EF_WAVE];
    int mine = 0;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += (size_t)gridDim.x * kBlock) {
        const u64 e = graph[i];
        mine += (e & 1) && !ef_is_empty(e) ? 1 : 0;
    }
    mine = ef_wave_sum_i32(mine);
    if (ef_lane() == 0) wave_cnt[threadIdx.x / EF_WAVE] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int w = 0; w < kBlock / EF_WAVE; ++w) tot += wave_cnt[w];
        if (tot) atomicAdd(out, (u64)tot);
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

// Rows of at most G entries: a group of G lanes per row, ranks by broadcast inside the group.
template <int G>
__global__ void __launch_bounds__(kBlock)
get_graph_group_kernel(const u64 *__restrict__ graph, int n, int K, int *__restrict__ ids,
                       float *__restrict__ dists, unsigned char *__restrict__ flags)
{
    const int gl = threadIdx.x & (G - 1);
    const size_t i = ((size_t)blockIdx.x * kBlock + threadIdx.x) / G;
    const bool mine = i < (size_t)n && gl < K;
    const u64 e = mine ? graph[i * K + gl] : ~0ULL;
    int rank = 0;
    for (int k = 0; k < K; ++k) rank += __shfl(e, k, G) < e ? 1 : 0;
    if (!mine) return;
    const size_t dst = i * K + rank;
    const bool empty = ef_is_empty(e);
    ids[dst] = empty ? -1 : ef_id(e);
    dists[dst] = empty ? __uint_as_float(EF_INF_BITS) : __uint_as_float(ef_dist_bits(e));
    if (flags) flags[dst] = empty ? 0 : (unsigned char)(e & 1);
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
    int *nw, *od, *nw_c, *od_c, *work, *work_count, *rnew_c, *rold_c, *ovf_count, *ulist, *upd_block;
    int2 *ucount;
    void *overflow;
    u64 *rnew, *rold, *list_max, *active, *fresh;
    u32 *offer_runs, *run_table;
    int *gid;      // ids of all graph entries (joins of more than 32 vectors)
    long long *part;
    u32 *worst;
    float *norms;
    u32 *xmax;      // bits of the largest |coordinate| of the data
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
    w.part = (long long *)take(((size_t)n / EF_WAVE + 1) * 3 * 8);      // prepare blocks hold >= 64 points
    const int n_lists = join_classes(K + 2 * L, true).n;      // (without the register joins there are no more lists)
    w.work = (int *)take((size_t)n * n_lists * 4);
    w.work_count = (int *)take(kMaxClasses * 4);     // list sizes
    w.rnew_c = (int *)take((size_t)n * 4);
    w.rold_c = (int *)take((size_t)n * 4);
    // reverse lists: either the overflow queues of the counter scheme or the offer runs and
    // their table of the bucket scheme
    const bool bkt = bucketed_lists(n, K, L);
    const size_t n_bkt = (size_t)(n + kBktRows - 1) / kBktRows, n_buckets = (size_t)((n - 1) >> bucket_shift(L)) + 1;
    w.overflow = take(bkt ? 0 : ovf_region_for(n, K) * kOvfQueues * sizeof(Overflow));
    w.offer_runs = (u32 *)take(bkt ? n_bkt * kBktRows * (size_t)(K > L ? K : L) * 4 : 0);
    w.run_table = (u32 *)take(bkt ? n_buckets * n_bkt * 4 : 0);
    w.ovf_count = (int *)take((size_t)kOvfQueues * kOvfCounterPitch * 4);
    w.ulist = (int *)take((size_t)n * (K + 2 * L) * 4);
    w.ucount = (int2 *)take((size_t)n * 8);
    w.upd_block = (int *)take((size_t)(2 * kRegGrid + (n_lists - 2) * kMaxLargeGrid) * 4);
    w.rnew = (u64 *)take((size_t)n * L * 8);
    w.rold = (u64 *)take((size_t)n * L * 8);
    w.list_max = (u64 *)take((size_t)n * 2 * 8);
    w.active = (u64 *)take((size_t)(n + 63) / 64 * 8);
    w.fresh = (u64 *)take(8);
    w.worst = (u32 *)take((size_t)n * 4);
    w.norms = (float *)take((size_t)n * 4);
    w.xmax = (u32 *)take(8);
    w.gid = (int *)take(K + 2 * L > 32 ? (size_t)n * K * 4 : 0);
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
    case EFANNA_ESCRATCH: return "input needs more scratch memory than the library's fixed array holds";
    default: return "unknown status";
    }
}

extern "C" size_t efanna_init_workspace_bytes(int64_t n, int32_t levels)
{
    if (n < 1) return 0;
    // one leaf index per point and visited level above the leaves
    return levels > 0 ? align_up((size_t)n * (size_t)levels * 4) : 256;
}

extern "C" int efanna_init_graph(const float *X, int64_t n, int32_t d, const int32_t *perm,
                                 const int32_t *leaf_off, int32_t max_leaves,
                                 const int32_t *n_leaves, const efanna_node *nodes,
                                 const int32_t *leaf_up, int32_t tree_depth,
                                 int32_t conquer_depth, int32_t n_trees,
                                 int32_t leaf_size, int32_t k, efanna_entry *graph_, void *ws,
                                 size_t ws_bytes, void *stream)
{
    if (!X || !perm || !leaf_off || !n_leaves || !graph_ || (!nodes) != (!leaf_up)) return EFANNA_EINVAL;
    if (nodes && conquer_depth < 0) return EFANNA_EINVAL;
    if (n < 2 || d < 1 || n_trees < 1 || n_trees > EFANNA_MAX_TREES || leaf_size < 1 ||
        leaf_size > EFANNA_MAX_LEAF || k < 1 || k > EFANNA_MAX_K || k >= n || max_leaves < 1 ||
        n >= 2147483647LL - 256)
        return EFANNA_EINVAL;
    // levels above the leaves that the conquer step visits (none without nodes)
    const int levels = nodes ? (tree_depth - conquer_depth + 1 > 64 ? 64 : tree_depth - conquer_depth + 1) : 0;
    if (nodes && tree_depth - conquer_depth + 1 > 64) return EFANNA_EUNSUPPORTED;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < efanna_init_workspace_bytes(n, levels))
        return EFANNA_EWORKSPACE;
    if (n * (int64_t)k >= 2147483647LL) return EFANNA_EINVAL;   // LDS row indices are 32-bit
    for (int t = 0; t < n_trees; ++t)
        if (n_leaves[t] < 1 || n_leaves[t] > max_leaves) return EFANNA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 *const graph = (u64 *)graph_;
    const int stride = d + kRowPad;
    const size_t lds = (size_t)(align4(leaf_size * stride) + align4(leaf_size * leaf_size)) * 4 +
                       (size_t)leaf_size * k * 8 + (size_t)leaf_size * (leaf_size + 1) * 8 +
                       (size_t)leaf_size * 8;
    // (a block per leaf and, with leaves of 64 and rows of 100, one block per CU: sixteen waves
    // of it keep the CU busy through the loads of the rows)
    const int block_threads = 4 * EF_WAVE * ((leaf_size + 15) / 16);
    const bool reg_ok = leaf_size <= 16 && d % 4 == 0 && ((uintptr_t)X & 15) == 0;
    if (leaf_size > EF_WAVE) return EFANNA_EUNSUPPORTED;
    if (reg_ok) {
        const size_t reg_lds = (size_t)16 * k * 8 + (size_t)16 * kCandPitch * 8 + 16 * 4;
        const size_t conquer_lds = (size_t)2 * 16 * k * 8 + (size_t)16 * kCandPitch * 8 + 16 * 16 * 4;
        for (int t = 0; t < n_trees; ++t) {
            const int32_t *perm_t = perm + (size_t)t * n, *off_t = leaf_off + (size_t)t * (max_leaves + 1);
            init_reg_kernel<<<min(n_leaves[t], kLeafGrid), EF_WAVE, reg_lds, st>>>(
                X, d, perm_t, off_t, n_leaves[t], k, graph, t == 0);
            if (levels > 0) {
                int *etab = (int *)ws;
                classify_kernel<<<min(grid_for((size_t)n_leaves[t], kBlock / EF_WAVE), 256 * 8), kBlock, 0, st>>>(
                    X, d, perm_t, off_t, n_leaves[t], nodes + (size_t)t * (max_leaves + 1),
                    leaf_up + (size_t)t * (max_leaves + 1), conquer_depth, levels, etab);
                conquer_kernel<<<min(n_leaves[t], kLeafGrid), EF_WAVE, conquer_lds, st>>>(
                    X, d, perm_t, off_t, n_leaves[t], etab, levels, k, graph);
            }
        }
        EF_HIP_CHECK(hipGetLastError());
        return EFANNA_OK;
    }
    if (lds > kLdsLimit) return EFANNA_EUNSUPPORTED;
    EF_HIP_CHECK(hipFuncSetAttribute((const void *)init_tree_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const size_t any_lds = (size_t)(kBlock / EF_WAVE) * (2 * k + EF_WAVE) * 8;
    for (int t = 0; t < n_trees; ++t) {
        const int32_t *perm_t = perm + (size_t)t * n, *off_t = leaf_off + (size_t)t * (max_leaves + 1);
        init_tree_kernel<<<n_leaves[t], block_threads, lds, st>>>(
            X, d, stride, q4_magic_for(d), leaf_size, perm_t, off_t, k, graph, t == 0);
        if (levels > 0) {      // above the leaves: the general kernels (any leaf size up to 64, any d)
            int *etab = (int *)ws;
            classify_any_kernel<<<min(grid_for((size_t)n_leaves[t], kBlock / EF_WAVE), 256 * 8), kBlock, 0, st>>>(
                X, d, perm_t, off_t, n_leaves[t], nodes + (size_t)t * (max_leaves + 1),
                leaf_up + (size_t)t * (max_leaves + 1), conquer_depth, levels, etab);
            conquer_any_kernel<<<min(n_leaves[t], 256 * 64), kBlock, any_lds, st>>>(
                X, d, perm_t, off_t, n_leaves[t], etab, levels, k, graph);
        }
    }
    EF_HIP_CHECK(hipGetLastError());
    return EFANNA_OK;
}

extern "C" size_t efanna_nndescent_workspace_bytes(int64_t n, int32_t k, int32_t sample_L)
{
    if (n < 1 || k < 1 || sample_L < 1) return 0;
    return carve_nnd(nullptr, n, k, sample_L).bytes;
}

namespace {

// Scratch of the entry point that allocates nothing: device memory that the code object
// brings along, one copy per GPU.  Host code never uses the array's name as an address (on
// the host it is only a handle for hipGetSymbolAddress): the address on each device is
// looked up once, with that device current, and kept.
__device__ __align__(256) unsigned char noalloc_scratch[EFANNA_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> noalloc_scratch_ptr[kMaxDevices];

// The scratch array's address on the current device (nullptr and a status on failure).
int noalloc_scratch_address(void **out)
{
    *out = nullptr;
    int dev = -1;
    EF_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return EFANNA_EUNSUPPORTED;
    void *p = noalloc_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        EF_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(noalloc_scratch)));
        if (!p) return EFANNA_EHIP;
        noalloc_scratch_ptr[dev].store(p, std::memory_order_release);      // racing callers store the same address
    }
    *out = p;
    return EFANNA_OK;
}

int nndescent_run(const float *X, int64_t n, int32_t d, int32_t k, efanna_entry *graph_, int32_t iters,
                  int32_t sample_L, uint64_t seed, int32_t first_iter, float delta, int32_t cross_old,
                  int32_t *iters_done, uint64_t *stats_, float *phase_ms, void *ws, size_t ws_bytes, void *stream);

}  // namespace

extern "C" int efanna_nndescent(const float *X, int64_t n, int32_t d, int32_t k,
                                efanna_entry *graph_, int32_t iters, int32_t sample_L,
                                uint64_t seed, int32_t first_iter, float delta, int32_t cross_old,
                                int32_t *iters_done, uint64_t *stats_, float *phase_ms, void *ws,
                                size_t ws_bytes, void *stream)
{
    return nndescent_run(X, n, d, k, graph_, iters, sample_L, seed, first_iter, delta, cross_old, iters_done,
                         stats_, phase_ms, ws, ws_bytes, stream);
}

extern "C" int efanna_nndescent_noalloc(const float *X, int64_t n, int32_t d, int32_t k,
                                        efanna_entry *graph_, int32_t iters, int32_t sample_L,
                                        uint64_t seed, int32_t first_iter, uint64_t *stats_,
                                        void *stream)
{
    if (n < 1 || k < 1 || sample_L < 1) return EFANNA_EINVAL;
    if (efanna_nndescent_workspace_bytes(n, k, sample_L) > (size_t)EFANNA_NOALLOC_SCRATCH_BYTES)
        return EFANNA_ESCRATCH;
    void *scratch = nullptr;
    const int rc = noalloc_scratch_address(&scratch);
    if (rc != EFANNA_OK) return rc;
    // no early termination (it reads a counter back after every iteration) and no phase timing
    // (it creates events): neither allocates device memory, but both make the call wait
    return nndescent_run(X, n, d, k, graph_, iters, sample_L, seed, first_iter, 0.0f, 0, nullptr, stats_,
                         nullptr, scratch, (size_t)EFANNA_NOALLOC_SCRATCH_BYTES, stream);
}

namespace {

int nndescent_run(const float *X, int64_t n, int32_t d, int32_t k, efanna_entry *graph_, int32_t iters,
                  int32_t sample_L, uint64_t seed, int32_t first_iter, float delta, int32_t cross_old,
                  int32_t *iters_done, uint64_t *stats_, float *phase_ms, void *ws, size_t ws_bytes, void *stream)
{
    if (iters_done) *iters_done = 0;
    if (!X || !graph_ || !(delta >= 0.0f)) return EFANNA_EINVAL;
    u64 *const graph = (u64 *)graph_;
    u64 *const stats = (u64 *)stats_;
    if (n < 2 || d < 1 || k < 1 || k > EFANNA_MAX_K || k >= n || iters < 0 || sample_L < 1 ||
        sample_L > EFANNA_MAX_SAMPLE || first_iter < 0 || n >= 2147483647LL - 256)
        return EFANNA_EINVAL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < efanna_nndescent_workspace_bytes(n, k, sample_L))
        return EFANNA_EWORKSPACE;
    const int K = k, L = sample_L;
    const int dpad = (d + 15) & ~15;
    const int stride = dpad + kRowPad;
    // a join gathers at most K + 2L vectors: new and old sets together come from one row
    // of K entries, each reverse list adds at most L
    const int max_rows = K + 2 * L;
    // work lists: joins of at most 16 and at most 32 vectors run from register operands (needs
    // 16-byte aligned rows), the rest through LDS row buffers, one launch per size class
    const bool reg_ok = (d & 3) == 0 && ((uintptr_t)X & 15) == 0;
    const int rows1 = reg_ok ? 32 : 0;
    const JoinClasses jc = join_classes(max_rows, reg_ok);
    const int n_upd_block = 2 * kRegGrid + (jc.n - 2) * kMaxLargeGrid;
    struct Shape {
        int cap_rows, threads, s_cap, q_cap, grid;
        size_t lds;
    };
    auto shape_for = [&](int cap_rows) {
        Shape sh;
        sh.cap_rows = cap_rows;
        const long blocks = (long)((cap_rows + 15) / 16) * ((cap_rows + 15) / 16);
        sh.threads = blocks <= 2 ? 64 : (blocks <= 9 ? 128 : (blocks <= 36 ? 256 : 512));
        const long pairs = (long)cap_rows * (cap_rows - 1) / 2;
        for (bool fits = false; !fits; sh.threads /= 2) {
            const int n_waves = sh.threads / EF_WAVE;
            // a round of blocks adds at most 256 survivors per wave, and the list is emptied
            // whenever the next round might not fit; more room means fewer drains
            sh.s_cap = 256 * n_waves;
            if (pairs > sh.s_cap && pairs <= 1024) sh.s_cap = align4((int)pairs);
            if (cap_rows <= 16) sh.s_cap = 128;     // a single block of at most 120 pairs
            // (pairs that a row already knows are not queued: a few hundred proposals per join at most)
            for (sh.q_cap = min(4 * sh.threads, 512); sh.q_cap >= 128 && !fits; sh.q_cap /= 2) {
                sh.lds = join_lds_floats(cap_rows, stride, sh.s_cap) * 4 +
                         (size_t)sh.q_cap * sizeof(Proposal);
                fits = sh.lds <= kLdsLimit;
                if (fits) break;
            }
            if (fits || sh.threads == EF_WAVE) break;
        }
        const int n_waves = sh.threads / EF_WAVE;
        // persistent grid: as many blocks as fit the 256 CUs at once, twice over
        long per_cu = (long)(kLdsLimit / sh.lds);
        const long by_waves = 32 / n_waves;
        if (per_cu > by_waves) per_cu = by_waves;
        if (per_cu < 1) per_cu = 1;
        sh.grid = (int)(256 * per_cu * 2);
        return sh;
    };
    Shape large[kMaxClasses];
    size_t large_lds = 0;
    for (int c = 2; c < jc.n; ++c) {
        large[c] = shape_for(jc.bound[c]);
        large_lds = large[c].lds > large_lds ? large[c].lds : large_lds;
    }
    // joins of more than 32 vectors: register tiles for vectors of at most 128 coordinates, else rows in LDS
    const bool tiles = reg_ok && d <= 128;
    if (tiles && max_rows > rows1 && tile_lds_bytes(max_rows, 256) > kLdsLimit) return EFANNA_EUNSUPPORTED;
    if (!tiles && max_rows > rows1 && large_lds > kLdsLimit) return EFANNA_EUNSUPPORTED;
    // joins of at most 16 vectors from registers (d <= 128): room for a whole point's proposals
    // (240) above the drain mark; the others drain between rounds as well (joins of 17..32
    // vectors: 256 entries measured 3 % faster than 128, 512 no better)
    auto reg_q_cap_for = [&](int R) { return R == 16 ? (d <= 128 ? 512 : 256) : (d <= 128 ? 256 : 384); };
    auto reg_lds = [&](int R) {
        const int reg_q_cap = reg_q_cap_for(R);
        return (size_t)(6 * R + align4(R * (R - 1) / 2 + 8)) * 4 +
               (size_t)reg_q_cap * sizeof(Proposal);
    };
    const int reg_grid = kRegGrid;
    // prepare: one thread per point with max_rows ids of LDS each
    int prep_threads = (int)(65536 / ((size_t)(max_rows | 1) * 4)) / EF_WAVE * EF_WAVE;
    prep_threads = prep_threads > kBlock ? kBlock : (prep_threads < EF_WAVE ? EF_WAVE : prep_threads);
    const size_t prep_lds = (size_t)prep_threads * (max_rows | 1) * 4;
    // long lists: a wave per point with a hash table of at least twice the longest list
    const bool prep_wave = max_rows > 96;
    int prep_hash = 128;
    while (prep_hash < 2 * max_rows) prep_hash <<= 1;
    const size_t prep_wave_lds = (size_t)(kBlock / EF_WAVE) * (prep_hash + max_rows + EF_WAVE) * 4;
    const int prep_wave_grid = min(grid_for((size_t)n, kBlock), 256 * 8);
    const int n_part = prep_wave ? prep_wave_grid : grid_for((size_t)n, prep_threads);
    // filter margins: Gram-form rounding error <= (2*dpad + 4) u (|a|^2 + |b|^2), u = 2^-24,
    // doubled; the fixed-order distance is within (d/16 + 8) u of the true one, doubled twice
    const float margin_rel = (float)((4.0 * dpad + 16.0) * 5.9604644775390625e-08);
    const float thr_scale = (float)(1.0 + 4.0 * (d / 16.0 + 8.0) * 5.9604644775390625e-08);
    // The register joins filter with Gram blocks of the vectors in half precision, rounded towards
    // zero after a scaling by a power of two that keeps them below 2^15: a coordinate moves by at
    // most 2^-10 of itself or, below 2^-14, by 2^-24.  The blocks' diagonals are the rounded
    // vectors' squared norms, so the filter's left side is the squared distance D'^2 of the rounded
    // vectors up to the accumulation error, and |D' - D| <= r(a) + r(b) with
    // r(x) = u |x'| + r0, u = 2^-10 / (1 - 2^-10) (+ slack for the square root and the norm's own
    // error), r0 = 1.01 sqrt(d) 2^-24.  The margin on the norms pays for the three accumulations in
    // single precision: four times (dpad + 4) 2^-23, a bound that holds whether the matrix unit
    // rounds or truncates its partial sums.
    const float margin_f16 = (float)(4.0 * (dpad + 4.0) * 1.1920928955078125e-07 + 16.0 * 5.9604644775390625e-08);
    const float thr_scale_f16 = (float)((1.0 + 4.0 * (d / 16.0 + 8.0) * 5.9604644775390625e-08) * (1.0 + 1e-6));
    const float u_f16 = (float)(1.01 / 1023.0);
    const float rho0_f16 = (float)(1.01 * sqrt((double)d) * 5.9604644775390625e-08);
    hipStream_t st = (hipStream_t)stream;
    NndWs w = carve_nnd(ws, n, K, L);
    // reverse lists by buckets (short rows and lists): LDS of an offer block (words) or a list
    // block (keys) with `per_row` of them per row, and one int per bucket or offer block twice over
    const bool bkt = bucketed_lists(n, K, L);
    const int n_bkt = (int)((n + kBktRows - 1) / kBktRows);      // offer blocks
    const int bshift = bucket_shift(L), n_buckets = (int)(((n - 1) >> bshift) + 1);
    auto bkt_lds = [&](int per_row) { return (size_t)kBktRows * per_row * 4 + ((size_t)2 * n_buckets + 4) * 4; };
    if (bkt) {
        EF_HIP_CHECK(hipFuncSetAttribute(K <= 16 ? (const void *)sample_bucket_kernel<2> : (const void *)sample_bucket_kernel<4>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)bkt_lds(L)));
        EF_HIP_CHECK(hipFuncSetAttribute((const void *)reverse_old_bucket_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)bkt_lds(K)));
        // (list lengths of 10 and 20 are compiled in: the scan of a list unrolls, 8 % off the kernel)
        EF_HIP_CHECK(hipFuncSetAttribute(L == 10   ? (const void *)bucket_lists_kernel<10, 10>
                                         : L == 20 ? (const void *)bucket_lists_kernel<9, 20>
                                         : bshift == 10 ? (const void *)bucket_lists_kernel<10, 0>
                                                        : (const void *)bucket_lists_kernel<9, 0>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)bucket_lists_lds(L, n_bkt)));
    }
    if (max_rows > rows1 && tiles && tile_lds_bytes(max_rows, 256) > 64 * 1024) {
        EF_HIP_CHECK(hipFuncSetAttribute((const void *)join_tile_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)tile_lds_bytes(max_rows, 256)));
        EF_HIP_CHECK(hipFuncSetAttribute((const void *)join_tile_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)tile_lds_bytes(max_rows, 256)));
    }
    if (max_rows > rows1 && !tiles)
        EF_HIP_CHECK(hipFuncSetAttribute(K >= 2 * EF_WIDE_PIECES ? (const void *)join_kernel<true>
                                                                 : (const void *)join_kernel<false>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)large_lds));
    zero_u64_kernel<<<1, EF_WAVE, 0, st>>>((u64 *)w.xmax, 1);
    norms_kernel<<<min(grid_for((size_t)n * 16, kBlock), 256 * 8), kBlock, 0, st>>>(X, (int)n, d, w.norms, w.xmax);
    if (stats) zero_u64_kernel<<<grid_for((size_t)iters * 4 + 1, kBlock), kBlock, 0, st>>>(stats, iters * 4);
    // optional phase timing: events around the sampling and the join of every iteration
    struct PhaseEvents {      // destroyed on every way out of the call
        std::vector<hipEvent_t> list;
        ~PhaseEvents()
        {
            for (hipEvent_t e : list) (void)hipEventDestroy(e);
        }
    } events;
    hipEvent_t *ev = nullptr;
    if (phase_ms && iters > 0) {
        events.list.reserve((size_t)iters * 5);
        for (int e = 0; e < iters * 5; ++e) {
            hipEvent_t one;
            EF_HIP_CHECK(hipEventCreate(&one));
            events.list.push_back(one);
        }
        ev = events.list.data();
    }
    int done = 0;
    for (int it = 0; it < iters; ++it) {
        const int g = first_iter + it;
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[5 * it], st));
        // (the bucket scheme writes every list count itself: only the small arrays are reset)
        fill_reverse_kernel<<<grid_for(bkt ? (size_t)n_upd_block : (size_t)n, kBlock), kBlock, 0, st>>>(
            w.rnew_c, w.rold_c, w.list_max, bkt ? (size_t)0 : (size_t)n, w.work_count, w.upd_block,
            n_upd_block, w.ovf_count);
        {
            const u64 kn = ef_stream_key(seed, 2 * g), ko = ef_stream_key(seed, 2 * g + 1);
            Overflow *ovf = (Overflow *)w.overflow;
            const size_t ovf_region = ovf_region_for(n, K);
#define EF_SAMPLE(G, E)                                                                          \
    sample_kernel<G, E><<<grid_for((size_t)n * G, kBlock), kBlock, 0, st>>>(                     \
        graph, (int)n, K, L, kn, w.nw, w.od, w.nw_c, w.od_c, w.rnew, w.rnew_c, ovf,              \
        ovf_region, w.ovf_count, w.worst)
#define EF_BUCKET_LISTS(RUN_CAP, KEY, LISTS, COUNTS)                                             \
    do {                                                                                         \
        if (L == 10)                                                                             \
            bucket_lists_kernel<10, 10><<<n_buckets, kBktThreads, bucket_lists_lds(L, n_bkt), st>>>( \
                w.offer_runs, w.run_table, n_bkt, RUN_CAP, KEY, (int)n, L, (u32 *)(LISTS), COUNTS); \
        else if (L == 20)                                                                        \
            bucket_lists_kernel<9, 20><<<n_buckets, kBktThreads, bucket_lists_lds(L, n_bkt), st>>>( \
                w.offer_runs, w.run_table, n_bkt, RUN_CAP, KEY, (int)n, L, (u32 *)(LISTS), COUNTS); \
        else if (bshift == 10)                                                                   \
            bucket_lists_kernel<10, 0><<<n_buckets, kBktThreads, bucket_lists_lds(L, n_bkt), st>>>( \
                w.offer_runs, w.run_table, n_bkt, RUN_CAP, KEY, (int)n, L, (u32 *)(LISTS), COUNTS); \
        else                                                                                     \
            bucket_lists_kernel<9, 0><<<n_buckets, kBktThreads, bucket_lists_lds(L, n_bkt), st>>>( \
                w.offer_runs, w.run_table, n_bkt, RUN_CAP, KEY, (int)n, L, (u32 *)(LISTS), COUNTS); \
    } while (0)
#define EF_REVERSE_OLD(G)                                                                        \
    reverse_old_kernel<G><<<grid_for((size_t)n * G, kBlock), kBlock, 0, st>>>(                   \
        w.od, (int)n, K, L, ko, w.active, w.rold, w.rold_c, ovf, ovf_region, w.ovf_count)
            if (bkt) {
                if (K <= 16)
                    sample_bucket_kernel<2><<<n_bkt, kBktThreads, bkt_lds(L), st>>>(
                        graph, (int)n, K, L, w.nw, w.od, w.nw_c, w.od_c, w.worst, n_buckets, bshift, w.offer_runs, w.run_table);
                else
                    sample_bucket_kernel<4><<<n_bkt, kBktThreads, bkt_lds(L), st>>>(
                        graph, (int)n, K, L, w.nw, w.od, w.nw_c, w.od_c, w.worst, n_buckets, bshift, w.offer_runs, w.run_table);
                EF_BUCKET_LISTS(kBktRows * L, kn, w.rnew, w.rnew_c);
            } else if (K <= 16) EF_SAMPLE(16, 1);
            else if (K <= 32) EF_SAMPLE(32, 1);
            else if (K <= 64) EF_SAMPLE(64, 1);
            else EF_SAMPLE(64, 2);
            active_kernel<<<grid_for((size_t)n, kBlock), kBlock, 0, st>>>(w.nw_c, w.rnew_c, (int)n, w.active);
            if (bkt) {
                reverse_old_bucket_kernel<<<n_bkt, kBktThreads, bkt_lds(K), st>>>(
                    w.od, (int)n, K, w.active, n_buckets, bshift, w.offer_runs, w.run_table);
                EF_BUCKET_LISTS(kBktRows * K, ko, w.rold, w.rold_c);
            } else if (K <= 16) EF_REVERSE_OLD(16);
            else if (K <= 32) EF_REVERSE_OLD(32);
            else EF_REVERSE_OLD(64);
#undef EF_SAMPLE
#undef EF_REVERSE_OLD
#undef EF_BUCKET_LISTS
            if (bkt) {
            } else if (L >= 2 * EF_WIDE_PIECES)
                reverse_overflow_kernel<true><<<dim3(kOvfBlocksPerQueue, kOvfQueues), kBlock, 0, st>>>(
                    ovf, ovf_region, w.ovf_count, (size_t)n, w.rnew, w.rold, w.list_max, L);
            else
                reverse_overflow_kernel<false><<<dim3(kOvfBlocksPerQueue, kOvfQueues), kBlock, 0, st>>>(
                    ovf, ovf_region, w.ovf_count, (size_t)n, w.rnew, w.rold, w.list_max, L);
        }
#define EF_PREPARE(IDS32)                                                                          \
    prepare_kernel<IDS32><<<grid_for((size_t)n, prep_threads), prep_threads, prep_lds, st>>>(       \
        w.nw, w.od, w.nw_c, w.od_c, w.rnew, w.rold, w.rnew_c, w.rold_c, (int)n, K, L, max_rows,     \
        (u32)(((1ULL << 32) + max_rows - 1) / max_rows), jc, w.ulist, w.ucount, w.work,            \
        w.work_count, w.part)
#define EF_PREPARE_WAVE(IDS32)                                                                      \
    prepare_wave_kernel<IDS32><<<prep_wave_grid, kBlock, prep_wave_lds, st>>>(                      \
        w.nw, w.od, w.nw_c, w.od_c, w.rnew, w.rold, w.rnew_c, w.rold_c, (int)n, K, L, max_rows,     \
        prep_hash, jc, w.ulist, w.ucount, w.work, w.work_count, w.part)
        if (prep_wave) {
            if (bkt) EF_PREPARE_WAVE(true);
            else EF_PREPARE_WAVE(false);
        } else {
            if (bkt) EF_PREPARE(true);
            else EF_PREPARE(false);
        }
#undef EF_PREPARE_WAVE
#undef EF_PREPARE
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[5 * it + 1], st));
        if (tiles && max_rows > rows1)
            graph_ids_kernel<<<min(grid_for((size_t)n * K, kBlock), 256 * 64), kBlock, 0, st>>>(graph, (size_t)n * K, w.gid);
        // One pass over the joins; with cross_old two, all pairs of two new members of every join
        // before any pair of a new and an old one (the phase events are recorded in the last pass:
        // the split by join size then says little).
        const int n_pass = cross_old ? 2 : 1;
        for (int pass = 0; pass < n_pass; ++pass) {
        const int mode = cross_old ? 1 + pass : 0;
        const bool timed = ev && pass == n_pass - 1;
        if (reg_ok) {
#define EF_JOIN_REG_K(NB, ONE, LIST, KT)                                                           \
    join_reg_kernel<NB, ONE, KT><<<reg_grid, EF_WAVE, reg_lds(16 * NB), st>>>(                     \
        X, d, K, w.work + (size_t)(LIST) * n, w.work_count + (LIST), reg_q_cap_for(16 * NB), \
        (ONE) ? margin_f16 : margin_rel, (ONE) ? thr_scale_f16 : thr_scale, u_f16, rho0_f16,       \
        w.ulist, w.ucount, max_rows, graph, w.worst, w.upd_block + (LIST) * reg_grid, mode,        \
        kDenseSurvivors, w.xmax)
    // (a row length of 10 is compiled in: 3 % off the joins of 17..32 vectors)
#define EF_JOIN_REG(NB, ONE, LIST)                                                                 \
    do {                                                                                           \
        if (K == 10) EF_JOIN_REG_K(NB, ONE, LIST, 10);                                             \
        else EF_JOIN_REG_K(NB, ONE, LIST, 0);                                                      \
    } while (0)
            if (d <= 128) EF_JOIN_REG(1, true, 0);
            else EF_JOIN_REG(1, false, 0);
            if (timed) EF_HIP_CHECK(hipEventRecord(ev[5 * it + 2], st));
            if (max_rows > 16) {
                if (d <= 128) EF_JOIN_REG(2, true, 1);
                else EF_JOIN_REG(2, false, 1);
            }
#undef EF_JOIN_REG
#undef EF_JOIN_REG_K
        } else if (timed) {
            EF_HIP_CHECK(hipEventRecord(ev[5 * it + 2], st));
        }
        if (timed) EF_HIP_CHECK(hipEventRecord(ev[5 * it + 3], st));
#define EF_JOIN_LARGE(WIDE, C)                                                                     \
    join_kernel<WIDE><<<large[C].grid, large[C].threads, large[C].lds, st>>>(                      \
        X, w.norms, d, dpad, stride, q4_magic_for(d), K, (u32)(((1ULL << 32) + K - 1) / K),       \
        w.work + (size_t)(C) * n, w.work_count + (C),                                              \
        large[C].cap_rows, large[C].s_cap, large[C].q_cap, margin_rel, thr_scale, w.ulist,         \
        w.ucount, max_rows, graph, w.worst, w.upd_block + 2 * reg_grid + ((C) - 2) * kMaxLargeGrid, mode)
        // the larger classes first: their blocks run longest
        for (int c = jc.n - 1; c >= 2 && max_rows > rows1; --c) {
            if (tiles) {      // vectors of at most 128 coordinates pass through registers
                const int tq = 256;
                const size_t tl = tile_lds_bytes(jc.bound[c], tq);
                long per_cu = (long)(kLdsLimit / tl);
                per_cu = per_cu > 4 * kTileWaves ? 4 * kTileWaves : (per_cu < 1 ? 1 : per_cu);      // by registers
                const int tgrid = (int)(256 * per_cu * 4);
                int *upd = w.upd_block + 2 * reg_grid + (c - 2) * kMaxLargeGrid;
                const u32 km = (u32)(((1ULL << 32) + K - 1) / K);
                const u32 kqm = K >= 4 ? (u32)(((1ULL << 32) + (K >> 2) - 1) / (K >> 2)) : 0u;
                if (K > 16 && (K & 1) == 0 && ((uintptr_t)graph & 15) == 0)
                    join_tile_kernel<true><<<tgrid, EF_WAVE, tl, st>>>(
                        X, w.norms, d, K, km, kqm, w.gid, w.work + (size_t)c * n, w.work_count + c, jc.bound[c], tq,
                        margin_rel, thr_scale, w.ulist, w.ucount, max_rows, graph, w.worst, upd, mode);
                else
                    join_tile_kernel<false><<<tgrid, EF_WAVE, tl, st>>>(
                        X, w.norms, d, K, km, kqm, w.gid, w.work + (size_t)c * n, w.work_count + c, jc.bound[c], tq,
                        margin_rel, thr_scale, w.ulist, w.ucount, max_rows, graph, w.worst, upd, mode);
            } else if (K >= 2 * EF_WIDE_PIECES) EF_JOIN_LARGE(true, c);
            else EF_JOIN_LARGE(false, c);
        }
#undef EF_JOIN_LARGE
        }      // pass
        if (ev) EF_HIP_CHECK(hipEventRecord(ev[5 * it + 4], st));
        if (stats)
            stats_kernel<<<16, kBlock, 0, st>>>(w.part, n_part, w.upd_block,
                                                n_upd_block, stats + 4 * it);
        done = it + 1;
        if (delta > 0.0f) {      // early termination: the host looks at the count after every iteration
            u64 fresh = 0;
            zero_u64_kernel<<<1, kBlock, 0, st>>>(w.fresh, 1);
            count_new_kernel<<<1024, kBlock, 0, st>>>(graph, (size_t)n * K, w.fresh);
            EF_HIP_CHECK(hipMemcpyAsync(&fresh, w.fresh, 8, hipMemcpyDeviceToHost, st));
            EF_HIP_CHECK(hipStreamSynchronize(st));
            if ((double)fresh < (double)delta * (double)n * (double)K) break;
        }
    }
    if (iters_done) *iters_done = done;
    EF_HIP_CHECK(hipGetLastError());
    if (ev) {
        EF_HIP_CHECK(hipStreamSynchronize(st));
        for (int it = 0; it < iters; ++it) {
            for (int ph = 0; ph < 4; ++ph) {
                if (it < done)
                    EF_HIP_CHECK(hipEventElapsedTime(&phase_ms[4 * it + ph], ev[5 * it + ph], ev[5 * it + ph + 1]));
                else
                    phase_ms[4 * it + ph] = 0.0f;
            }
        }
    }
    return EFANNA_OK;
}

}  // namespace

extern "C" int efanna_get_graph(const efanna_entry *graph_, int64_t n, int32_t k, int32_t *ids,
                                float *dists, uint8_t *flags, void *stream)
{
    const u64 *const graph = (const u64 *)graph_;
    if (!graph || !ids || !dists || n < 1 || k < 1 || k > EFANNA_MAX_K) return EFANNA_EINVAL;
    if (k <= 16)
        get_graph_group_kernel<16><<<grid_for((size_t)n * 16, kBlock), kBlock, 0, (hipStream_t)stream>>>(
            graph, (int)n, k, ids, dists, flags);
    else if (k <= 32)
        get_graph_group_kernel<32><<<grid_for((size_t)n * 32, kBlock), kBlock, 0, (hipStream_t)stream>>>(
            graph, (int)n, k, ids, dists, flags);
    else
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
