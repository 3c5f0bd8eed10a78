// Device-side helpers shared by the gfx950 kernels: counter-based generator, packed
// graph entries, the lock-free bounded list insertion and small wave utilities.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/efanna.h"

typedef unsigned long long u64;
typedef unsigned int u32;

#define EF_WAVE 64
#define EF_INF_BITS 0x7F800000u

// a failed HIP call ends the entry point with EFANNA_EHIP; with EFANNA_DEBUG set in the
// environment the call and the runtime's message are printed to stderr first
#define EF_HIP_CHECK(expr)                                                                     \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) {                                                                \
            if (getenv("EFANNA_DEBUG"))                                                        \
                fprintf(stderr, "efanna: %s:%d: %s -> %s\n", __FILE__, __LINE__, #expr,        \
                        hipGetErrorString(e_));                                                \
            return EFANNA_EHIP;                                                                \
        }                                                                                      \
    } while (0)

// ---- counter-based generator (SplitMix64 finaliser) ---------------------------------
__host__ __device__ inline u64 ef_mix64(u64 z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
// stream key for (seed, k): tree index for node draws, iteration stream for reverse hashes
__host__ __device__ inline u64 ef_stream_key(u64 seed, int k)
{
    return ef_mix64(seed + 0x9E3779B97F4A7C15ULL * (u64)(k + 1));
}

// coordinate of the exact mean test of Alg. 2: multiples of 2^-20 as integers
__device__ inline long long ef_quantise(float x) { return (long long)rint((double)x * 1048576.0); }

// What a tree node's split test looks at.  dim >= 0: the quantised coordinate dim (clamped into
// the vector: foreign tables cannot lead out of it).  dim <= -3: a random projection, the sum of
// eight quantised coordinates with signs, both drawn from the 30-bit number r = -3 - dim that the
// node's draw supplies - term k takes z = mix((r << 8) + k + golden), coordinate z mod d, minus if
// the top bit of z is set.  dim -1 (and -2): no test.  coord(j) returns coordinate j of the vector.
constexpr int kProjectionTerms = 8;
__host__ __device__ inline bool ef_has_test(int dim) { return dim >= 0 || dim <= -3; }
__host__ __device__ inline int ef_projection_code(u64 draw) { return -3 - (int)((draw >> 34) & 0x3FFFFFFFULL); }
template <class Coord>
__device__ inline long long ef_node_value(Coord coord, int d, int dim)
{
    if (dim >= 0) return ef_quantise(coord(dim < d ? dim : d - 1));
    const u64 r = (u64)(u32)(-3 - dim);
    long long v = 0;
#pragma unroll
    for (int k = 0; k < kProjectionTerms; ++k) {
        const u64 z = ef_mix64((r << 8) + (u64)k + 0x9E3779B97F4A7C15ULL);
        const long long q = ef_quantise(coord((int)(z % (u64)d)));
        v += (z >> 63) ? -q : q;
    }
    return v;
}

// ---- packed graph entries -------------------------------------------------------------
__device__ inline u64 ef_pack(float dist, int id, int is_new)
{
    return ((u64)__float_as_uint(dist) << 32) | ((u64)(u32)id << 1) | (u64)(is_new & 1);
}
// slot s of an empty row: +inf with a per-slot id so that all entries of a row differ
__host__ __device__ inline u64 ef_empty_entry(int slot)
{
    return ((u64)EF_INF_BITS << 32) | ((u64)(0x7FFFFFFFu - (u32)slot) << 1);
}
__device__ inline u32 ef_dist_bits(u64 e) { return (u32)(e >> 32); }
__device__ inline int ef_id(u64 e) { return (int)((u32)e >> 1); }
__device__ inline bool ef_is_empty(u64 e) { return ef_dist_bits(e) >= EF_INF_BITS; }

__device__ inline u64 ef_load_coherent(const u64 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline u32 ef_load_coherent(const u32 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- coherent 16-byte row loads -----------------------------------------------------------
// Graph rows and reverse lists are read while other waves update them, so the loads must come
// from the point of coherence (as an agent-scope atomic load does), but the widest atomic
// load is 8 bytes and every load is one transaction at the memory side.  Reading a row in
// 16-byte pieces halves that count.  The compiler has no coherent 16-byte load, hence the
// inline assembly: `NP` loads from p, p + 16, ... and the wait for them, in one statement
// so that nothing can touch the destination registers before the data has arrived.
typedef u32 ef_u32x4 __attribute__((ext_vector_type(4)));

__device__ inline void ef_load_row_pieces_1(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %1, off offset:0 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_2(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %2, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %2, off offset:16 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_3(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %3, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %3, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %3, off offset:32 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_4(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %4, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %4, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %4, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %4, off offset:48 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_5(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %5, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %5, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %5, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %5, off offset:48 sc1\n\t"
                     "global_load_dwordx4 %4, %5, off offset:64 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3]), "=&v"(q[4])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_6(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %6, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %6, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %6, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %6, off offset:48 sc1\n\t"
                     "global_load_dwordx4 %4, %6, off offset:64 sc1\n\t"
                     "global_load_dwordx4 %5, %6, off offset:80 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3]), "=&v"(q[4]), "=&v"(q[5])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_7(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %7, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %7, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %7, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %7, off offset:48 sc1\n\t"
                     "global_load_dwordx4 %4, %7, off offset:64 sc1\n\t"
                     "global_load_dwordx4 %5, %7, off offset:80 sc1\n\t"
                     "global_load_dwordx4 %6, %7, off offset:96 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3]), "=&v"(q[4]), "=&v"(q[5]), "=&v"(q[6])
                 : "v"(p)
                 : "memory");
}

__device__ inline void ef_load_row_pieces_8(const void *p, ef_u32x4 (&q)[8])
{
    asm volatile(
                     "global_load_dwordx4 %0, %8, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %8, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %8, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %8, off offset:48 sc1\n\t"
                     "global_load_dwordx4 %4, %8, off offset:64 sc1\n\t"
                     "global_load_dwordx4 %5, %8, off offset:80 sc1\n\t"
                     "global_load_dwordx4 %6, %8, off offset:96 sc1\n\t"
                     "global_load_dwordx4 %7, %8, off offset:112 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3]), "=&v"(q[4]), "=&v"(q[5]), "=&v"(q[6]), "=&v"(q[7])
                 : "v"(p)
                 : "memory");
}

// twenty-five pieces (fifty entries) at once: for long rows, in kernels with registers to spare
constexpr int EF_WIDE_PIECES = 25;
__device__ inline void ef_load_row_pieces_wide(const void *p, ef_u32x4 (&q)[EF_WIDE_PIECES])
{
    asm volatile(
                     "global_load_dwordx4 %0, %25, off offset:0 sc1\n\t"
                     "global_load_dwordx4 %1, %25, off offset:16 sc1\n\t"
                     "global_load_dwordx4 %2, %25, off offset:32 sc1\n\t"
                     "global_load_dwordx4 %3, %25, off offset:48 sc1\n\t"
                     "global_load_dwordx4 %4, %25, off offset:64 sc1\n\t"
                     "global_load_dwordx4 %5, %25, off offset:80 sc1\n\t"
                     "global_load_dwordx4 %6, %25, off offset:96 sc1\n\t"
                     "global_load_dwordx4 %7, %25, off offset:112 sc1\n\t"
                     "global_load_dwordx4 %8, %25, off offset:128 sc1\n\t"
                     "global_load_dwordx4 %9, %25, off offset:144 sc1\n\t"
                     "global_load_dwordx4 %10, %25, off offset:160 sc1\n\t"
                     "global_load_dwordx4 %11, %25, off offset:176 sc1\n\t"
                     "global_load_dwordx4 %12, %25, off offset:192 sc1\n\t"
                     "global_load_dwordx4 %13, %25, off offset:208 sc1\n\t"
                     "global_load_dwordx4 %14, %25, off offset:224 sc1\n\t"
                     "global_load_dwordx4 %15, %25, off offset:240 sc1\n\t"
                     "global_load_dwordx4 %16, %25, off offset:256 sc1\n\t"
                     "global_load_dwordx4 %17, %25, off offset:272 sc1\n\t"
                     "global_load_dwordx4 %18, %25, off offset:288 sc1\n\t"
                     "global_load_dwordx4 %19, %25, off offset:304 sc1\n\t"
                     "global_load_dwordx4 %20, %25, off offset:320 sc1\n\t"
                     "global_load_dwordx4 %21, %25, off offset:336 sc1\n\t"
                     "global_load_dwordx4 %22, %25, off offset:352 sc1\n\t"
                     "global_load_dwordx4 %23, %25, off offset:368 sc1\n\t"
                     "global_load_dwordx4 %24, %25, off offset:384 sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                 : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3]), "=&v"(q[4]), "=&v"(q[5]), "=&v"(q[6]), "=&v"(q[7]), "=&v"(q[8]), "=&v"(q[9]), "=&v"(q[10]), "=&v"(q[11]), "=&v"(q[12]), "=&v"(q[13]), "=&v"(q[14]), "=&v"(q[15]), "=&v"(q[16]), "=&v"(q[17]), "=&v"(q[18]), "=&v"(q[19]), "=&v"(q[20]), "=&v"(q[21]), "=&v"(q[22]), "=&v"(q[23]), "=&v"(q[24])
                 : "v"(p)
                 : "memory");
}

// pieces 0..np-1 of the row at p (16-byte aligned) into q; the rest of q is zero
__device__ inline void ef_load_row_pieces(const void *p, int np, ef_u32x4 (&q)[8])
{
#pragma unroll
    for (int k = 0; k < 8; ++k) q[k] = (ef_u32x4){0u, 0u, 0u, 0u};
    switch (np) {
    case 1: ef_load_row_pieces_1(p, q); break;
    case 2: ef_load_row_pieces_2(p, q); break;
    case 3: ef_load_row_pieces_3(p, q); break;
    case 4: ef_load_row_pieces_4(p, q); break;
    case 5: ef_load_row_pieces_5(p, q); break;
    case 6: ef_load_row_pieces_6(p, q); break;
    case 7: ef_load_row_pieces_7(p, q); break;
    default: ef_load_row_pieces_8(p, q); break;
    }
}

// ---- lock-free bounded insertion ---------------------------------------------------------
// `list` holds `cap` distinct 64-bit keys.  The call makes the list hold the `cap`
// smallest keys of (list U {key}), where two keys are the same element when they agree
// after dropping the lowest `ignore` bits (the new mark of a graph entry).
//
// Why concurrent calls are safe without a lock: a slot is only ever overwritten by a
// smaller key (compare-and-swap of the slot that held the maximum of a snapshot), so
// slot values decrease monotonically.  A successful CAS proves that slot still held the
// snapshot's maximum; every other slot can only have got smaller since it was read, so
// the replaced key was the true maximum at that instant, and the inserted key cannot
// have appeared elsewhere in the meantime (it would have had to replace a maximum no
// smaller than the one just replaced).  The final content is therefore the set of the
// `cap` smallest keys ever offered, whatever the interleaving.
//
// Returns true if the key went in; *new_max then holds an upper bound of the list's
// maximum after the insertion.
template <bool WIDE, bool REFINE = false>
__device__ inline bool ef_bounded_insert_t(u64 *list, int cap, u64 key, int ignore, u64 *new_max)
{
    const u64 kcmp = key >> ignore;
    if (REFINE && cap <= 16) {
        // Short lists: one snapshot.  A compare-and-swap that fails hands back what the slot
        // holds now, which is all that is needed to go on: the snapshot is corrected in that
        // one slot and the maximum taken again, without a second read of the list.  (The
        // argument above only needs every slot to have been read at some time before the swap
        // that succeeds, and the swapped slot to hold the snapshot's maximum.)
        const bool wide = (cap & 1) == 0 && ((uintptr_t)list & 15) == 0;
        u64 e[16];
        if (wide) {
            ef_u32x4 q[8];
            ef_load_row_pieces(list, cap >> 1, q);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                e[2 * k] = ((u64)q[k].y << 32) | q[k].x;
                e[2 * k + 1] = ((u64)q[k].w << 32) | q[k].z;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) e[k] = k < cap ? ef_load_coherent(list + k) : 0;
        }
        for (;;) {
            u64 mx = 0, mx2 = 0;
            int ms = 0;
            bool dup = false;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                if (k >= cap) break;
                dup |= (e[k] >> ignore) == kcmp;
                if (e[k] > mx) {
                    mx2 = mx;
                    mx = e[k];
                    ms = k;
                } else if (e[k] > mx2) {
                    mx2 = e[k];
                }
            }
            if (dup || kcmp >= (mx >> ignore)) return false;
            const u64 seen = atomicCAS(list + ms, mx, key);
            if (seen == mx) {
                *new_max = key > mx2 ? key : mx2;
                return true;
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) e[k] = k == ms ? seen : e[k];
        }
    }
    for (;;) {
        u64 mx = 0, mx2 = 0;
        int ms = 0;
        bool dup = false;
        auto see = [&](u64 e, int slot) {
            dup |= (e >> ignore) == kcmp;
            if (e > mx) {
                mx2 = mx;
                mx = e;
                ms = slot;
            } else if (e > mx2) {
                mx2 = e;
            }
        };
        // sixteen slots in flight at a time (fifty with WIDE, while the row has as many left): a
        // row of up to 16 entries costs one memory round trip instead of one per slot
        const bool wide = (cap & 1) == 0 && ((uintptr_t)list & 15) == 0;
        int s0 = 0;
        if (WIDE && wide) {
            for (; s0 + 2 * EF_WIDE_PIECES <= cap; s0 += 2 * EF_WIDE_PIECES) {
                ef_u32x4 q[EF_WIDE_PIECES];
                ef_load_row_pieces_wide(list + s0, q);
#pragma unroll
                for (int k = 0; k < EF_WIDE_PIECES; ++k) {
                    see(((u64)q[k].y << 32) | q[k].x, s0 + 2 * k);
                    see(((u64)q[k].w << 32) | q[k].z, s0 + 2 * k + 1);
                }
            }
        }
        for (; s0 < cap; s0 += 16) {
            u64 e[16];
            if (wide) {      // even length, 16-byte aligned: eight 16-byte pieces
                ef_u32x4 q[8];
                ef_load_row_pieces(list + s0, min(8, (cap - s0) >> 1), q);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    e[2 * k] = ((u64)q[k].y << 32) | q[k].x;
                    e[2 * k + 1] = ((u64)q[k].w << 32) | q[k].z;
                }
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) e[k] = s0 + k < cap ? ef_load_coherent(list + s0 + k) : 0;
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                if (s0 + k >= cap) break;
                see(e[k], s0 + k);
            }
        }
        if (dup || kcmp >= (mx >> ignore)) return false;
        u64 seen = atomicCAS(list + ms, mx, key);
        if (seen == mx) {
            *new_max = key > mx2 ? key : mx2;
            return true;
        }
    }
}

__device__ inline bool ef_bounded_insert(u64 *list, int cap, u64 key, int ignore, u64 *new_max)
{
    return ef_bounded_insert_t<false>(list, cap, key, ignore, new_max);
}

// ---- the same insertion by a group of sixteen lanes (long rows) ----------------------------
// n (1..4) pieces from n addresses, in flight together
__device__ inline void ef_load_pieces_at(const void *p0, const void *p1, const void *p2, const void *p3,
                                         int n, ef_u32x4 (&q)[4])
{
    switch (n) {
    case 1:
        asm volatile(
                     "global_load_dwordx4 %0, %1, off sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q[0])
                     : "v"(p0)
                     : "memory");
        break;
    case 2:
        asm volatile(
                     "global_load_dwordx4 %0, %2, off sc1\n\t"
                     "global_load_dwordx4 %1, %3, off sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q[0]), "=&v"(q[1])
                     : "v"(p0), "v"(p1)
                     : "memory");
        break;
    case 3:
        asm volatile(
                     "global_load_dwordx4 %0, %3, off sc1\n\t"
                     "global_load_dwordx4 %1, %4, off sc1\n\t"
                     "global_load_dwordx4 %2, %5, off sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2])
                     : "v"(p0), "v"(p1), "v"(p2)
                     : "memory");
        break;
    default:
        asm volatile(
                     "global_load_dwordx4 %0, %4, off sc1\n\t"
                     "global_load_dwordx4 %1, %5, off sc1\n\t"
                     "global_load_dwordx4 %2, %6, off sc1\n\t"
                     "global_load_dwordx4 %3, %7, off sc1\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3])
                     : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
                     : "memory");
    }
}

// All sixteen lanes of a group (lane gl = 0..15 of it) call this with the same arguments and get
// the same result.  Lane gl reads the 16-byte pieces gl, gl + 16, ... of the row, so that the
// group fetches 256 contiguous bytes per load: a quarter of the memory transactions that a lane
// reading the whole row alone needs, and one round trip for rows of up to 128 entries.  The
// row must be 16-byte aligned and of even length; the group's lanes must all be active.
// slot (or null): receives the slot the key went into.
__device__ inline bool ef_bounded_insert_g16(u64 *list, int cap, u64 key, int ignore, u64 *new_max, int gl,
                                             int *slot = nullptr)
{
    const u64 kcmp = key >> ignore;
    const int np = cap >> 1;
    for (;;) {
        u64 mx = 0, mx2 = 0;
        int ms = 0;
        bool dup = false;
        for (int p0 = 0; p0 < np; p0 += 64) {
            const int n_ld = min(4, (np - p0 + 15) >> 4);
            ef_u32x4 q[4];
            const ef_u32x4 *row = reinterpret_cast<const ef_u32x4 *>(list);
            // pieces beyond the row read its last piece again and are not looked at
            ef_load_pieces_at(row + min(p0 + gl, np - 1), row + min(p0 + gl + 16, np - 1),
                              row + min(p0 + gl + 32, np - 1), row + min(p0 + gl + 48, np - 1), n_ld, q);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int piece = p0 + gl + 16 * k;
                if (k >= n_ld || piece >= np) continue;
                const u64 e2[2] = {((u64)q[k].y << 32) | q[k].x, ((u64)q[k].w << 32) | q[k].z};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    dup |= (e2[h] >> ignore) == kcmp;
                    if (e2[h] > mx) {
                        mx2 = mx;
                        mx = e2[h];
                        ms = 2 * piece + h;
                    } else if (e2[h] > mx2) {
                        mx2 = e2[h];
                    }
                }
            }
        }
        // the group's largest and second largest entry (entries of a row are distinct)
        for (int m = 8; m >= 1; m >>= 1) {
            const u64 omx = __shfl_xor(mx, m, 16), omx2 = __shfl_xor(mx2, m, 16);
            const int oms = __shfl_xor(ms, m, 16);
            dup |= (bool)__shfl_xor((int)dup, m, 16);
            if (omx > mx) {
                mx2 = mx > omx2 ? mx : omx2;
                mx = omx;
                ms = oms;
            } else if (omx > mx2) {
                mx2 = omx;
            }
        }
        if (dup || kcmp >= (mx >> ignore)) return false;
        u64 seen = 0;
        if (gl == 0) seen = atomicCAS(list + ms, mx, key);
        seen = __shfl(seen, 0, 16);
        if (seen == mx) {
            *new_max = key > mx2 ? key : mx2;
            if (slot) *slot = ms;
            return true;
        }
    }
}

// ---- wave utilities ---------------------------------------------------------------------
__device__ inline int ef_lane() { return (int)(threadIdx.x & (EF_WAVE - 1)); }

__device__ inline long long ef_wave_sum_i64(long long v)
{
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, EF_WAVE);
    return v;
}
__device__ inline int ef_wave_sum_i32(int v)
{
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, EF_WAVE);
    return v;
}
// inclusive prefix sum over the wave
__device__ inline int ef_wave_scan_i32(int v)
{
    const int lane = ef_lane();
    for (int o = 1; o < EF_WAVE; o <<= 1) {
        int t = __shfl_up(v, o, EF_WAVE);
        if (lane >= o) v += t;
    }
    return v;
}

// Squared L2 distance in the library's fixed order, evaluated by a group of 16
// consecutive lanes: lane l of the group owns partial sum l.  Every lane of the group
// returns the full value.  All 16 lanes must be active.
__device__ inline float ef_group_reduce16(float acc)
{
    acc += __shfl_xor(acc, 8, 16);
    acc += __shfl_xor(acc, 4, 16);
    acc += __shfl_xor(acc, 2, 16);
    acc += __shfl_xor(acc, 1, 16);
    return acc;
}

// 16 partial sums per lane (one per pair of a 4x4 tile) across a 16-lane group ->
// lane l keeps the total of pair l.  Same adds, in the same tree, as ef_group_reduce16
// applied to each pair, but with 15 exchanges instead of 64.
__device__ inline float ef_group_transpose_reduce16(const float (&acc)[16], int gl)
{
    float a8[8], a4[4], a2[2];
    const bool b3 = gl & 8, b2 = gl & 4, b1 = gl & 2, b0 = gl & 1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float keep = b3 ? acc[k + 8] : acc[k];
        float send = b3 ? acc[k] : acc[k + 8];
        a8[k] = keep + __shfl_xor(send, 8, 16);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float keep = b2 ? a8[k + 4] : a8[k];
        float send = b2 ? a8[k] : a8[k + 4];
        a4[k] = keep + __shfl_xor(send, 4, 16);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float keep = b1 ? a4[k + 2] : a4[k];
        float send = b1 ? a4[k] : a4[k + 2];
        a2[k] = keep + __shfl_xor(send, 2, 16);
    }
    float keep = b0 ? a2[1] : a2[0];
    float send = b0 ? a2[0] : a2[1];
    return keep + __shfl_xor(send, 1, 16);
}
