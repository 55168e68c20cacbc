// PRT-TFB best-first search (Alg. 2, Sec. 3.3): one wavefront owns one query from the
// entry nodes to the final top-K.  Included by the instantiation units pag_search_nq*_cw*.hip.
//
// Wave-level data placement (64 lanes):
//   query        registers, NQ float4 per lane (element chunk c*64+lane)
//   W            registers, NW slots per lane (b <= 64 NW).  Up to 128 nodes (NW <= 2): sorted ascending by key, rank r
//                in slot r/64 of lane r%64.  Above (NW >= 4): unsorted, entry i in slot i/64 of lane i%64; the node to
//                expand and the farthest member are found by wave-wide minima / maxima, the farthest one is cached
//   R_L          up to 128 nodes: registers, same placement (capacity K <= b); above: the front of a per-wave HBM buffer
//   table T      LDS, float [Ppad][16]
//   seen set     short searches: LDS open-addressing hash of node ids (exact; overflows into a
//                per-wave HBM bitmap).  Long searches: every id goes to the per-wave HBM bitmap,
//                an LDS Bloom filter says which lookups can skip it, and the LDS table is a
//                direct-mapped cache of recently admitted ids (most re-encounters are recent)
//   R_F, R_T     rings (power-of-two buffers, the last b pushes are valid): LDS, or per-wave HBM
//                buffers for working sets above 128 nodes, which are pushed to rarely and read
//                once per round
//   SA, SB       scratch for scatters and sorts: LDS for working sets of up to 128 nodes; above, two per-wave HBM buffers
//                that are touched at round ends only (SA holds R_L in front and sorts R_L + W, SB sorts the rings)
// A key packs (dist bits << 32) | (id << 1) | visited, so that unsigned comparison orders by
// (dist, id); distances are sums of squares, hence non-negative and monotone as bit patterns.
//
// One hop evaluates the projection test for all neighbours of u at once, lane s <-> neighbour
// slot s, against the threshold read when u is popped; the hop's passers enter W as if they
// were admitted one after another in ascending (dist, id) order, which a merge by ranks
// reproduces exactly: the b smallest of W + passers stay, displaced W members go to R_T
// (largest first), passers that do not fit go to R_F (smallest first).
#pragma once

#include "pag_internal.h"
#include "pag_wave.h"

#include <type_traits>

namespace pagk {

__device__ __forceinline__ u32 rdlane(u32 v, int l) { return (u32)__builtin_amdgcn_readlane((int)v, l); }
__device__ __forceinline__ u64 rdlane64(u64 v, int l) {
    u32 lo = rdlane((u32)v, l), hi = rdlane((u32)(v >> 32), l);
    return ((u64)hi << 32) | lo;
}
// The workgroup is a single wavefront and its LDS operations execute in program order, so all that
// cross-lane LDS traffic needs is that the compiler keeps the accesses in place and that the LDS
// queue has drained.  Unlike __syncthreads() this does not wait for global loads in flight
// (prefetched records, seen-set words), which is the point.
__device__ __forceinline__ void lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ u32 uniform(u32 v) { return (u32)__builtin_amdgcn_readfirstlane((int)v); }

__device__ __forceinline__ u32 hash_slot(u32 id, u32 hlog) { return (id * 2654435761u) >> (32 - hlog); }

__device__ __forceinline__ bool hash_contains(const u32* H, u32 hlog, u32 id) {
    const u32 mask = (1u << hlog) - 1;
    u32 p = hash_slot(id, hlog);
    for (;;) {
        u32 v = H[p];
        if (v == id) return true;
        if (v == PAG_EMPTY) return false;
        p = (p + 1) & mask;
    }
}

__device__ __forceinline__ void hash_insert(u32* H, u32 hlog, u32 id) {
    const u32 mask = (1u << hlog) - 1;
    u32 p = hash_slot(id, hlog);
    for (;;) {
        u32 old = atomicCAS(&H[p], PAG_EMPTY, id);
        if (old == PAG_EMPTY || old == id) return;
        p = (p + 1) & mask;
    }
}

// Bloom filter over the ids that live in the HBM bitmap (two hash functions, LDS bit array):
// "no" is definite, so most lookups of unseen nodes never touch HBM.
__device__ __forceinline__ bool bloom_maybe(const u32* B, u32 blog, u32 id) {
    const u32 h1 = (id * 0x9E3779B1u) >> (32 - blog), h2 = (id * 0x85EBCA77u) >> (32 - blog);
    return ((B[h1 >> 5] >> (h1 & 31)) & (B[h2 >> 5] >> (h2 & 31)) & 1u) != 0;
}
__device__ __forceinline__ void bloom_set(u32* B, u32 blog, u32 id) {
    const u32 h1 = (id * 0x9E3779B1u) >> (32 - blog), h2 = (id * 0x85EBCA77u) >> (32 - blog);
    atomicOr(&B[h1 >> 5], 1u << (h1 & 31));
    atomicOr(&B[h2 >> 5], 1u << (h2 & 31));
}

// dst[rank] = src[i], rank = number of smaller keys; keys are distinct.  Quadratic: for short lists.
__device__ __forceinline__ void rank_sort(const u64* src, u64* dst, u32 n, int lane) {
    for (u32 i = lane; i < n; i += 64) {
        const u64 k = src[i];
        u32 r = 0;
        for (u32 j = 0; j < n; ++j) r += (src[j] < k) ? 1u : 0u;
        dst[r] = k;
    }
}

// In-place ascending bitonic sort of S[0, n) in LDS by one wave; S has room for n rounded up to a power
// of two (the tail is padded with the largest key).
__device__ __forceinline__ void bitonic_sort(u64* S, u32 n, int lane) {
    u32 N = 64;
    while (N < n) N <<= 1;
    for (u32 i = n + lane; i < N; i += 64) S[i] = PAG_KEY_INVALID;
    lds_sync();
    for (u32 k = 2; k <= N; k <<= 1)
        for (u32 j = k >> 1; j > 0; j >>= 1) {
            for (u32 t = lane; t < N / 2; t += 64) {
                const u32 i = ((t & ~(j - 1)) << 1) | (t & (j - 1));   // bit j clear
                const u32 l = i | j;
                const u64 x = S[i], y = S[l];
                if ((x > y) == ((i & k) == 0)) { S[i] = y; S[l] = x; }
            }
            lds_sync();
        }
}

// Ascending bitonic sort of 64 * NS keys held in registers, key e in slot e / 64 of lane e % 64 (pad with the
// largest key).  Compare-exchange steps at distances below 64 go across lanes (one exchange per slot), those at
// distances of 64 and more pair up slots of the same lane.  No memory is touched.
template <int NS, int D>
__device__ __forceinline__ void bitonic_slot_step(u64 (&x)[NS], u32 k) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if ((s & D) == 0) {
            const bool asc = ((64u * (u32)s) & k) == 0;
            const u64 a = x[s], b = x[s | D];
            const u64 lo = a < b ? a : b, hi = a < b ? b : a;
            x[s] = asc ? lo : hi;
            x[s | D] = asc ? hi : lo;
        }
}

template <int NS>
__device__ __forceinline__ void bitonic_registers(u64 (&x)[NS], int lane) {
    for (u32 k = 2; k <= 64u * NS; k <<= 1) {
        // slot distance D pairs keys 64 D apart: part of the stages k >= 128 D
        if constexpr (NS >= 32) { if (k >= 16u * 128u) bitonic_slot_step<NS, 16>(x, k); }
        if constexpr (NS >= 16) { if (k >= 8u * 128u) bitonic_slot_step<NS, 8>(x, k); }
        if constexpr (NS >= 8) { if (k >= 4u * 128u) bitonic_slot_step<NS, 4>(x, k); }
        if constexpr (NS >= 4) { if (k >= 2u * 128u) bitonic_slot_step<NS, 2>(x, k); }
        if constexpr (NS >= 2) { if (k >= 128u) bitonic_slot_step<NS, 1>(x, k); }
        for (u32 j = (k >> 1) < 32u ? (k >> 1) : 32u; j > 0; j >>= 1) {
            const bool lower = ((u32)lane & j) == 0;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const u64 other = (u64)__shfl_xor((unsigned long long)x[s], (int)j, 64);
                const bool asc = ((64u * (u32)s + (u32)lane) & k) == 0;
                const u64 lo = x[s] < other ? x[s] : other, hi = x[s] < other ? other : x[s];
                x[s] = (lower == asc) ? lo : hi;
            }
        }
    }
}

// Sorts the n keys in `a` ascending and returns where the result lives.  Working sets whose lists
// are always short (by_ranks) go through the rank sort into `b`; the others sort in place, and
// their `b` does not exist.
__device__ __forceinline__ const u64* sort_keys(u64* a, u64* b, u32 n, bool by_ranks, int lane) {
    if (by_ranks) {
        rank_sort(a, b, n, lane);
        lds_sync();
        return b;
    }
    bitonic_sort(a, n, lane);
    return a;
}

// Optional per-phase timers (diagnostic builds only): every mark first drains all outstanding
// memory operations, so the phases are timed as if they did not overlap.
#ifdef PAG_PHASE_TIMERS
#define PAG_MARK(i)                                                  \
    do {                                                             \
        __builtin_amdgcn_s_waitcnt(0);                               \
        const u64 t__ = wall_clock64();                              \
        s_phase[i] += t__ - t_last;                                  \
        t_last = t__;                                                \
    } while (0)
#else
#define PAG_MARK(i) do {} while (0)
#endif

// S = sum_l T[l][code_l] over the CW * 8 subspaces of one neighbour, added in increasing l.
// The LDS gathers of 16 subspaces are issued together, then consumed in order.  `t_base` is the
// LDS byte address of T, a multiple of 64, so that "4 * code" can be OR-ed into it and the row
// offset 64 * l rides in the instruction.
typedef __attribute__((address_space(3))) const float* lds_cfloat_ptr;
template <int CW>
__device__ __forceinline__ float table_sum(u32 t_base, const u32 (&cwv)[CW]) {
    float S = 0.f;
#pragma unroll
    for (int k = 0; k < CW; k += 2) {
        float t[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const u32 wd = cwv[k + j / 8];
            const int sh = 4 * (j % 8) - 2;
            const u32 x = sh < 0 ? wd << 2 : wd >> sh;
            t[j] = ((lds_cfloat_ptr)(uintptr_t)((x & 60u) | t_base))[(k * 8 + j) * PAG_NCODE];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) S = S + t[j];
    }
    return S;
}

// NQ: chunks of a stored vector per lane (a chunk is what one lane loads at once); NW: entries of
// W / R_L per lane; VM: how the store is read -- 0: fp32, 16-byte chunks of 4 elements; 1: 16-bit
// floats, 16-byte chunks of 8 elements; 2: 16-bit floats, 8-byte chunks of 4 elements (for row
// lengths that would leave half of the lanes idle in the last 16-byte chunk); 16-bit values are
// widened to fp32 on use; CW: dwords of 4-bit codes per neighbour (2, 4 or 8 for up to 16, 32 or
// 64 subspaces).
template <int NQ, int NW, int VM, int CW>
struct Wave {
    static constexpr bool HALF = VM != 0;
    static constexpr int EPC = VM == 1 ? 8 : 4;     // elements per chunk
    using Chunk = std::conditional_t<VM == 2, uint2, uint4>;
    // constant for the kernel
    const SearchArgs A;
    const int lane;
    float* T;
    u32 t_base;                     // LDS byte address of T
    u32* H;
    u32* BL;
    u64 *SA, *SB, *RF, *RT;
    u32* bitmap;
    // per query
    static constexpr int QV = NQ * EPC / 4;         // float4 registers holding the query
    static constexpr bool RINGS_IN_HBM = NW > 2;    // matches the host's LDS carve-up
    static constexpr bool BIG = NW > 2;             // large working sets: W unsorted, see admit_unsorted
    u64 wmax;                       // BIG: key of W's farthest member, valid while nW == b
    u64 nx_key;                     // BIG: key of the node to expand next (PAG_KEY_INVALID: W has no unvisited node)
    bool nx_known;                  // BIG: nx_key is up to date
    u64 GM, GU;                     // BIG: lane s < NW holds slot s's farthest member (0: slot empty) and its closest
                                    // unvisited member (PAG_KEY_INVALID: none); the other lanes hold 0 / PAG_KEY_INVALID
    float4 q[QV];
    u64 W[NW];
    u64 RL[NW > 2 ? 1 : NW];        // unused for large working sets: their R_L is SA[0, nRL)
    u32 nW, nRL;
    u32 cntF, hdF, cntT, hdT;       // rings: valid entries (<= b) and total pushes; slot = push number & ring mask
    u32 n_hash, n_spill;
    // The last TAILS chunk rows of the NQ may lie partly or wholly beyond the end of a row (the host
    // picks NQ = the rows needed, or one more where that count is not instantiated): per such chunk the
    // index this lane reads (0 if past the end) and a mask (all ones if inside the row, else zero)
    static constexpr int TAILS = NQ >= 5 ? 2 : 1;
    u32 tail_idx[TAILS];
    u32 tail_mask[TAILS];
    // adjacency record requested ahead of time for the node that will be expanded next
    u32 nx_id;                      // whose record pf_* holds (PAG_EMPTY: none)
    u32 pf_id, pf_cw[CW];
    float pf_a, pf_c;
    u64 Hk;                         // indexing: PES buffer H(v), lane i = i-th closest surviving node (Alg. 1)
    // statistics (wave-uniform)
    u32 s_hops, s_tests, s_passes, s_exact, s_rounds, s_rf, s_rt, s_spill, s_queries;
#ifdef PAG_PHASE_TIMERS
    u64 s_phase[6];
    u64 t_last;
#endif

    __device__ Wave(const SearchArgs& a, unsigned char* smem, int ln) : A(a), lane(ln) {
        T = (float*)smem;
        t_base = (u32)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
        H = (u32*)(smem + a.off_hash);
        BL = (u32*)(smem + a.off_bloom);
        SA = (u64*)(smem + a.off_sa);
        SB = (u64*)(smem + a.off_sb);
        if constexpr (RINGS_IN_HBM) {
            RF = a.rings + (u64)blockIdx.x * 3 * (u64)(a.ring_mask + 1);
            RT = RF + (a.ring_mask + 1);
            SA = RT + (a.ring_mask + 1);      // R_L of large working sets: b <= ring_mask + 1 keys
            SB = nullptr;
        } else {
            RF = (u64*)(smem + a.off_rf);
            RT = (u64*)(smem + a.off_rt);
        }
        bitmap = a.bitmap + (u64)blockIdx.x * a.bitmap_words;
#pragma unroll
        for (int t = 0; t < TAILS; ++t) {
            const u32 idx = (u32)(NQ - TAILS + t) * 64 + (u32)ln;
            const bool tail_ok = idx * (u32)EPC < a.d;
            tail_idx[t] = tail_ok ? idx : 0u;
            tail_mask[t] = tail_ok ? 0xFFFFFFFFu : 0u;
        }
        s_hops = s_tests = s_passes = s_exact = s_rounds = s_rf = s_rt = s_spill = s_queries = 0;
#ifdef PAG_PHASE_TIMERS
        for (int i = 0; i < 6; ++i) s_phase[i] = 0;
        t_last = wall_clock64();
#endif
    }

    // Wave priorities within the SIMD, used with the 16-bit store only: requesting rows comes first (3),
    // then the screening that leads to the requests (2), then the distance arithmetic (1), and the
    // bookkeeping of the merge last (0).  With short rows this is worth 9 %; with fp32 rows, where
    // memory throughput binds, it is not (and costs 1 % on long rows), so there it is left out.
    __device__ __forceinline__ void set_priority(int p) const {
        if constexpr (HALF) {
            if (p == 3) __builtin_amdgcn_s_setprio(3);
            else if (p == 2) __builtin_amdgcn_s_setprio(2);
            else if (p == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
    }

    // lane s < deg reads neighbour slot s of node u: id, a, c and its chunk of 4-bit codes.  The
    // other lanes read slot 0 and get an empty id (their a, c and codes are never used), so the
    // loads sit in straight-line code and can stay in flight across whatever follows.
    __device__ __forceinline__ void load_record(u32 u, u32& id, float& ea, float& ec, u32 (&cwv)[CW]) const {
        const uint8_t* rec = A.rec + (u64)u * A.rec_bytes;
        const bool in = (u32)lane < A.deg;
        const u32 sl = in ? (u32)lane : 0u;
        const u32 raw = ((const u32*)rec)[sl];
        id = in ? raw : PAG_EMPTY;
        ea = ((const float*)(rec + A.off_a))[sl];
        ec = ((const float*)(rec + A.off_c))[sl];
        const u32* cp = (const u32*)(rec + A.off_codes) + sl * CW;   // 16-byte aligned section
        if constexpr (CW == 2) {
            const uint2 t = *(const uint2*)cp;
            cwv[0] = t.x; cwv[1] = t.y;
        } else {
#pragma unroll
            for (int k = 0; k < CW; k += 4) {
                const uint4 t = *(const uint4*)(cp + k);
                cwv[k] = t.x; cwv[k + 1] = t.y; cwv[k + 2] = t.z; cwv[k + 3] = t.w;
            }
        }
    }

    // The node expanded next is the unvisited entry with the smallest rank after the merge: either the
    // first unvisited member of W or the smallest passer.  Both are known before W is physically
    // rebuilt, so its adjacency record is requested here and arrives while the merge completes.
    __device__ __forceinline__ void request_next(const u32 (&cntW)[NW], bool pass, u32 cP, u32 rP, u32 id_lane) {
        const u32 b = A.b;
        u32 best_r = 0xFFFFFFFFu, best_id = PAG_EMPTY;
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            const u32 idx = s * 64 + lane;
            const u32 r = idx + cntW[s];
            const u64 m = __ballot(idx < nW && !(W[s] & 1ull) && r < b);
            if (m && best_r == 0xFFFFFFFFu) {
                const int l = __ffsll((long long)m) - 1;
                best_r = rdlane(r, l);
                best_id = rdlane((u32)(W[s] & 0xFFFFFFFFull), l) >> 1;
            }
        }
        const u64 m2 = __ballot(pass && cP == 0 && rP < b);
        if (m2) {
            const int l = __ffsll((long long)m2) - 1;
            const u32 r2 = rdlane(rP, l);
            if (r2 < best_r) { best_r = r2; best_id = rdlane(id_lane, l); }
        }
        nx_id = best_id;
        if (best_id != PAG_EMPTY) load_record(best_id, pf_id, pf_a, pf_c, pf_cw);
    }

    // exact keys ||q - x_id||^2 (Alg. 2, exact-distance step) for the lanes in `mask`;
    // lane p receives the key of its own id.  Differences in fp32, squares summed in fp64,
    // one rounding to fp32 at the end.  Two buffers of GB vectors each alternate: while one is
    // reduced the other one's loads are in flight.  No load sits inside a branch (a buffer without
    // a passer left simply re-reads the last row), which keeps the wait counts exact.
    static constexpr int GB = NQ * (int)sizeof(Chunk) <= 64 ? 2 : 1;

    // Branch-free row load: only the last TAILS chunks can run past the row; there the lane re-reads
    // chunk 0 (in bounds) and the value is replaced by zeros, so no load ever sits inside a branch and
    // the loads of several rows stay in flight together.
    __device__ __forceinline__ void load_vec(Chunk (&v)[NQ], u32 id) const {
        const Chunk* p = (const Chunk*)((const char*)A.vec + (u64)id * A.d * (HALF ? 2 : 4));
#pragma unroll
        for (int c = 0; c < NQ - TAILS; ++c) v[c] = p[c * 64 + lane];
#pragma unroll
        for (int t = 0; t < TAILS; ++t) {
            Chunk x = p[tail_idx[t]];
            x.x &= tail_mask[t]; x.y &= tail_mask[t];
            if constexpr (VM != 2) { x.z &= tail_mask[t]; x.w &= tail_mask[t]; }
            v[NQ - TAILS + t] = x;
        }
    }

    // sum over this lane's elements of fl32(q - x)^2, accumulated in fp64
    __device__ __forceinline__ double lane_partial(const Chunk (&v)[NQ]) const {
        double a = 0.0;
#pragma unroll
        for (int c = 0; c < NQ; ++c) {
            if constexpr (VM == 1) {
                const float2 x0 = __half22float2(*(const __half2*)&v[c].x), x1 = __half22float2(*(const __half2*)&v[c].y);
                const float2 x2 = __half22float2(*(const __half2*)&v[c].z), x3 = __half22float2(*(const __half2*)&v[c].w);
                const float d0 = q[2 * c].x - x0.x, d1 = q[2 * c].y - x0.y, d2 = q[2 * c].z - x1.x, d3 = q[2 * c].w - x1.y;
                const float d4 = q[2 * c + 1].x - x2.x, d5 = q[2 * c + 1].y - x2.y;
                const float d6 = q[2 * c + 1].z - x3.x, d7 = q[2 * c + 1].w - x3.y;
                a = __builtin_fma((double)d0, (double)d0, a); a = __builtin_fma((double)d1, (double)d1, a);
                a = __builtin_fma((double)d2, (double)d2, a); a = __builtin_fma((double)d3, (double)d3, a);
                a = __builtin_fma((double)d4, (double)d4, a); a = __builtin_fma((double)d5, (double)d5, a);
                a = __builtin_fma((double)d6, (double)d6, a); a = __builtin_fma((double)d7, (double)d7, a);
            } else if constexpr (VM == 2) {
                const float2 x0 = __half22float2(*(const __half2*)&v[c].x), x1 = __half22float2(*(const __half2*)&v[c].y);
                const float d0 = q[c].x - x0.x, d1 = q[c].y - x0.y, d2 = q[c].z - x1.x, d3 = q[c].w - x1.y;
                a = __builtin_fma((double)d0, (double)d0, a); a = __builtin_fma((double)d1, (double)d1, a);
                a = __builtin_fma((double)d2, (double)d2, a); a = __builtin_fma((double)d3, (double)d3, a);
            } else {
                const float dx = q[c].x - __uint_as_float(v[c].x), dy = q[c].y - __uint_as_float(v[c].y);
                const float dz = q[c].z - __uint_as_float(v[c].z), dw = q[c].w - __uint_as_float(v[c].w);
                a = __builtin_fma((double)dx, (double)dx, a);
                a = __builtin_fma((double)dy, (double)dy, a);
                a = __builtin_fma((double)dz, (double)dz, a);
                a = __builtin_fma((double)dw, (double)dw, a);
            }
        }
        return a;
    }

    // request the rows of the next GB passers (or, when none is left, the last row again)
    __device__ __forceinline__ void issue(Chunk (&buf)[GB][NQ], int (&pl)[GB], u64& m, int& last, u32 id_lane) const {
        set_priority(3);
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            pl[g] = -1;
            if (m) { last = __ffsll((long long)m) - 1; m &= m - 1; pl[g] = last; }
            load_vec(buf[g], rdlane(id_lane, last));
        }
        set_priority(1);
    }

    __device__ __forceinline__ void reduce(const Chunk (&buf)[GB][NQ], const int (&pl)[GB], float& mine) const {
        double acc[GB];
#pragma unroll
        for (int g = 0; g < GB; ++g) acc[g] = lane_partial(buf[g]);
        const double tot = fold_sum<GB>(acc);
#pragma unroll
        for (int g = 0; g < GB; ++g) {
            const double t = __hiloint2double((int)rdlane((u32)__double2hiint(tot), g * (64 / GB)),
                                              (int)rdlane((u32)__double2loint(tot), g * (64 / GB)));
            if (lane == pl[g]) mine = (float)t;
        }
    }

    __device__ __forceinline__ float exact_keys(u32 id_lane, u64 mask) {
        float mine = 0.f;
        Chunk va[GB][NQ], vb[GB][NQ];
        int pa[GB], pb[GB];
        u64 m = mask;
        int last = __ffsll((long long)mask) - 1;
        int left = __popcll(mask);
        issue(va, pa, m, last, id_lane);
        for (;;) {
            // the scheduling barriers keep the requests for one buffer ahead of the arithmetic on the other
            issue(vb, pb, m, last, id_lane);
            __builtin_amdgcn_sched_barrier(0);
            reduce(va, pa, mine);
            left -= GB;
            if (left <= 0) break;
            issue(va, pa, m, last, id_lane);
            __builtin_amdgcn_sched_barrier(0);
            reduce(vb, pb, mine);
            left -= GB;
            if (left <= 0) break;
        }
        return mine;
    }

    // Admission of the lanes in `mask` (ids in id_lane): exact keys, seen-set insertion, merge into W.
    __device__ __forceinline__ void admit(u32 id_lane, u64 mask) {
        const u32 np = (u32)__popcll(mask);
        if (np == 0) {
            set_priority(0);
            if constexpr (BIG) {
                look_ahead();
            } else {
                u32 zero[NW];
#pragma unroll
                for (int s = 0; s < NW; ++s) zero[s] = 0;
                request_next(zero, false, 0, 0, id_lane);
            }
            return;
        }
        const u32 b = A.b;
        const bool pass = (mask >> lane) & 1ull;
        if constexpr (BIG) {
            admit_unsorted(id_lane, mask, np, pass);
            return;
        }
        PAG_MARK(2);
        const float dist = exact_keys(id_lane, mask);
        set_priority(0);
        PAG_MARK(3);
        s_exact += np;
        // seen set
        if (A.blog != 0) {
            // long searches: every node goes to the bitmap and the Bloom filter; the LDS table keeps the
            // most recently admitted id per slot (a hit there is definite)
            if (pass) {
                H[hash_slot(id_lane, A.hlog)] = id_lane;
                atomicOr(&bitmap[id_lane >> 5], 1u << (id_lane & 31));
                bloom_set(BL, A.blog, id_lane);
            }
            n_spill += np; s_spill += np;
        } else {
            // short searches: exact open-addressing hash, kept at most half full; beyond that the bitmap
            const bool spill = (n_hash + np) > (1u << (A.hlog - 1));
            if (pass) {
                if (!spill) hash_insert(H, A.hlog, id_lane);
                else atomicOr(&bitmap[id_lane >> 5], 1u << (id_lane & 31));
            }
            if (spill) { n_spill += np; s_spill += np; } else n_hash += np;
        }

        const u64 pk = pass ? (((u64)__float_as_uint(dist) << 32) | ((u64)id_lane << 1)) : PAG_KEY_INVALID;
        u32 cntW[NW];
#pragma unroll
        for (int s = 0; s < NW; ++s) cntW[s] = 0;
        u32 cP = 0, cPW = 0;
        for (u64 m = mask; m;) {
            const int p = __ffsll((long long)m) - 1;
            m &= m - 1;
            const u64 k = rdlane64(pk, p);
            u32 c = 0;
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                // keys are distinct, so one comparison tells both sides (an empty slot counts as larger)
                const bool lt = W[s] < k;
                c += (u32)__popcll(__ballot(lt));
                cntW[s] += lt ? 0u : 1u;
            }
            cP += (k < pk) ? 1u : 0u;
            if (lane == p) cPW = c;
        }
        const u32 total = nW + np;
        const u32 nW2 = total < b ? total : b;
        const u32 rP = cP + cPW;                                   // merged rank of my passer
        const u32 n_ins = (u32)__popcll(__ballot(pass && rP < b)); // passers that enter W
        const u32 n_f = np - n_ins;                                // false positives -> R_F
        const u32 n_ej = nW + n_ins - nW2;                         // displaced members -> R_T
        request_next(cntW, pass, cP, rP, id_lane);
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            const u32 idx = s * 64 + lane;
            if (idx < nW) {
                const u32 r = idx + cntW[s];
                if (r < b) SA[r] = W[s];
                else RT[(hdT + (nW - 1 - idx)) & A.ring_mask] = W[s];   // largest first
            }
        }
        if (pass) {
            if (rP < b) SA[rP] = pk;
            else {
                const u32 oi = cP - n_ins;                          // smallest first
                if (oi + b >= n_f) RF[(hdF + oi) & A.ring_mask] = pk;  // older ones would be overwritten anyway
            }
        }
        if (n_ej) {
            if (cntT + n_ej > b) s_rt += cntT + n_ej - b;
            cntT = cntT + n_ej < b ? cntT + n_ej : b;
            hdT += n_ej;
        }
        if (n_f) {
            if (cntF + n_f > b) s_rf += cntF + n_f - b;
            cntF = cntF + n_f < b ? cntF + n_f : b;
            hdF += n_f;
        }
        lds_sync();
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            const u32 idx = s * 64 + lane;
            W[s] = idx < nW2 ? SA[idx] : PAG_KEY_INVALID;
        }
        nW = nW2;
        lds_sync();
        PAG_MARK(4);
    }

    // ---- working sets above 128 nodes (NW >= 4): W is kept unsorted ----
    // Keeping up to 1024 keys sorted by rank costs a pass over all NW slots per passer and a round trip of the
    // whole set through LDS per hop.  What a hop needs of W is only its closest unvisited member, its farthest
    // member and the replacement of that one; the order of the rest matters at the round's end alone, where
    // everything is sorted anyway.

    // Keys are distance bits over (id << 1 | visited): an extreme key is found in two 32-bit steps -- the extreme
    // distance, then the extreme low word among the members at that distance -- each a handful of DPP
    // instructions, where a 64-bit reduction moves and compares register pairs.
    // W's slots (one register per lane each) keep their extremes in GM / GU, so that finding W's farthest member or
    // its closest unvisited one is a reduction over NW <= 16 lanes, and a change of one member costs a reduction over
    // that member's slot alone, reached through a uniform branch.

    // farthest member of slot S (0 if the slot is empty)
    template <int S>
    __device__ __forceinline__ u64 slot_max() const {
        const bool valid = (u32)(S * 64 + lane) < nW;
        const u32 hi = valid ? (u32)(W[S] >> 32) : 0u;
        const u32 mh = wave_extreme_u32<true>(hi);
        const u32 lo = (valid && hi == mh) ? (u32)W[S] : 0u;
        return ((u64)mh << 32) | wave_extreme_u32<true>(lo);
    }

    // closest unvisited member of slot S (PAG_KEY_INVALID if there is none)
    template <int S>
    __device__ __forceinline__ u64 slot_min_unvisited() const {
        const bool ok = (u32)(S * 64 + lane) < nW && !(W[S] & 1ull);
        const u32 hi = ok ? (u32)(W[S] >> 32) : 0xFFFFFFFFu;
        const u32 mh = wave_extreme_u32<false>(hi);
        const u32 lo = (ok && hi == mh) ? (u32)W[S] : 0xFFFFFFFFu;      // distances are finite: no member carries mh = ~0
        return ((u64)mh << 32) | wave_extreme_u32<false>(lo);
    }

    // extreme over the slots: lanes 0 .. NW - 1 of GM (MAX) or GU
    template <bool MAX>
    __device__ __forceinline__ u64 over_slots(u64 v) const {
        const u32 neutral = MAX ? 0u : 0xFFFFFFFFu;
        const u32 mh = row0_extreme_u32<MAX>((u32)(v >> 32));
        const u32 lo = (u32)(v >> 32) == mh ? (u32)v : neutral;
        return ((u64)mh << 32) | row0_extreme_u32<MAX>(lo);
    }

    // runs f(slot) for the one slot g (uniform), with the slot number as a compile-time constant
    template <int S = 0, class F>
    __device__ __forceinline__ void at_slot(int g, F&& f) {
        if constexpr (S < NW) {
            if (g == S) f(std::integral_constant<int, S>{});
            else at_slot<S + 1>(g, f);
        }
    }

    // finds the node that will be expanded next and requests its adjacency record
    __device__ __forceinline__ void look_ahead() {
        nx_key = over_slots<false>(GU);
        nx_known = true;
        nx_id = PAG_EMPTY;
        if (nx_key != PAG_KEY_INVALID) {
            nx_id = (u32)(nx_key & 0xFFFFFFFFull) >> 1;
            load_record(nx_id, pf_id, pf_a, pf_c, pf_cw);
        }
    }

    // Admission into an unsorted W.  The hop's passers are taken in ascending (dist, id) order, exactly as Alg. 2
    // admits them one after the other: while W has room a passer is appended; then a passer closer than W's
    // farthest member takes that member's place and the member goes to R_T; the first passer that is not closer
    // ends it -- the farthest member can only have come closer since, and the remaining passers are no smaller --,
    // and that passer and all after it go to R_F.
    __device__ __forceinline__ void admit_unsorted(u32 id_lane, u64 mask, u32 np, bool pass) {
        const u32 b = A.b;
        PAG_MARK(2);
        const float dist = exact_keys(id_lane, mask);
        set_priority(0);
        PAG_MARK(3);
        s_exact += np;
        if (A.blog != 0) {
            if (pass) {
                H[hash_slot(id_lane, A.hlog)] = id_lane;
                atomicOr(&bitmap[id_lane >> 5], 1u << (id_lane & 31));
                bloom_set(BL, A.blog, id_lane);
            }
            n_spill += np; s_spill += np;
        } else {
            const bool spill = (n_hash + np) > (1u << (A.hlog - 1));
            if (pass) {
                if (!spill) hash_insert(H, A.hlog, id_lane);
                else atomicOr(&bitmap[id_lane >> 5], 1u << (id_lane & 31));
            }
            if (spill) { n_spill += np; s_spill += np; } else n_hash += np;
        }
        const u64 pk = pass ? (((u64)__float_as_uint(dist) << 32) | ((u64)id_lane << 1)) : PAG_KEY_INVALID;
        // rank of my passer among the hop's passers (keys are distinct)
        u32 cP = 0;
        for (u64 m = mask; m;) {
            const int p = __ffsll((long long)m) - 1;
            m &= m - 1;
            cP += (rdlane64(pk, p) < pk) ? 1u : 0u;
        }
        u32 n_ej = 0, j = 0;
        for (; j < np; ++j) {
            const int src = __ffsll((long long)__ballot(pass && cP == j)) - 1;
            const u64 k = rdlane64(pk, src);
            if (nW < b) {
                const int slot = (int)(nW >> 6), ln = (int)(nW & 63u);
                at_slot(slot, [&](auto S_) { constexpr int S = decltype(S_)::value; if (lane == ln) W[S] = k; });
                if (lane == slot) { GM = k > GM ? k : GM; GU = k < GU ? k : GU; }
                nW++;
                if (nW == b) wmax = over_slots<true>(GM);
            } else if (k < wmax) {
                // the farthest member leaves for R_T (pushes of one hop: farthest first), the passer takes its place
                if (lane == 0) RT[(hdT + n_ej) & A.ring_mask] = wmax;
                n_ej++;
                const int g = __ffsll((long long)__ballot(GM == wmax)) - 1;       // its slot
                at_slot(g, [&](auto S_) {
                    constexpr int S = decltype(S_)::value;
                    if (W[S] == wmax) W[S] = k;
                    const u64 m = slot_max<S>();
                    if (lane == S) GM = m;
                });
                // the slot's closest unvisited member: the one that left was it only if it was the slot's last
                if (lane == g) GU = (GU == wmax) ? k : (k < GU ? k : GU);
                wmax = over_slots<true>(GM);
            } else {
                break;
            }
        }
        const u32 n_f = np - j;                                     // false positives -> R_F, smallest first
        if (pass && cP >= j) {
            const u32 oi = cP - j;
            if (oi + b >= n_f) RF[(hdF + oi) & A.ring_mask] = pk;   // older ones would be overwritten anyway
        }
        if (n_ej) {
            if (cntT + n_ej > b) s_rt += cntT + n_ej - b;
            cntT = cntT + n_ej < b ? cntT + n_ej : b;
            hdT += n_ej;
        }
        if (n_f) {
            if (cntF + n_f > b) s_rf += cntF + n_f - b;
            cntF = cntF + n_f < b ? cntF + n_f : b;
            hdF += n_f;
        }
        look_ahead();
        PAG_MARK(4);
    }

    __device__ __forceinline__ void run_query(u32 qi) {
        const u32 d = A.d, b = A.b, deg = A.deg;
        // ---- load query, table, reset state ----
        {
            const float4* qp = (const float4*)(A.qrot + (u64)qi * d);
#pragma unroll
            for (int c = 0; c < NQ; ++c) {
                const u32 idx = c * 64 + lane;
                if constexpr (VM == 1) {
                    const bool in = c < NQ - TAILS || idx * 8 < d;
                    q[2 * c] = in ? qp[2 * idx] : make_float4(0.f, 0.f, 0.f, 0.f);
                    q[2 * c + 1] = in ? qp[2 * idx + 1] : make_float4(0.f, 0.f, 0.f, 0.f);
                } else {
                    q[c] = (c < NQ - TAILS || idx * 4 < d) ? qp[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            const float4* tp = (const float4*)(A.tables + (u64)qi * A.Ppad * PAG_NCODE);
            for (u32 i = lane; i < A.Ppad * PAG_NCODE / 4; i += 64) ((float4*)T)[i] = tp[i];
            const uint4 e4 = make_uint4(PAG_EMPTY, PAG_EMPTY, PAG_EMPTY, PAG_EMPTY);
            for (u32 i = lane; i < (1u << A.hlog) / 4; i += 64) ((uint4*)H)[i] = e4;
            if (A.blog) {
                const uint4 z4 = make_uint4(0, 0, 0, 0);
                for (u32 i = lane; i < (1u << A.blog) / 128; i += 64) ((uint4*)BL)[i] = z4;
            }
#pragma unroll
            for (int s = 0; s < NW; ++s) W[s] = PAG_KEY_INVALID;
#pragma unroll
            for (int s = 0; s < (BIG ? 1 : NW); ++s) RL[s] = PAG_KEY_INVALID;
            nW = nRL = 0;
            cntF = hdF = cntT = hdT = 0;
            n_hash = n_spill = 0;
            Hk = PAG_KEY_INVALID;
            nx_id = PAG_EMPTY;
            wmax = 0; nx_key = PAG_KEY_INVALID; nx_known = false;
            GM = 0ull; GU = PAG_KEY_INVALID;
            __syncthreads();
        }
        s_queries++;
        u32 n_cand = 0;   // indexing mode: entries of R_L written so far

        // ---- b entry nodes (Alg. 2, entry step) ----
        {
            u32 ne = A.n_entry < b ? A.n_entry : b;
            for (u32 base = 0; base < ne; base += 64) {
                const u32 i = base + lane;
                u32 id = PAG_EMPTY;
                if (i < ne) id = A.entry[i];
                const bool ok = id != PAG_EMPTY && id < A.n_limit;
                admit(id, __ballot(ok));
            }
        }

        // ---- rounds ----
        for (u32 r = 0; r < A.Rmax; ++r) {
            if (nW == 0) break;
            s_rounds++;
            for (;;) {
                // closest unvisited member of W
                u64 ukey = 0;
                if constexpr (BIG) {
                    if (!nx_known) nx_key = over_slots<false>(GU);
                    nx_known = false;
                    if (nx_key == PAG_KEY_INVALID) break;
                    PAG_MARK(5);
                    ukey = nx_key;
                    const int g = __ffsll((long long)__ballot(GU == ukey)) - 1;        // its slot
                    at_slot(g, [&](auto S_) {
                        constexpr int S = decltype(S_)::value;
                        if (W[S] == ukey) W[S] |= 1ull;
                        const u64 m = slot_min_unvisited<S>();
                        if (lane == S) GU = m;
                    });
                    if (GM == ukey) GM |= 1ull;                                         // it may be its slot's farthest too
                    if (nW == b && (wmax | 1ull) == (ukey | 1ull)) wmax |= 1ull;
                } else {
                    int us = -1, ul = 0;
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        const u32 idx = s * 64 + lane;
                        const u64 m = __ballot(idx < nW && !(W[s] & 1ull));
                        if (us < 0 && m) { us = s; ul = __ffsll((long long)m) - 1; }
                    }
                    if (us < 0) break;
                    PAG_MARK(5);
#pragma unroll
                    for (int s = 0; s < NW; ++s)
                        if (s == us) {
                            ukey = rdlane64(W[s], ul);
                            if (lane == ul) W[s] |= 1ull;
                        }
                }
                s_hops++;
                set_priority(2);   // screening leads to the next loads: ahead of other waves' bookkeeping
                const u32 u = (u32)(ukey & 0xFFFFFFFFull) >> 1;
                const float Du = __uint_as_float((u32)(ukey >> 32));
                // threshold ||z_max - q||^2, read once per hop (Eq. 4); +inf while W is not full
                float Dmax = __builtin_inff();
                if (nW == b) {
                    if constexpr (BIG) {
                        Dmax = __uint_as_float((u32)(wmax >> 32));
                    } else {
                        const u32 wr = b - 1;
#pragma unroll
                        for (int s = 0; s < NW; ++s)
                            if ((int)(wr >> 6) == s) Dmax = __uint_as_float(rdlane((u32)(W[s] >> 32), wr & 63));
                    }
                }
                PAG_MARK(0);
                // adjacency record of u: normally already on its way (see request_next)
                u32 id;
                float ea, ec;
                u32 cwv[CW];
                if (u == nx_id) {
                    id = pf_id; ea = pf_a; ec = pf_c;
#pragma unroll
                    for (int k = 0; k < CW; ++k) cwv[k] = pf_cw[k];
                } else {
                    load_record(u, id, ea, ec, cwv);
                }
                nx_id = PAG_EMPTY;
                PAG_MARK(1);
                const bool in_graph = id != PAG_EMPTY && id < A.n_limit;
                // seen-set lookup.  Short searches: the exact LDS hash, then the bitmap word if the hash has
                // overflowed, requested now and consumed after the table sums.  Long searches: the LDS cache of
                // recent ids now; the Bloom filter and the bitmap only for the neighbours that pass the test
                // (a bitmap read costs more than the table sums of the seen neighbours it would spare).
                bool cand = in_graph;
                if (cand) cand = A.blog != 0 ? H[hash_slot(id, A.hlog)] != id : !hash_contains(H, A.hlog, id);
                u32 bm_word = 0;
                if (A.blog == 0 && n_spill && cand)
                    bm_word = __hip_atomic_load(&bitmap[id >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // counting mode of long searches: the second level is consulted for every neighbour, before the
                // test, so that `tests` counts the unseen neighbours only (same results, more bitmap reads)
                const bool resolve_first = A.blog != 0 && (A.flags & PAG_FLAG_EXACT_TEST_COUNT);
                if (resolve_first) {
                    u32 wd = 0;
                    if (cand && bloom_maybe(BL, A.blog, id))
                        wd = __hip_atomic_load(&bitmap[id >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    cand = cand && !((wd >> (id & 31)) & 1u);
                }
                // projection test: S = sum_l T[l][code_l] (increasing l), est = D_u + c - 2 a S
                float est = 0.f;
                const bool want_pes = A.pes != nullptr;   // indexing: every neighbour's estimate feeds Eq. 5
                if (!(A.flags & PAG_FLAG_NO_PRT)) {
                    float S = 0.f;
                    if (cand || (want_pes && in_graph)) {
                        S = table_sum<CW>(t_base, cwv);
                    }
                    est = __builtin_fmaf(-2.0f * ea, S, Du + ec);
                }
                if (A.blog != 0 && !resolve_first) {
                    // long searches: only neighbours that pass the test are looked up in the Bloom filter and the bitmap
                    const bool maybe = cand && ((A.flags & PAG_FLAG_NO_PRT) || est < Dmax) && bloom_maybe(BL, A.blog, id);
                    if (maybe) bm_word = __hip_atomic_load(&bitmap[id >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                const bool unseen = cand && !((bm_word >> (id & 31)) & 1u);
                bool pass = unseen;
                if (!(A.flags & PAG_FLAG_NO_PRT)) pass = unseen && (est < Dmax);
                if (A.blog == 0) cand = unseen;
                if (want_pes) {
                    // PES screening (Eq. 5): max_i (cos theta_i / cos beta_i - delta_i) < 0 for all neighbours
                    // <=> every estimate est_i exceeds D_u, i.e. no neighbour of u looks closer to v than
                    // u itself.  Then u -> v is a candidate edge; H(v) keeps the closest `deg` such nodes.
                    if (__ballot(in_graph && !(est > Du)) == 0ull) {
                        const u64 key = (ukey & ~1ull);
                        const u32 pos = (u32)__popcll(__ballot(Hk < key));
                        const u64 up = __shfl_up(Hk, 1, 64);
                        if ((u32)lane == pos) Hk = key;
                        else if ((u32)lane > pos) Hk = up;
                    }
                }
                if (A.flags & PAG_SEARCH_DISTINCT) {
                    // searches that overlap an insertion: a record read between two states of a reverse-edge pass may
                    // list one node in two slots; the first slot stands, the merge needs distinct keys
                    for (u64 m = __ballot(pass); m;) {
                        const int p = __ffsll((long long)m) - 1;
                        m &= m - 1;
                        if (lane > p && id == rdlane(id, p)) { pass = false; cand = false; }
                    }
                }
                const u64 cmask = __ballot(cand);
                const u64 pmask = __ballot(pass);
                s_tests += (u32)__popcll(cmask);
                s_passes += (u32)__popcll(pmask);
                admit(id, pmask);
            }

            // ---- round end (Alg. 2): W -> R_L, clear W; merge + sort rings; refill W; rest -> R_T ----
            nx_id = PAG_EMPTY;
            if (A.cand) {
                // indexing: R_L has room for every round's W (capacity efC >= Rmax * b is enforced by the host)
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    if (idx < nW && n_cand + idx < A.cand_cap) A.cand[(u64)qi * A.cand_cap + n_cand + idx] = W[s];
                }
                n_cand = n_cand + nW < A.cand_cap ? n_cand + nW : A.cand_cap;
            } else if constexpr (BIG) {
                // R_L <- best K of R_L + W: R_L (sorted, SA[0, nRL) in HBM) and W are sorted together in registers
                u64 x[2 * NW];
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    x[s] = idx < nW ? W[s] : PAG_KEY_INVALID;
                    x[NW + s] = idx < nRL ? SA[idx] : PAG_KEY_INVALID;
                }
                bitonic_registers<2 * NW>(x, lane);
                const u32 n = nRL + nW;
                nRL = n < A.K ? n : A.K;
#pragma unroll
                for (int s = 0; s < NW; ++s) {                  // K <= b <= 64 NW
                    const u32 idx = s * 64 + lane;
                    if (idx < nRL) SA[idx] = x[s];
                }
            } else {
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    if (idx < nRL) SA[idx] = RL[s];
                    if (idx < nW) SA[nRL + idx] = W[s];
                }
                lds_sync();
                const u32 n = nRL + nW;
                const u64* S = sort_keys(SA, SB, n, 2 * b <= PAG_RANK_SORT_MAX, lane);
                nRL = n < A.K ? n : A.K;
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    RL[s] = idx < nRL ? S[idx] : PAG_KEY_INVALID;
                }
                lds_sync();
            }
            if constexpr (BIG) {
                // this wave's own stores (ring pushes, R_L) must have landed before other lanes read them
                __threadfence();
                const u32 n = cntF + cntT;                       // <= 2b <= 128 NW
                u64 x[2 * NW];
#pragma unroll
                for (int s = 0; s < 2 * NW; ++s) {
                    const u32 i = s * 64 + lane;
                    u64 k = PAG_KEY_INVALID;
                    if (i < cntF) k = RF[(hdF - cntF + i) & A.ring_mask];
                    else if (i < n) k = RT[(hdT - cntT + (i - cntF)) & A.ring_mask];
                    x[s] = k;
                }
                bitonic_registers<2 * NW>(x, lane);
                nW = n < b ? n : b;
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    W[s] = idx < nW ? x[s] : PAG_KEY_INVALID;
                }
                // W is sorted now: a slot's farthest member is its last, its closest unvisited one the first unvisited
                GM = 0ull; GU = PAG_KEY_INVALID;
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 first = s * 64;
                    if (nW > first) {
                        const u32 cnt = nW - first < 64u ? nW - first : 64u;
                        const u64 far = rdlane64(W[s], (int)cnt - 1);
                        const u64 open = __ballot((u32)lane < cnt && !(W[s] & 1ull));
                        const u64 near = open ? rdlane64(W[s], __ffsll((long long)open) - 1) : PAG_KEY_INVALID;
                        if (lane == s) { GM = far; GU = near; }
                    }
                }
                wmax = nW == b ? over_slots<true>(GM) : 0ull;
                nx_known = false;
                const u32 rest = n - nW;                         // <= b; written worst first
#pragma unroll
                for (int s = 0; s < 2 * NW; ++s) {
                    const u32 e = s * 64 + lane;
                    if (e >= nW && e < n) RT[n - 1 - e] = x[s];
                }
                cntT = rest; hdT = rest;
                cntF = 0; hdF = 0;
            } else {
                for (u32 i = lane; i < cntF; i += 64) SA[i] = RF[(hdF - cntF + i) & A.ring_mask];
                for (u32 i = lane; i < cntT; i += 64) SA[cntF + i] = RT[(hdT - cntT + i) & A.ring_mask];
                lds_sync();
                const u32 n = cntF + cntT;
                const u64* S = sort_keys(SA, SB, n, 2 * b <= PAG_RANK_SORT_MAX, lane);
                nW = n < b ? n : b;
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const u32 idx = s * 64 + lane;
                    W[s] = idx < nW ? S[idx] : PAG_KEY_INVALID;
                }
                const u32 rest = n - nW;                         // <= b; written worst first
                for (u32 j = lane; j < rest; j += 64) RT[j] = S[n - 1 - j];
                cntT = rest; hdT = rest;
                cntF = 0; hdF = 0;
                lds_sync();
            }
        }

        // ---- output ----
        if (A.cand) {
            if (lane == 0) A.cand_cnt[qi] = n_cand;
            if (A.pes && (u32)lane < deg) A.pes[(u64)qi * deg + lane] = Hk;
        } else {
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                const u32 idx = s * 64 + lane;
                if (idx < A.K) {
                    long long oid = -1;
                    float od = __builtin_inff();
                    if (idx < nRL) {
                        u64 key;
                        if constexpr (BIG) key = SA[idx];
                        else key = RL[s];
                        oid = (long long)((u32)(key & 0xFFFFFFFFull) >> 1);
                        od = A.out_scale * __uint_as_float((u32)(key >> 32));
                    }
                    A.out_ids[(u64)qi * A.K + idx] = oid;
                    A.out_dists[(u64)qi * A.K + idx] = od;
                }
            }
        }
        // a spilled query leaves its bitmap clean for the next one
        if (n_spill) {
            uint4* bm = (uint4*)bitmap;
            const uint4 z = make_uint4(0, 0, 0, 0);
            for (u64 i = lane; i < A.bitmap_words / 4; i += 64) bm[i] = z;
            __threadfence();
        }
    }

    __device__ __forceinline__ void flush_stats() {
        if (lane == 0) {
            atomicAdd(&A.counters[CTR_QUERIES], (u64)s_queries);
            atomicAdd(&A.counters[CTR_HOPS], (u64)s_hops);
            atomicAdd(&A.counters[CTR_TESTS], (u64)s_tests);
            atomicAdd(&A.counters[CTR_PASSES], (u64)s_passes);
            atomicAdd(&A.counters[CTR_EXACT], (u64)s_exact);
            atomicAdd(&A.counters[CTR_ROUNDS], (u64)s_rounds);
            atomicAdd(&A.counters[CTR_RF_OVER], (u64)s_rf);
            atomicAdd(&A.counters[CTR_RT_OVER], (u64)s_rt);
            atomicAdd(&A.counters[CTR_SPILLS], (u64)s_spill);
#ifdef PAG_PHASE_TIMERS
            for (int i = 0; i < 6; ++i) atomicAdd(&A.counters[CTR_PHASE0 + i], s_phase[i]);
#endif
        }
    }
};

// Persistent waves: every wave pulls query numbers from one counter until the batch is drained,
// so long and short searches balance themselves; the loop ends for every wave once the counter
// passes nq.
template <int NQ, int NW, int VM, int CW>
// Short rows leave room for four waves per SIMD (128 VGPRs, a few dwords of spill); longer rows
// keep their registers for loads in flight.  Working sets above 128 nodes hold W in 4 NW registers per lane:
// three waves per SIMD up to 512 nodes, two for 1024 (measured: a third wave there spills W and costs 50 %).
__attribute__((amdgpu_waves_per_eu(VM == 2 && NQ <= 3 && NW <= 2 ? 5 : (NQ <= 3 && NW <= 2 ? 4 : (NQ <= 4 && NW > 2 ? (NW >= 16 ? 2 : 3) : 1)), 8)))
__global__ void __launch_bounds__(64) k_search(const SearchArgs A) {
    extern __shared__ __align__(64) unsigned char smem[];   // the table sits first: see table_sum
    const int lane = threadIdx.x;
    Wave<NQ, NW, VM, CW> w(A, smem, lane);
    for (;;) {
        u32 qi = 0;
        if (lane == 0) qi = atomicAdd(A.qcounter, 1u);
        qi = uniform(qi);
        if (qi >= A.nq) break;
        if (A.order) qi = A.order[qi];
        w.run_query(qi);
    }
    w.flush_stats();
}

}  // namespace pagk

// One translation unit per (NQ, CW) defines the selector below: the kernels for every number of
// W / R_L entries per lane (working sets of up to 64, 128, 256, 512, 1024 nodes) and the three ways of reading the store.
typedef void (*pag_search_fn)(const SearchArgs);
#define PAG_SEARCH_INSTANCES(NQ, CW)                                                                  \
    template <int VM>                                                                                 \
    static pag_search_fn pag_search_by_nw(int nw) {                                                   \
        switch (nw) {                                                                                 \
            case 1: return (pag_search_fn)pagk::k_search<NQ, 1, VM, CW>;                              \
            case 2: return (pag_search_fn)pagk::k_search<NQ, 2, VM, CW>;                              \
            case 4: return (pag_search_fn)pagk::k_search<NQ, 4, VM, CW>;                              \
            case 8: return (pag_search_fn)pagk::k_search<NQ, 8, VM, CW>;                              \
            case 16: return (pag_search_fn)pagk::k_search<NQ, 16, VM, CW>;                            \
            default: return nullptr;                                                                  \
        }                                                                                             \
    }                                                                                                 \
    pag_search_fn pag_search_fn_nq##NQ##_cw##CW(int nw, int vm) {                                     \
        return vm == 0 ? pag_search_by_nw<0>(nw) : (vm == 1 ? pag_search_by_nw<1>(nw) : pag_search_by_nw<2>(nw)); \
    }
