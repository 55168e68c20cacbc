// Batch-synchronous index construction and online insertion (Alg. 1, Step 1; Sec. 4.1).
//
// The paper inserts nodes one after another.  Here a batch of new nodes searches the graph built
// so far concurrently (the same PRT-TFB search kernel as for queries, with ef = efC,
// b = min(efC, 100) and R_L collecting every round's W), then
//   1. RobustPrune (Eq. 1, alpha = 1) over each node's R_L gives N_out(v);
//   2. the reverse edges (u <- v for u in N_out(v)) are grouped by target with a radix sort and
//      one wave per target applies them in ascending (distance, id) order;
//   3. the inference information (codes, a, c) of every new or moved edge is recomputed.
// Batches start small and grow with the graph so that early nodes see most of their peers.
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "pag_internal.h"
#include "pag_wave.h"

namespace {

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// squared distance between the vector staged in LDS and row `id`, all lanes get the result
__device__ __forceinline__ float dist_lds(const pag_vecs& V, u32 d, const float* s, u32 id, int lane) {
    const float4* q = (const float4*)s;
    double acc = 0.0;
    for (u32 c = lane; c < d / 4; c += 64) {
        const float4 a = q[c], b = pag_vload4(V, id, c);
        const float dx = a.x - b.x, dy = a.y - b.y, dz = a.z - b.z, dw = a.w - b.w;
        acc = __builtin_fma((double)dx, (double)dx, acc);
        acc = __builtin_fma((double)dy, (double)dy, acc);
        acc = __builtin_fma((double)dz, (double)dz, acc);
        acc = __builtin_fma((double)dw, (double)dw, acc);
    }
    return (float)wave_sum(acc);
}

// squared distances between the vector staged in LDS and four rows at once (their loads are in
// flight together); all lanes get all four results
__device__ __forceinline__ void dist_lds4(const pag_vecs& V, u32 d, const float* s, const u32 (&id)[4], float (&out)[4]) {
    const float4* q = (const float4*)s;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (u32 c = threadIdx.x; c < d / 4; c += 64) {
        const float4 a = q[c];
        float4 b[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) b[g] = pag_vload4(V, id[g], c);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float dx = a.x - b[g].x, dy = a.y - b[g].y, dz = a.z - b[g].z, dw = a.w - b[g].w;
            acc[g] = __builtin_fma((double)dx, (double)dx, acc[g]);
            acc[g] = __builtin_fma((double)dy, (double)dy, acc[g]);
            acc[g] = __builtin_fma((double)dz, (double)dz, acc[g]);
            acc[g] = __builtin_fma((double)dw, (double)dw, acc[g]);
        }
    }
    const double tot = pagk::fold_sum<4>(acc);
#pragma unroll
    for (int g = 0; g < 4; ++g) out[g] = (float)pagk::fold_total<4>(tot, g);
}

__device__ __forceinline__ void stage(const pag_vecs& V, u32 d, u32 id, float* s, int lane) {
    for (u32 c = lane; c < d / 4; c += 64) ((float4*)s)[c] = pag_vload4(V, id, c);
}

// ---- initial nodes: each of the n_init listed nodes is linked to its nearest min(deg, n_init-1) peers ----
__global__ void __launch_bounds__(64) k_init_clique(pag_vecs vec, uint8_t* __restrict__ recs,
                                                    pag_layout L, const u32* __restrict__ nodes, u32 n_init) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sv = (float*)smem;                       // [d]
    u64* keys = (u64*)(sv + L.d);                   // [n_init]
    u64* sorted = keys + n_init;                    // [n_init]
    const u32 vi = blockIdx.x;
    const u32 v = nodes[vi];
    const int lane = threadIdx.x;
    stage(vec, L.d, v, sv, lane);
    __syncthreads();
    for (u32 o = 0; o < n_init; ++o) {
        const u32 w = nodes[o];
        const float dist = dist_lds(vec, L.d, sv, w, lane);
        if (lane == 0) keys[o] = o == vi ? PAG_KEY_INVALID : (((u64)__float_as_uint(dist) << 32) | w);
    }
    __syncthreads();
    for (u32 i = lane; i < n_init; i += 64) {
        const u64 k = keys[i];
        u32 r = 0;
        for (u32 j = 0; j < n_init; ++j) r += (keys[j] < k) ? 1u : 0u;     // keys are distinct: they carry the node id
        sorted[r] = k;
    }
    __syncthreads();
    u32* ids = (u32*)(recs + (u64)v * L.rec_bytes);
    const u32 take = n_init - 1 < L.deg ? n_init - 1 : L.deg;
    if ((u32)lane < L.deg) ids[lane] = (u32)lane < take ? (u32)(sorted[lane] & 0xFFFFFFFFull) : PAG_EMPTY;
}

// rows of the listed nodes, widened to fp32, gathered into one contiguous block (the batch's queries)
__global__ void __launch_bounds__(64) k_gather_rows(pag_vecs vec, u32 d, const u32* __restrict__ nodes, float* __restrict__ out) {
    const u32 v = nodes[blockIdx.x];
    float4* o = (float4*)(out + (u64)blockIdx.x * d);
    for (u32 c = threadIdx.x; c < d / 4; c += 64) o[c] = pag_vload4(vec, v, c);
}

// segment bounds of the per-node candidate lists for the segmented sort
__global__ void k_cand_segments(const u32* __restrict__ cand_cnt, u32 m, u32 cand_cap, int* __restrict__ seg_begin,
                                int* __restrict__ seg_end) {
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m) return;
    const u32 c = cand_cnt[i] < cand_cap ? cand_cnt[i] : cand_cap;
    seg_begin[i] = (int)(i * cand_cap);
    seg_end[i] = (int)(i * cand_cap + c);
}

// ---- RobustPrune over R_L of each new node (Eq. 1, alpha = 1) ----
// cand_sorted: per node the keys collected by the search (dist bits << 32 | id << 1 | visited), sorted ascending by a
// segmented radix sort over bits 1..63.  Cut to efC, then scanned in order: a candidate is kept unless an already kept
// s has ||s - c||^2 <= ||v - c||^2.  Writes N_out(v) into v's record and one reverse pair per kept neighbour:
// key = target << 32 | dist bits, value = v.
// The kernel is bound by the rows it fetches: while thousands of nodes are pruned at once, a node's kept rows stay in
// no cache.  Most occlusion tests are decided by the first few neighbours kept (the closest ones), so the first J kept
// rows stay in LDS, where every later candidate meets them without memory traffic, and the candidates stream through
// registers, C at a time, NB groups in flight.  Kept rows beyond J are fetched G at a time, for the candidates that
// the first J did not occlude.  J is small on purpose: the waves that the LDS leaves room for matter more than the
// rows it holds.  NQ: 16-byte chunks of a row per lane.
template <int NQ, int C, int G>
struct PruneRows {
    const pag_vecs& V;
    const u32 d4;            // 16-byte chunks per row
    const int lane;
    float4* K;               // [J][NQ * 64] kept rows (zero-padded chunks)

    __device__ __forceinline__ void load_row(u32 id, float4 (&r)[NQ]) const {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const u32 c = (u32)lane + 64u * q;
            r[q] = c < d4 ? pag_vload4(V, id, c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    __device__ __forceinline__ static void accumulate(const float4& a, const float4& b, double& acc) {
        const float dx = a.x - b.x, dy = a.y - b.y, dz = a.z - b.z, dw = a.w - b.w;
        acc = __builtin_fma((double)dx, (double)dx, acc);
        acc = __builtin_fma((double)dy, (double)dy, acc);
        acc = __builtin_fma((double)dz, (double)dz, acc);
        acc = __builtin_fma((double)dw, (double)dw, acc);
    }
    // squared distances of the C candidate rows to kept row j (LDS); every lane gets all C
    __device__ __forceinline__ void to_lds_row(const float4 (&rows)[C][NQ], u32 j, float (&out)[C]) const {
        double acc[C];
#pragma unroll
        for (int i = 0; i < C; ++i) acc[i] = 0.0;
        const float4* kr = K + (size_t)j * (NQ * 64);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const float4 k = kr[lane + 64 * q];
#pragma unroll
            for (int i = 0; i < C; ++i) accumulate(rows[i][q], k, acc[i]);
        }
        const double t = pagk::fold_sum<C>(acc);
#pragma unroll
        for (int i = 0; i < C; ++i) out[i] = (float)pagk::fold_total<C>(t, i);
    }
    // squared distances of the C candidate rows to G rows fetched from memory
    __device__ __forceinline__ void to_memory_rows(const float4 (&rows)[C][NQ], const u32 (&sid)[G], float (&out)[C][G]) const {
        float4 kb[G][NQ];
#pragma unroll
        for (int g = 0; g < G; ++g) load_row(sid[g], kb[g]);
#pragma unroll
        for (int i = 0; i < C; ++i) {
            double acc[G];
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = 0.0;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int g = 0; g < G; ++g) accumulate(rows[i][q], kb[g][q], acc[g]);
            const double t = pagk::fold_sum<G>(acc);
#pragma unroll
            for (int g = 0; g < G; ++g) out[i][g] = (float)pagk::fold_total<G>(t, g);
        }
    }
    // squared distance between two candidate rows
    __device__ __forceinline__ float between(const float4 (&a)[NQ], const float4 (&b)[NQ]) const {
        double acc = 0.0;
#pragma unroll
        for (int q = 0; q < NQ; ++q) accumulate(a[q], b[q], acc);
        return (float)wave_sum(acc);
    }
};

template <int NQ, int C, int G, int NB>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 4)))
k_prune(pag_vecs vec, uint8_t* __restrict__ recs, pag_layout L, const u32* __restrict__ nodes, u32 m,
            const u64* __restrict__ cand_sorted, const u32* __restrict__ cand_cnt, u32 cand_cap, u32 efC, u32 J,
            const u64* __restrict__ pes, float* __restrict__ e2, u64* __restrict__ rev_keys, u32* __restrict__ rev_vals,
            const u32* __restrict__ taken) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (blockIdx.x >= m) return;
    // nodes pruned side by side are neighbours when the insertion search took them in its own order: their
    // candidate lists overlap, and so do the rows they fetch
    const u32 vi = taken ? taken[blockIdx.x] : blockIdx.x;
    const int lane = threadIdx.x;
    u32* kept = (u32*)(smem + (size_t)J * NQ * 1024);       // [deg]
    const PruneRows<NQ, C, G> P{vec, L.d / 4, lane, (float4*)smem};
    const u64* sorted = cand_sorted + (u64)vi * cand_cap;   // ascending by (dist, id); bit 0 is the visited flag
    const u32 v = nodes[vi];
    u32 nc = cand_cnt[vi];
    if (nc > cand_cap) nc = cand_cap;
    if (nc > efC) nc = efC;
    u32 nk = 0;
    u32 my_id = PAG_EMPTY;       // lane s holds kept[s]
    u32 my_key = 0;

    // The sorted keys are read 64 at a time, one per lane, a block ahead of the rows that they name: a row request
    // never waits for its key.
    u32 kbase = 0;
    u64 kcur = (u32)lane < nc ? sorted[lane] : 0ull;
    u64 knxt = 64u + lane < nc ? sorted[64u + lane] : 0ull;
    u64 key[NB][C];
    float4 row[NB][C][NQ];
    auto fetch = [&](u32 ci, u64 (&gk)[C], float4 (&rows)[C][NQ]) {
        if (ci >= kbase + 64) {
            kcur = knxt;
            kbase += 64;
            knxt = kbase + 64u + lane < nc ? sorted[kbase + 64u + lane] : 0ull;
        }
#pragma unroll
        for (int i = 0; i < C; ++i) {
            const u32 at = (ci + i < nc ? ci + i : nc - 1) - kbase;      // C divides 64: a group lies in one block
            const u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)kcur, (int)at);
            const u32 hi = (u32)__builtin_amdgcn_readlane((int)(u32)(kcur >> 32), (int)at);
            gk[i] = ((u64)hi << 32) | lo;
            P.load_row(lo >> 1, rows[i]);
        }
    };
    // decides the C candidates at positions ci .. of the list, in order
    auto decide = [&](u32 ci, const u64 (&key)[C], const float4 (&rows)[C][NQ]) {
        u32 cid[C];
        float dv[C];
        bool occ[C];
#pragma unroll
        for (int i = 0; i < C; ++i) {
            cid[i] = (u32)(key[i] & 0xFFFFFFFFull) >> 1;
            dv[i] = __uint_as_float((u32)(key[i] >> 32));
            // a node that is searched for a second time finds itself: never its own neighbour
            occ[i] = !(ci + i < nc) || cid[i] == v;
        }
        const u32 in_lds = nk < J ? nk : J;
        for (u32 j = 0; j < in_lds; ++j) {
            bool all = true;
#pragma unroll
            for (int i = 0; i < C; ++i) all = all && occ[i];
            if (all) break;
            float dd[C];
            P.to_lds_row(rows, j, dd);
#pragma unroll
            for (int i = 0; i < C; ++i) occ[i] = occ[i] || dd[i] <= dv[i];
        }
        for (u32 s0 = J; s0 < nk; s0 += G) {
            bool all = true;
#pragma unroll
            for (int i = 0; i < C; ++i) all = all && occ[i];
            if (all) break;
            u32 sid[G];
            float dd[C][G];
#pragma unroll
            for (int g = 0; g < G; ++g) sid[g] = kept[s0 + g < nk ? s0 + g : nk - 1];   // a repeated last entry changes nothing
            P.to_memory_rows(rows, sid, dd);
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int g = 0; g < G; ++g) occ[i] = occ[i] || dd[i][g] <= dv[i];
        }
        bool kept_here[C];
        bool wrote = false;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            kept_here[i] = false;
            if (nk < L.deg) {
#pragma unroll
                for (int j = 0; j < i; ++j)
                    if (kept_here[j] && !occ[i]) occ[i] = P.between(rows[j], rows[i]) <= dv[i];
                if (!occ[i]) {
                    if ((u32)lane == nk) { my_id = cid[i]; my_key = (u32)(key[i] >> 32); kept[nk] = cid[i]; }
                    if (nk < J) {
                        float4* kr = P.K + (size_t)nk * (NQ * 64);
#pragma unroll
                        for (int q = 0; q < NQ; ++q) kr[lane + 64 * q] = rows[i][q];
                    }
                    nk++;
                    kept_here[i] = true;
                    wrote = true;
                }
            }
        }
        if (wrote) __syncthreads();      // one wave per workgroup: orders the LDS writes before the next reads
    };

    // NB groups of C rows are in flight: a buffer is refilled as soon as its group is decided
#pragma unroll
    for (int b = 0; b < NB; ++b)
        if ((u32)(b * C) < nc) fetch(b * C, key[b], row[b]);
    for (u32 ci = 0; ci < nc && nk < L.deg; ci += NB * C) {
        bool done = false;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const u32 c0 = ci + b * C;
            if (!done) {
                if (c0 >= nc || nk >= L.deg) done = true;
                else {
                    decide(c0, key[b], row[b]);
                    if (c0 + NB * C < nc) fetch(c0 + NB * C, key[b], row[b]);
                }
            }
        }
        if (done) break;
    }
    __syncthreads();
    u32* ids = (u32*)(recs + (u64)v * L.rec_bytes);
    if ((u32)lane < L.deg) {
        ids[lane] = my_id;
        // ||w - v||^2 as the search computed it: what the reverse-edge step reads should v be a target in the same batch
        e2[(u64)v * L.deg + lane] = my_id == PAG_EMPTY ? 0.f : __uint_as_float(my_key);
        const u64 o = (u64)vi * L.deg + lane;
        rev_keys[o] = my_id == PAG_EMPTY ? PAG_KEY_INVALID : (((u64)my_id << 32) | my_key);
        rev_vals[o] = v;
        if (pes) {
            // PES candidates u -> v (Alg. 1, H(v)): pairs flagged in bit 31 of the distance word (a
            // non-negative float never sets it), so that they sort behind the ordinary reverse edges
            // of the same target and are only granted free slots.  Nodes already chosen as
            // out-neighbours of v have their ordinary pair.
            const u64 hk = pes[(u64)vi * L.deg + lane];
            u64 pk = PAG_KEY_INVALID;
            if (hk != PAG_KEY_INVALID) {
                const u32 u = (u32)(hk & 0xFFFFFFFFull) >> 1;
                bool dup = u == v;
                for (u32 s = 0; s < nk; ++s) dup = dup || kept[s] == u;
                if (!dup) pk = ((u64)u << 32) | 0x80000000ull | (hk >> 32);
            }
            const u64 o2 = (u64)m * L.deg + o;
            rev_keys[o2] = pk;
            rev_vals[o2] = v;
        }
    }
}

template <int NQ>
static int launch_prune(hipStream_t s, const pag_index* ix, const u32* nodes, u32 m, const u64* cand_sorted,
                        const u32* cand_cnt, u32 cand_cap, const u64* pes, u64* rev_keys, u32* rev_vals, const u32* taken) {
    const pag_layout& L = ix->L;
    // kept rows held in LDS (slots of NQ KB): four, more while they fit 16 KB, fewer beyond 36 KB.  Measured on
    // 1M x 768 / 1024 / 1536 and 250k x 3072: 16 / 16 / 24 / 36 KB are the fastest; larger sets lose more waves than
    // they save reads.
    u32 J = std::max<u32>(4u, 16u / NQ);
    J = std::min<u32>(J, 36u / NQ);
    J = std::min<u32>(J, L.deg);
    const u32 lds = J * NQ * 1024u + L.deg * 4;
    hipLaunchKernelGGL((k_prune<NQ, 2, 2, 2>), dim3(m), dim3(64), lds, s, pag_vecs_of(ix), ix->rec, L, nodes, m, cand_sorted,
                       cand_cnt, cand_cap, ix->efC, J, pes, ix->e2, rev_keys, rev_vals, taken);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

// ---- reverse edges, one wave per target (Sec. 2.1, N_in(v); Eq. 1) ----
// Sorted pairs (target << 32 | dist bits, source).  The wave whose pair starts a target's segment
// walks the segment.  For an incoming v at squared distance duv:
//   refuse if some w in N_out(u) has ||w-u||^2 <= duv and ||w-v||^2 <= duv;
//   else take a free slot; if the list is full, drop the neighbours farther than v that v now
//   occludes (||v-f||^2 <= ||f-u||^2), or failing that the farthest of N_out(u) + {v}.
// Pairs that come from the PES buffers H(v) (flag in bit 31 of the distance word) pass the same
// Eq. 1 check but are only ever given a free slot.
// Every slot that received a new neighbour is appended to `edges` for the inference-information pass.
__global__ void __launch_bounds__(64) k_reverse(pag_vecs vec, uint8_t* __restrict__ recs,
                                                float* __restrict__ e2, pag_layout L,
                                                const u64* __restrict__ keys, const u32* __restrict__ vals,
                                                u32 n_pairs, u32* __restrict__ edges, u32* __restrict__ n_edges) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sv = (float*)smem;
    const u32 i0 = blockIdx.x;
    if (i0 >= n_pairs) return;
    const u64 k0 = keys[i0];
    if (k0 == PAG_KEY_INVALID) return;
    const u32 u = (u32)(k0 >> 32);
    if (i0 > 0 && (u32)(keys[i0 - 1] >> 32) == u) return;       // not the head of its segment
    const int lane = threadIdx.x;
    uint8_t* rec = recs + (u64)u * L.rec_bytes;
    u32 id = PAG_EMPTY;
    float we2 = 0.f;
    if ((u32)lane < L.deg) { id = ((const u32*)rec)[lane]; we2 = e2[(u64)u * L.deg + lane]; }
    u64 changed = 0;
    for (u32 i = i0; i < n_pairs; ++i) {
        const u64 k = keys[i];
        if (k == PAG_KEY_INVALID || (u32)(k >> 32) != u) break;
        const u32 v = vals[i];
        const bool from_pes = (k >> 31) & 1ull;
        const float duv = __uint_as_float((u32)(k & 0x7FFFFFFFull));
        const bool valid = (u32)lane < L.deg && id != PAG_EMPTY;
        if (v == u || __ballot(valid && id == v)) continue;
        // PES candidates are only added to available out-degree slots (Alg. 1, last loop)
        if (from_pes && __ballot((u32)lane < L.deg && id == PAG_EMPTY) == 0ull) continue;
        stage(vec, L.d, v, sv, lane);
        __syncthreads();
        // lane s gets ||w_s - v||^2
        float dwv = 0.f;
        for (u64 mm = __ballot(valid); mm;) {
            const int p = __ffsll((long long)mm) - 1;
            mm &= mm - 1;
            const u32 w = (u32)__builtin_amdgcn_readlane((int)id, p);
            const float dd = dist_lds(vec, L.d, sv, w, lane);
            if (lane == p) dwv = dd;
        }
        __syncthreads();
        if (__ballot(valid && we2 <= duv && dwv <= duv)) continue;                 // Eq. 1: v is occluded
        const u64 freem = __ballot((u32)lane < L.deg && id == PAG_EMPTY);
        int slot = -1;
        if (freem) {
            slot = __ffsll((long long)freem) - 1;
        } else {
            const bool farther = we2 > duv || (we2 == duv && id > v);
            const u64 dropm = __ballot(valid && farther && dwv <= we2);
            if (dropm) {
                slot = __ffsll((long long)dropm) - 1;
                if ((dropm >> lane) & 1ull) { id = PAG_EMPTY; we2 = 0.f; }
            } else {
                // farthest neighbour by (e2, id)
                u64 fk = valid ? (((u64)__float_as_uint(we2) << 32) | id) : 0ull;
                u64 best = fk;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) {
                    const u64 other = __shfl_xor(best, o, 64);
                    best = other > best ? other : best;
                }
                const u64 vk = ((u64)__float_as_uint(duv) << 32) | v;
                if (vk < best) slot = __ffsll((long long)__ballot(valid && fk == best)) - 1;
            }
        }
        if (slot >= 0) {
            if (lane == slot) { id = v; we2 = duv; }
            changed |= 1ull << slot;
        }
    }
    if ((u32)lane < L.deg) {
        ((u32*)rec)[lane] = id;
        e2[(u64)u * L.deg + lane] = we2;
        if (id == PAG_EMPTY) {                                // a dropped neighbour leaves a clean slot
            ((float*)(rec + L.off_a))[lane] = 0.f;
            ((float*)(rec + L.off_c))[lane] = 0.f;
            u32* cw = (u32*)(rec + L.off_codes) + (u32)lane * L.cw;
            for (u32 k = 0; k < L.cw; ++k) cw[k] = 0u;
        }
    }
    const u32 nch = (u32)__popcll(changed);
    if (nch) {
        u32 base = 0;
        if (lane == 0) base = atomicAdd(n_edges, nch);
        base = (u32)__builtin_amdgcn_readfirstlane((int)base);
        if ((changed >> lane) & 1ull) {
            const u32 idx = base + (u32)__popcll(changed & ((1ull << lane) - 1));
            edges[2 * (u64)idx] = u;
            edges[2 * (u64)idx + 1] = (u32)lane;
        }
    }
}

// ---- is a batch a region of its own? ----
// The nodes of a batch do not see each other.  For n_sample nodes of the batch, spread evenly over it, this counts
// the batch-mates and the older nodes of the graph (n_probe of each, spread evenly) that lie closer than the
// farthest neighbour the node has just been given: added to out[2i] (mates) and out[2i+1] (older nodes).  In a batch drawn from
// the same distribution as the graph the two fractions agree; where the batch-mates are many times denser (new
// data inserted next to none of the old) the batch is linked a second time, now that its nodes are in the graph,
// in eight parts taken one after the other.
// order: the ids being inserted, in insertion order; the first `done` of them and all ids below n_begin are in the
// graph already, the batch is order[done .. done + m).
__global__ void __launch_bounds__(64) k_batch_density(pag_vecs vec, const uint8_t* __restrict__ recs, const float* __restrict__ e2,
                                                      pag_layout L, const u32* __restrict__ order, u64 n_begin, u64 done, u32 m,
                                                      u32 n_sample, u32 n_probe, u32* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sv = (float*)smem;
    const int lane = threadIdx.x;
    const u32* nodes = order + done;
    const u64 graph = n_begin + done;
    const u32 x = nodes[(u64)blockIdx.x * m / n_sample];
    stage(vec, L.d, x, sv, lane);
    __syncthreads();
    float far = 0.f;
    if ((u32)lane < L.deg && ((const u32*)(recs + (u64)x * L.rec_bytes))[lane] != PAG_EMPTY) far = e2[(u64)x * L.deg + lane];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) far = fmaxf(far, __shfl_xor(far, o, 64));
    u32 c_mate = 0, c_old = 0;
    // the probes of one node are shared out over gridDim.y waves
    const u32 per = (n_probe + gridDim.y - 1) / gridDim.y;
    const u32 j0 = blockIdx.y * per, j1 = j0 + per < n_probe ? j0 + per : n_probe;
    for (u32 j = j0; j < j1; j += 2) {
        u32 y[4];
        float dd[4];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const u32 jj = j + g < j1 ? j + g : j1 - 1;
            y[g] = nodes[(u64)jj * m / n_probe];
            const u64 t = (u64)jj * graph / n_probe;
            y[2 + g] = t < n_begin ? (u32)t : order[t - n_begin];
        }
        dist_lds4(vec, L.d, sv, y, dd);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const bool in = j + g < j1;
            c_mate += (in && y[g] != x && dd[g] < far) ? 1u : 0u;
            c_old += (in && dd[2 + g] < far) ? 1u : 0u;
        }
    }
    if (lane == 0) { atomicAdd(&out[2 * blockIdx.x], c_mate); atomicAdd(&out[2 * blockIdx.x + 1], c_old); }
}

struct BuildWs {
    u64* cand = nullptr; u64* cand_sorted = nullptr; u32* cand_cnt = nullptr; u64* pes = nullptr;
    u64 *rk_in = nullptr, *rk_out = nullptr; u32 *rv_in = nullptr, *rv_out = nullptr;
    u32* edges = nullptr; u32* n_edges = nullptr;
    u32* order = nullptr;
    const u32* taken = nullptr;    // the order in which the last insertion search took its points (null: as listed)
    u32* density = nullptr;
    void* sort_tmp = nullptr; size_t sort_bytes = 0;
    int *seg_begin = nullptr, *seg_end = nullptr;
    void* seg_tmp = nullptr; size_t seg_bytes = 0;
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};   // phase marks of one linking pass
    ~BuildWs() {
        for (auto& e : ev) if (e) (void)hipEventDestroy(e);
        void* p[] = { cand, cand_sorted, cand_cnt, pes, rk_in, rk_out, rv_in, rv_out, edges, n_edges, order, density, sort_tmp, seg_begin, seg_end, seg_tmp };
        for (void* x : p) if (x) (void)hipFree(x);
    }
};

#define PAG_ALLOC(ptr, bytes)                                                                   \
    do {                                                                                        \
        hipError_t e__ = hipMalloc((void**)&(ptr), (bytes) ? (bytes) : 16);                      \
        if (e__ != hipSuccess) { pag_set_error(std::string("hipMalloc (build): ") + hipGetErrorString(e__)); return PAG_ENOMEM; } \
    } while (0)

}  // namespace

// Workspaces of the insertion search for batches of up to max_batch nodes.
static int alloc_candidate_ws(BuildWs& ws, u64 max_batch, u32 cand_cap, u32 deg, bool use_pes, hipStream_t s) {
    if (max_batch * cand_cap > 0x7FFFFFFFull) { pag_set_error("build: batch x ef_construction exceeds 2^31 candidate slots"); return PAG_EUNSUPPORTED; }
    PAG_ALLOC(ws.cand, max_batch * cand_cap * 8);
    PAG_ALLOC(ws.cand_sorted, max_batch * cand_cap * 8);
    PAG_ALLOC(ws.cand_cnt, max_batch * 4);
    if (use_pes) PAG_ALLOC(ws.pes, max_batch * deg * 8);
    PAG_ALLOC(ws.seg_begin, max_batch * 4);
    PAG_ALLOC(ws.seg_end, max_batch * 4);
    PAG_HIP(hipcub::DeviceSegmentedRadixSort::SortKeys(nullptr, ws.seg_bytes, ws.cand, ws.cand_sorted, (int)(max_batch * cand_cap),
                                                       (int)max_batch, ws.seg_begin, ws.seg_end, 1, 64, s));
    PAG_ALLOC(ws.seg_tmp, ws.seg_bytes);
    return PAG_OK;
}

// The search of Alg. 1 for m points (rotated rows `qrot`) over the nodes below n_limit: tables, the PRT-TFB search in
// indexing mode (ef = efC, b = min(efC, 100), every round's W collected, PES screening into ws.pes), then every
// point's candidates sorted by (dist, id) -- bits 1..63 of the keys, the visited flag aside -- into ws.cand_sorted.
static int search_candidates(pag_index* ix, BuildWs& ws, const float* qrot, u64 m, u32 b, u32 cand_cap, u64 n_limit) {
    const pag_layout& L = ix->L;
    hipStream_t s = ix->stream;
    int rc;
    if ((rc = pag_launch_tables(s, qrot, m, L, ix->cb, ix->ws_tab))) return rc;
    SearchArgs a;
    u32 lds = 0;
    int grid = 0;
    if ((rc = pag_search_common(ix, b, ix->efC, n_limit, &a, &lds, &grid))) return rc;
    a.qrot = qrot; a.tables = ix->ws_tab; a.nq = (u32)m; a.K = b;
    a.flags &= ~(u32)PAG_FLAG_NO_PRT;          // indexing always runs with the projection test on
    a.cand = ws.cand; a.cand_cnt = ws.cand_cnt; a.cand_cap = cand_cap;
    a.pes = ws.pes;
    // more points than resident waves: those that search side by side are chosen to be neighbours
    if (!(ix->flags & PAG_FLAG_KEEP_QUERY_ORDER) && m > (u64)grid && (rc = pag_order_queries(ix, qrot, m, &a.order))) return rc;
    ws.taken = a.order;
    if ((rc = pag_launch_zero_u32(s, ix->d_qcounter, 1))) return rc;
    if (ws.ev[0]) PAG_HIP(hipEventRecord(ws.ev[0], s));
    if ((rc = pag_launch_search(ix, a, lds, &grid))) return rc;
    if (ws.ev[1]) PAG_HIP(hipEventRecord(ws.ev[1], s));
    hipLaunchKernelGGL(k_cand_segments, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, s, ws.cand_cnt, (u32)m, cand_cap,
                       ws.seg_begin, ws.seg_end);
    PAG_HIP(hipGetLastError());
    PAG_HIP(hipcub::DeviceSegmentedRadixSort::SortKeys(ws.seg_tmp, ws.seg_bytes, ws.cand, ws.cand_sorted, (int)(m * cand_cap), (int)m,
                                                       ws.seg_begin, ws.seg_end, 1, 64, s));
    return PAG_OK;
}

// grows a workspace of the index to `need` floats
static int ensure_floats(float** p, u64* cap, u64 need) {
    if (*cap >= need) return PAG_OK;
    if (*p) (void)hipFree(*p);
    *p = nullptr; *cap = 0;
    PAG_ALLOC(*p, need * 4);
    *cap = need;
    return PAG_OK;
}

// splitmix64: the generator behind the insertion order
static inline u64 next_random(u64& state) {
    u64 z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Inserts the nodes [n_begin, n_end), whose rows are already in the store, into the graph.  They are
// taken in a pseudo-random order fixed by the index seed, not in id order: the nodes of one batch do
// not see each other, so a batch of consecutive ids of an input that arrives sorted (by cluster, by
// source, by time) would hold exactly the points that should have become each other's neighbours;
// and the entry list, the first 1024 nodes of the order, would sit in one corner of the data.
int pag_build_range(pag_index* ix, u64 n_begin, u64 n_end) {
    if (n_end <= n_begin) return PAG_OK;
    const pag_layout& L = ix->L;
    hipStream_t s = ix->stream;
    for (double& ms : ix->build_phase_ms) ms = 0.0;
    const u32 b = std::min<u32>(ix->efC, 100);
    const u32 Rmax = std::max<u32>(1, (ix->efC + b - 1) / b);
    const u32 cand_cap = Rmax * b;
    int rc;
    const u64 count = n_end - n_begin;
    BuildWs ws;
    {
        std::vector<u32> order(count);
        for (u64 i = 0; i < count; ++i) order[i] = (u32)(n_begin + i);
        u64 state = ix->seed ^ (0xA0761D6478BD642Full * (n_begin + 1));
        if (!(ix->flags & PAG_FLAG_KEEP_ORDER))
            for (u64 i = count - 1; i > 0; --i) {             // Fisher-Yates
                const u64 j = next_random(state) % (i + 1);
                std::swap(order[i], order[j]);
            }
        PAG_ALLOC(ws.order, count * 4);
        PAG_HIP(hipMemcpyAsync(ws.order, order.data(), count * 4, hipMemcpyHostToDevice, s));
        // the entry list grows with the first nodes of the order until it holds 1024
        const u32 have = n_begin == 0 ? 0u : ix->n_entry;
        if (have < 1024) {
            const u32 add = (u32)std::min<u64>(count, 1024 - have);
            PAG_HIP(hipMemcpyAsync(ix->entry + have, order.data(), add * 4, hipMemcpyHostToDevice, s));
        }
        if (n_begin == 0) ix->n_entry = 0;
        PAG_HIP(hipStreamSynchronize(s));                    // `order` (host) is released here
    }
    const u32 entry_before = ix->n_entry;
    u64 done = 0;                                            // nodes of the range inserted so far
    if (n_begin == 0) {
        const u32 n_init = (u32)std::min<u64>(n_end, b);
        if (n_init > 1) {
            const u32 lds = L.d * 4 + 2 * n_init * 8;
            hipLaunchKernelGGL(k_init_clique, dim3(n_init), dim3(64), lds, s, pag_vecs_of(ix), ix->rec, L, ws.order, n_init);
            PAG_HIP(hipGetLastError());
        }
        // also for a lone first node: its record leaves this pass with clean free slots
        if ((rc = pag_launch_edge_info_of(s, ix, ws.order, n_init))) return rc;
        done = n_init;
    }
    ix->n_entry = (u32)std::min<u64>(entry_before + done, 1024);
    if (done >= count) { PAG_HIP(hipStreamSynchronize(s)); return PAG_OK; }

    u64 max_batch = ix->subbatch ? ix->subbatch : std::min<u64>(16384, std::max<u64>(1024, n_end / 50));
    max_batch = std::min<u64>(max_batch, count);       // a small insertion gets small workspaces
    const bool use_pes = !(ix->flags & PAG_FLAG_NO_PES);
    if ((rc = alloc_candidate_ws(ws, max_batch, cand_cap, L.deg, use_pes, s))) return rc;
    for (auto& e : ws.ev) PAG_HIP(hipEventCreate(&e));
    const u64 max_pairs = max_batch * L.deg * (use_pes ? 2 : 1);
    PAG_ALLOC(ws.rk_in, max_pairs * 8);
    PAG_ALLOC(ws.rk_out, max_pairs * 8);
    PAG_ALLOC(ws.rv_in, max_pairs * 4);
    PAG_ALLOC(ws.rv_out, max_pairs * 4);
    PAG_ALLOC(ws.edges, max_pairs * 8);
    PAG_ALLOC(ws.n_edges, 16);
    PAG_HIP(hipcub::DeviceRadixSort::SortPairs(nullptr, ws.sort_bytes, ws.rk_in, ws.rk_out, ws.rv_in, ws.rv_out,
                                               (int)max_pairs, 0, 64, s));
    PAG_ALLOC(ws.sort_tmp, ws.sort_bytes);
    // the rows of a batch, gathered (its queries), and their tables
    if ((rc = ensure_floats(&ix->ws_qrot, &ix->ws_qrot_cap, max_batch * L.d))) return rc;
    if ((rc = ensure_floats(&ix->ws_tab, &ix->ws_tab_cap, max_batch * L.Ppad * PAG_NCODE))) return rc;
    constexpr u32 kDensitySamples = 128, kDensityProbes = 2048;
    constexpr double kCrowdedRatio = 4.0;
    PAG_ALLOC(ws.density, kDensitySamples * 2 * 4);
    // one linking pass over `m` listed nodes: search, RobustPrune, reverse edges, inference information
    auto link = [&](const u32* nodes, u64 m) -> int {
        int rc;
        // 1. the new nodes are their own queries (already rotated): rows gathered and widened to fp32
        hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)m), dim3(64), 0, s, pag_vecs_of(ix), L.d, nodes, ix->ws_qrot);
        PAG_HIP(hipGetLastError());
        // 2. + 3. PRT-TFB search of the graph built so far, candidates sorted.  Nodes that are not inserted yet have
        //    empty records and no in-edges, and the entry list holds inserted nodes only, so they cannot be reached.
        if ((rc = search_candidates(ix, ws, ix->ws_qrot, m, b, cand_cap, n_end))) return rc;
        //    RobustPrune -> N_out(v), reverse pairs
        {
#define PRUNE_ARGS s, ix, nodes, (u32)m, ws.cand_sorted, ws.cand_cnt, cand_cap, ws.pes, ws.rk_in, ws.rv_in, ws.taken
            const u32 nq = (L.d / 4 + 63) / 64;          // 16-byte chunks of a row per lane
            if (nq <= 1) rc = launch_prune<1>(PRUNE_ARGS);
            else if (nq == 2) rc = launch_prune<2>(PRUNE_ARGS);
            else if (nq == 3) rc = launch_prune<3>(PRUNE_ARGS);
            else if (nq == 4) rc = launch_prune<4>(PRUNE_ARGS);
            else if (nq <= 6) rc = launch_prune<6>(PRUNE_ARGS);
            else if (nq <= 8) rc = launch_prune<8>(PRUNE_ARGS);
            else rc = launch_prune<12>(PRUNE_ARGS);
#undef PRUNE_ARGS
            if (rc) return rc;
        }
        PAG_HIP(hipEventRecord(ws.ev[2], s));
        // 4. group reverse pairs by target
        const u32 n_pairs = (u32)(m * L.deg * (use_pes ? 2 : 1));
        PAG_HIP(hipcub::DeviceRadixSort::SortPairs(ws.sort_tmp, ws.sort_bytes, ws.rk_in, ws.rk_out, ws.rv_in, ws.rv_out,
                                                   (int)n_pairs, 0, 64, s));
        // 5. apply them
        if ((rc = pag_launch_zero_u32(s, ws.n_edges, 1))) return rc;
        hipLaunchKernelGGL(k_reverse, dim3(n_pairs), dim3(64), L.d * 4, s, pag_vecs_of(ix), ix->rec, ix->e2, L, ws.rk_out,
                           ws.rv_out, n_pairs, ws.edges, ws.n_edges);
        PAG_HIP(hipGetLastError());
        PAG_HIP(hipEventRecord(ws.ev[3], s));
        // 6. inference information of the new forward edges and of every changed reverse slot
        if ((rc = pag_launch_edge_info_of(s, ix, nodes, m))) return rc;
        PAG_HIP(hipEventRecord(ws.ev[4], s));
        u32 n_edges = 0;
        PAG_HIP(hipMemcpyAsync(&n_edges, ws.n_edges, 4, hipMemcpyDeviceToHost, s));
        PAG_HIP(hipStreamSynchronize(s));
        for (int i = 0; i < 4; ++i) {            // search kernel | sort + RobustPrune | pair sort + reverse edges | inference information
            float ms = 0.f;
            PAG_HIP(hipEventElapsedTime(&ms, ws.ev[i], ws.ev[i + 1]));
            ix->build_phase_ms[i] += ms;
        }
        return pag_launch_edge_info_list(s, ix, ws.edges, n_edges);
    };
    while (done < count) {
        const u64 graph = n_begin + done;                  // nodes in the graph so far
        u64 m = std::min<u64>(count - done, max_batch);
        m = std::min<u64>(m, std::max<u64>(1, graph / 2));
        const u32* nodes = ws.order + done;
        if ((rc = link(nodes, m))) return rc;
        done += m;
        ix->n_entry = (u32)std::min<u64>(entry_before + done, 1024);
        // The nodes of the batch did not see each other.  Where they crowd a region of their own (sampled: around them
        // batch-mates are several times denser, relative to the batch, than older nodes are relative to the graph), they
        // are linked once more now that they are part of the graph.
        if (m >= 64 && graph >= 64) {
            const u32 ns = kDensitySamples, np = (u32)std::min<u64>(std::min<u64>(m, graph), kDensityProbes);
            if ((rc = pag_launch_zero_u32(s, ws.density, 2 * ns))) return rc;
            hipLaunchKernelGGL(k_batch_density, dim3(ns, 8), dim3(64), L.d * 4, s, pag_vecs_of(ix), ix->rec, ix->e2, L, ws.order, n_begin,
                               done - m, (u32)m, ns, np, ws.density);
            PAG_HIP(hipGetLastError());
            u32 h[kDensitySamples * 2];
            PAG_HIP(hipMemcpyAsync(h, ws.density, sizeof h, hipMemcpyDeviceToHost, s));
            PAG_HIP(hipStreamSynchronize(s));
            double mates = 0.0, older = 0.0;
            for (u32 i = 0; i < ns; ++i) { mates += h[2 * i]; older += h[2 * i + 1]; }
            // both counts are out of ns * np probes: their ratio compares the two densities directly
            const bool crowded = mates >= 32.0 && mates > kCrowdedRatio * std::max(older, 1.0);
            if (crowded) {
                // in eight parts, one after the other: what one part links is there for the next
                constexpr u64 kParts = 8;
                for (u64 k = 0; k < kParts; ++k) {
                    const u64 j0 = m * k / kParts, j1 = m * (k + 1) / kParts;
                    if (j1 > j0 && (rc = link(nodes + j0, j1 - j0))) return rc;
                }
                ix->relinked_batches++;
            }
        }
    }
    PAG_HIP(hipStreamSynchronize(s));
    return PAG_OK;
}

// What inserting each of the m raw vectors X into the index as it stands would start from (Alg. 1, the search of one
// insertion; Eq. 5): R_L cut to efC and the PES buffer H(v), copied to host arrays.  The index is not changed.
extern "C" int pag_insertion_candidates(const pag_index* cix, const float* X, uint64_t m, uint32_t* cand_ids,
                                        float* cand_keys, uint32_t* cand_count, uint32_t* pes_ids, float* pes_keys,
                                        uint32_t* pes_count) {
    pag_index* ix = const_cast<pag_index*>(cix);   // workspaces are mutable state of the handle
    if (!ix || !X || !cand_ids || !cand_keys || !cand_count || !pes_ids || !pes_keys || !pes_count) {
        pag_set_error("pag_insertion_candidates: null argument");
        return PAG_EINVAL;
    }
    if (m == 0) return PAG_OK;
    int prev = -1;
    (void)hipGetDevice(&prev);
    if (prev != ix->device) (void)hipSetDevice(ix->device);
    struct Restore { int prev, cur; ~Restore() { if (prev >= 0 && prev != cur) (void)hipSetDevice(prev); } } restore{prev, ix->device};
    try {
        const pag_layout& L = ix->L;
        hipStream_t s = ix->stream;
        const u32 efC = ix->efC;
        const u32 b = std::min<u32>(efC, 100);
        const u32 Rmax = std::max<u32>(1, (efC + b - 1) / b);
        const u32 cand_cap = Rmax * b;
        const bool use_pes = !(ix->flags & PAG_FLAG_NO_PES);
        const u64 chunk = std::min<u64>(m, 4096);
        int rc;
        BuildWs ws;
        if ((rc = alloc_candidate_ws(ws, chunk, cand_cap, L.deg, use_pes, s))) return rc;
        if ((rc = ensure_floats(&ix->ws_qrot, &ix->ws_qrot_cap, chunk * L.d))) return rc;
        if ((rc = ensure_floats(&ix->ws_tab, &ix->ws_tab_cap, chunk * L.Ppad * PAG_NCODE))) return rc;
        if (ix->metric == PAG_COS && (rc = ensure_floats(&ix->ws_norm, &ix->ws_norm_cap, chunk * L.d))) return rc;
        __half* half_rows = nullptr;
        struct FreeHalf { __half*& p; ~FreeHalf() { if (p) (void)hipFree(p); } } free_half{half_rows};
        if (ix->vec_half) PAG_ALLOC(half_rows, chunk * L.d * 2);
        std::vector<u64> keys(chunk * cand_cap), hk(use_pes ? chunk * L.deg : 0);
        std::vector<u32> cnt(chunk);
        for (u64 c0 = 0; c0 < m; c0 += chunk) {
            const u64 cm = std::min<u64>(chunk, m - c0);
            // the row the vector would be stored as: normalised (COS), rotated, rounded if the store is 16-bit
            const float* src = X + c0 * L.d;
            if (ix->metric == PAG_COS) {
                if ((rc = pag_launch_normalise(s, src, cm, L.d, ix->ws_norm))) return rc;
                src = ix->ws_norm;
            }
            if ((rc = pag_launch_rotate(s, src, cm, L.d, ix->rot, ix->ws_qrot))) return rc;
            if (ix->vec_half) {
                if ((rc = pag_launch_convert(s, ix->ws_qrot, 0, half_rows, 1, cm * L.d))) return rc;
                if ((rc = pag_launch_convert(s, half_rows, 1, ix->ws_qrot, 0, cm * L.d))) return rc;
            }
            if ((rc = search_candidates(ix, ws, ix->ws_qrot, cm, b, cand_cap, ix->n))) return rc;
            PAG_HIP(hipMemcpyAsync(keys.data(), ws.cand_sorted, cm * cand_cap * 8, hipMemcpyDeviceToHost, s));
            PAG_HIP(hipMemcpyAsync(cnt.data(), ws.cand_cnt, cm * 4, hipMemcpyDeviceToHost, s));
            if (use_pes) PAG_HIP(hipMemcpyAsync(hk.data(), ws.pes, cm * L.deg * 8, hipMemcpyDeviceToHost, s));
            PAG_HIP(hipStreamSynchronize(s));
            for (u64 i = 0; i < cm; ++i) {
                const u32 nc = std::min<u32>(std::min<u32>(cnt[i], cand_cap), efC);
                cand_count[c0 + i] = nc;
                for (u32 k = 0; k < efC; ++k) {
                    const u64 key = k < nc ? keys[i * cand_cap + k] : 0ull;
                    cand_ids[(c0 + i) * efC + k] = k < nc ? (u32)(key & 0xFFFFFFFFull) >> 1 : PAG_EMPTY;
                    const u32 bits = (u32)(key >> 32);
                    std::memcpy(&cand_keys[(c0 + i) * efC + k], &bits, 4);
                }
                u32 nh = 0;
                for (u32 k = 0; k < L.deg; ++k) {
                    const u64 key = use_pes ? hk[i * L.deg + k] : PAG_KEY_INVALID;
                    const bool ok = key != PAG_KEY_INVALID;
                    pes_ids[(c0 + i) * L.deg + k] = ok ? (u32)(key & 0xFFFFFFFFull) >> 1 : PAG_EMPTY;
                    const u32 bits = ok ? (u32)(key >> 32) : 0u;
                    std::memcpy(&pes_keys[(c0 + i) * L.deg + k], &bits, 4);
                    nh += ok ? 1u : 0u;
                }
                pes_count[c0 + i] = nh;
            }
        }
        return PAG_OK;
    } catch (const std::bad_alloc&) {
        pag_set_error("pag_insertion_candidates: host allocation failed");
        return PAG_ENOMEM;
    }
}
