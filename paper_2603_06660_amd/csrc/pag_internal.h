// Internal declarations shared by the translation units of the PAG library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <string>

#include "pag.h"

typedef unsigned long long u64;
typedef uint32_t u32;

#define PAG_EMPTY 0xFFFFFFFFu
#define PAG_NCODE 16        // projection vectors per subspace (Appendix D (1)): one code is 4 bits
#define PAG_KEY_INVALID 0xFFFFFFFFFFFFFFFFull
#define PAG_MAX_B 1024      // working-set size limit: sixteen entries per lane
#define PAG_RANK_SORT_MAX 256  // lists up to this length are sorted by ranks, longer ones by a bitonic network
#define PAG_LDS_RING_MAX_B 128  // larger working sets keep R_F / R_T in HBM (the kernel's NW > 2 instantiations)
#define PAG_MAX_DEG 64      // one neighbour per lane
#define PAG_MAX_CW 8        // code dwords per neighbour: up to 64 subspaces
#define PAG_SEARCH_DISTINCT (1u << 30)  // SearchArgs.flags, internal: a hop drops an id that an earlier slot of the record also lists
#define PAG_STATIC_SCRATCH_BYTES (48u << 20)   // the device array behind pag_search_static, per GPU
#define PAG_STATIC_QUERY_FLOATS (4ull << 20)    // of which at most 16 MB hold rotated queries, tables and normalised copies

void pag_set_error(const std::string& msg);

#define PAG_HIP(call)                                                                        \
    do {                                                                                     \
        hipError_t e__ = (call);                                                             \
        if (e__ != hipSuccess) {                                                             \
            pag_set_error(std::string(#call) + ": " + hipGetErrorString(e__));               \
            return PAG_EHIP;                                                                 \
        }                                                                                    \
    } while (0)

// Device-side statistics, summed with atomics by every wave when it retires.
enum {
    CTR_QUERIES = 0, CTR_HOPS, CTR_TESTS, CTR_PASSES, CTR_EXACT, CTR_ROUNDS, CTR_RF_OVER,
    CTR_RT_OVER, CTR_SPILLS, CTR_PHASE0, CTR_PHASE1, CTR_PHASE2, CTR_PHASE3, CTR_PHASE4, CTR_PHASE5, CTR_COUNT
};

// Adjacency record of node u (one burst of whole 128-byte lines):
//   [ids deg x u32][a deg x f32][c deg x f32][pad to 16 B][codes deg x (cw dwords)]   padded to 128 bytes
// codes of neighbour slot s: dword l/8 of its chunk holds the code of subspace l in bits 4*(l%8).
struct pag_layout {
    u32 d, P, dsub, deg;
    u32 Ppad;        // P rounded up to 16, 32 or 64 (table rows beyond P are zero)
    u32 cw;          // code dwords per neighbour = Ppad / 8
    u32 rec_bytes;   // record size
    u32 off_a, off_c, off_codes;
};

// Row-major vector store: fp32 elements, or 16-bit floats (the paper's own payload, Sec. 4.2).
// A 16-bit store holds values that are exactly representable, so every kernel widens them to fp32
// and then computes exactly as it would on an fp32 store holding those values.
struct pag_vecs {
    const void* base;
    u32 d;
    u32 half;   // 0: float, 1: __half
};

__device__ __forceinline__ float4 pag_vload4(const pag_vecs& V, u64 row, u32 c4) {   // elements [4*c4, 4*c4+4)
    if (V.half) {
        const uint2 raw = *(const uint2*)((const __half*)V.base + row * V.d + 4 * (u64)c4);
        const __half2 lo = *(const __half2*)&raw.x, hi = *(const __half2*)&raw.y;
        const float2 a = __half22float2(lo), b = __half22float2(hi);
        return make_float4(a.x, a.y, b.x, b.y);
    }
    return ((const float4*)((const float*)V.base + row * V.d))[c4];
}

__device__ __forceinline__ float pag_vload1(const pag_vecs& V, u64 row, u32 k) {
    if (V.half) return __half2float(((const __half*)V.base)[row * V.d + k]);
    return ((const float*)V.base)[row * V.d + k];
}

struct pag_index {
    int device;
    hipStream_t stream;
    pag_layout L;
    int32_t metric;
    u64 n, capacity;
    u32 efC, search_b, subbatch, flags, seen_log2;
    u64 seed;
    // HBM-resident index
    void* vec;       // [capacity * d]   rotated vectors, float or __half (vec_half)
    u32 vec_half;
    uint8_t* rec;    // [capacity * rec_bytes]
    float* e2;       // [capacity * deg] ||w-u||^2 per edge (indexing only)
    float* rot;      // [d * d]          Q (row-major)
    float* cb;       // [P * 16 * dsub]
    u32* entry;      // [n_entry]
    u32 n_entry;
    u32 concurrent_view;   // a searcher's view: its searches may overlap a pag_insert that rewrites records
    // workspaces (grown on demand, kept between calls)
    float* ws_qrot;  u64 ws_qrot_cap;     // floats
    float* ws_tab;   u64 ws_tab_cap;      // floats
    float* ws_norm;  u64 ws_norm_cap;     // floats (normalised copies for COS)
    u32* ws_bitmap;  u64 ws_bitmap_cap;   // u32 words: per-wave seen-set spill bitmaps
    u64* ws_rings;   u64 ws_rings_cap;    // u64 keys: per-wave R_F / R_T / R_L of large working sets
    u32* ws_order;   u64 ws_order_cap;    // u32 words: workspace of pag_order_queries
    u32* d_qcounter;                      // persistent-wave work counter
    u64* d_counters;                      // CTR_COUNT
    hipEvent_t ev[4];
    int num_cu;
    double last_search_ms, last_prepare_ms, last_build_ms;
    double build_phase_ms[4];             // of the last pag_build / pag_insert: search kernel, sort + RobustPrune, pair sort + reverse edges, inference information
    u64 relinked_batches;                 // insertion batches that were linked a second time (crowded regions)
    u32 insert_failed;                    // a pag_insert stopped half way: the index answers searches but takes no more vectors
};

struct SearchArgs {
    const void* vec;         // float or __half rows, see the kernel's HALF parameter
    const uint8_t* rec;
    const float* qrot;       // [nq * d] rotated queries
    const float* tables;     // [nq * Ppad * 16]
    const u32* entry;
    u32 n_entry;
    u32 n_limit;             // only nodes < n_limit belong to the graph
    u32 d, deg, Ppad, cw, rec_bytes, off_a, off_c, off_codes;
    u32 nq, K, b, Rmax, hlog, blog, flags;   // hlog: log2 slots of the LDS hash; blog: log2 bits of the Bloom filter (0 = none)
    u32 off_hash, off_bloom, off_sa, off_sb, off_rf, off_rt;   // LDS offsets (bytes)
    u32 ring_mask;           // rings live in power-of-two buffers of >= b slots; only the last b pushes are valid
    u64* rings;              // [grid * 3 * (ring_mask + 1)] per-wave R_F, R_T and R_L when b > PAG_LDS_RING_MAX_B, else unused
    long long* out_ids;      // [nq * K]       (search mode)
    float* out_dists;        // [nq * K]
    float out_scale;         // 1 for L2, 0.5 for IP / COS
    u64* cand;               // [nq * cand_cap] keys of R_L (indexing mode), sorted per round
    u32* cand_cnt;           // [nq]
    u32 cand_cap;
    u64* pes;                // [nq * deg] indexing mode: PES buffer H(v), ascending keys, PAG_KEY_INVALID = empty; null = off
    const u32* order;        // [nq] the order in which the waves take the queries (null: as numbered)
    u32* qcounter;
    u64* counters;
    u32* bitmap;             // [grid * bitmap_words]
    u64 bitmap_words;
};

// kernels / launchers (defined in the .hip files)
int pag_launch_search(const pag_index* ix, const SearchArgs& a, u32 lds_bytes, int* grid_out);
int pag_search_lds_bytes(const pag_layout& L, u32 b, u32 hlog, u32 blog, SearchArgs* a);
int pag_search_max_grid(const pag_index* ix, u32 b, u32 lds_bytes, int* grid);

int pag_launch_rotate(hipStream_t s, const float* X, u64 rows, u32 d, const float* rot, float* out);
int pag_launch_tables(hipStream_t s, const float* qrot, u64 rows, const pag_layout& L, const float* cb, float* tables);
int pag_launch_normalise(hipStream_t s, const float* X, u64 rows, u32 d, float* out);
int pag_launch_zero_u32(hipStream_t s, u32* p, u64 count);
// The order in which a batch of rotated queries is best taken (queries that run side by side should search the same
// part of the graph); *order points into ix->ws_order.  Allocates (grows ix->ws_order).
int pag_order_queries(pag_index* ix, const float* qrot, u64 nq, const u32** order);
int pag_launch_convert(hipStream_t s, const void* src, u32 src_half, void* dst, u32 dst_half, u64 count);   // float <-> __half, round to nearest even
int pag_launch_exact(hipStream_t s, const pag_index* ix, const float* qrot, u64 nq, const u32* ids, u32 m, float* keys);
int pag_launch_screen(hipStream_t s, const pag_index* ix, const float* tables, u64 nq, const u32* u, const float* Du, float* est);
// recomputes every slot of nodes [node_begin, node_end) into records / e2 rows that start at node out_base
int pag_launch_edge_info_nodes(hipStream_t s, const pag_index* ix, u64 node_begin, u64 node_end, uint8_t* recs,
                               float* e2, u64 out_base);
int pag_launch_row_reads(hipStream_t s, const pag_index* ix, u64 rows, u64 stride, u32* sink, int grid);
int pag_launch_hop_traffic(hipStream_t s, const pag_index* ix, u64 hops, u32* bitmap, u64 bitmap_words, u32* sink, int grid);
int pag_launch_edge_info_list(hipStream_t s, const pag_index* ix, const u32* edge_list, u64 n_edges);
int pag_launch_edge_info_of(hipStream_t s, const pag_index* ix, const u32* nodes, u64 m);   // every slot of m listed nodes (device ids)

int pag_search_common(pag_index* ix, u32 b, u32 ef, u64 n_limit, SearchArgs* a, u32* lds, int* grid);
inline pag_vecs pag_vecs_of(const pag_index* ix) { return pag_vecs{ ix->vec, ix->L.d, ix->vec_half }; }
inline size_t pag_vec_elem(const pag_index* ix) { return ix->vec_half ? 2 : 4; }
int pag_build_range(pag_index* ix, u64 n_begin, u64 n_end);   // batch-synchronous insertion of nodes [n_begin, n_end)
