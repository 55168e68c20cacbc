// Stand-alone kernels for single steps of the method: batched exact distances, the projection
// screen of one expanded node, and the inference information of edges (Sec. 3.1, Appendix B/C).
#include "pag_internal.h"

namespace {

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// keys[i*m+j] = fl32( sum_k fl32(q_i[k] - x_id[k])^2 ), one wave per (i, j); float4 loads.
__global__ void __launch_bounds__(64) k_exact(pag_vecs V, const float* __restrict__ qrot,
                                              u64 nq, u32 d, u64 n, const u32* __restrict__ ids, u32 m,
                                              float* __restrict__ keys) {
    const u64 pair = blockIdx.x;
    if (pair >= nq * m) return;
    const int lane = threadIdx.x;
    const u32 id = ids[pair];
    if (id >= n) { if (lane == 0) keys[pair] = __builtin_nanf(""); return; }
    const float4* q = (const float4*)(qrot + (pair / m) * d);
    double acc = 0.0;
    for (u32 c = lane; c < d / 4; c += 64) {
        const float4 a = q[c], b = pag_vload4(V, id, c);
        const float dx = a.x - b.x, dy = a.y - b.y, dz = a.z - b.z, dw = a.w - b.w;
        acc = __builtin_fma((double)dx, (double)dx, acc);
        acc = __builtin_fma((double)dy, (double)dy, acc);
        acc = __builtin_fma((double)dz, (double)dz, acc);
        acc = __builtin_fma((double)dw, (double)dw, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) keys[pair] = (float)acc;
}

// est[i*deg+s] = fmaf(-2 a_s, S_s, Du_i + c_s),  S_s = sum_l T_i[l][code_sl] over increasing l.
__global__ void __launch_bounds__(64) k_screen(const uint8_t* __restrict__ recs, pag_layout L, u64 n,
                                               const float* __restrict__ tables, u64 nq,
                                               const u32* __restrict__ us, const float* __restrict__ Dus,
                                               float* __restrict__ est) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* T = (float*)smem;
    const u64 qi = blockIdx.x;
    if (qi >= nq) return;
    const int lane = threadIdx.x;
    const float* tp = tables + qi * L.Ppad * PAG_NCODE;
    for (u32 i = lane; i < L.Ppad * PAG_NCODE; i += 64) T[i] = tp[i];
    __syncthreads();
    const u32 u = us[qi];
    if ((u32)lane >= L.deg) return;
    float out = __builtin_nanf("");
    if (u < n) {
        const uint8_t* rec = recs + (u64)u * L.rec_bytes;
        const u32 id = ((const u32*)rec)[lane];
        if (id != PAG_EMPTY) {
            const float a = ((const float*)(rec + L.off_a))[lane];
            const float c = ((const float*)(rec + L.off_c))[lane];
            const u32* cp = (const u32*)(rec + L.off_codes) + (u32)lane * L.cw;
            float S = 0.f;
            for (u32 k = 0; k < L.cw; ++k) {
                const u32 wd = cp[k];
                for (u32 t = 0; t < 8; ++t) S = S + T[(k * 8 + t) * PAG_NCODE + ((wd >> (4 * t)) & 15u)];
            }
            out = __builtin_fmaf(-2.0f * a, S, Dus[qi] + c);
        }
    }
    est[qi * L.deg + lane] = out;
}

// Inference information of one edge (u, slot) per wave.
//   codes[l] = argmax_j <r_jl, (w-u)_l>  (ties -> smallest j), k ascending fp64 sums
//   e2 = ||w-u||^2, maxsum = sum_l best_l, off = sum_l <u_l, r*_l>  (l ascending)
//   a = ||w-u|| / max(maxsum/||w-u||, 1e-6), c = e2 + 2 a off; both 0 when w == u
// Lane l owns subspace l (l, l+64, ...).  Results go straight into the adjacency record and e2;
// `recs` and `e2_out` start at node `out_base` (0 for the index itself, or a scratch copy of a range).
__global__ void __launch_bounds__(64) k_edge_info(pag_vecs V, uint8_t* __restrict__ recs,
                                                  float* __restrict__ e2_out, pag_layout L,
                                                  const float* __restrict__ cb, const u32* __restrict__ edges,
                                                  u64 n_edges, const u32* __restrict__ nodes, u64 node_begin, u64 out_base) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* diff = (float*)smem;               // [d]
    float* uu = diff + L.d;                   // [d]
    double* best = (double*)(uu + L.d);       // [P]
    double* offs = best + L.P;                // [P]
    u32* code = (u32*)(offs + L.P);           // [Ppad]
    const int lane = threadIdx.x;
    u32 u, slot;
    if (edges) {
        if (blockIdx.x >= n_edges) return;
        u = edges[2 * (u64)blockIdx.x];
        slot = edges[2 * (u64)blockIdx.x + 1];
    } else {
        // every slot of a listed node, or of the node range that starts at node_begin
        u = nodes ? nodes[blockIdx.x / L.deg] : (u32)(node_begin + blockIdx.x / L.deg);
        slot = blockIdx.x % L.deg;
    }
    uint8_t* rec = recs + ((u64)u - out_base) * L.rec_bytes;
    float* e2_row = e2_out + ((u64)u - out_base) * L.deg;
    const u32 w = ((const u32*)rec)[slot];
    u32* cw_out = (u32*)(rec + L.off_codes) + slot * L.cw;
    if (w == PAG_EMPTY) {
        if (lane == 0) {
            ((float*)(rec + L.off_a))[slot] = 0.f;
            ((float*)(rec + L.off_c))[slot] = 0.f;
            e2_row[slot] = 0.f;
        }
        if ((u32)lane < L.cw) cw_out[lane] = 0u;
        return;
    }
    double e2p = 0.0;
    for (u32 k = lane; k < L.d; k += 64) {
        const float a = pag_vload1(V, u, k), df = pag_vload1(V, w, k) - a;
        uu[k] = a; diff[k] = df;
        e2p = __builtin_fma((double)df, (double)df, e2p);
    }
    for (u32 l = L.P + lane; l < L.Ppad; l += 64) code[l] = 0u;
    const double e2 = wave_sum(e2p);
    __syncthreads();
    // Four subspaces at a time: each 16-lane row takes one subspace, each of its lanes one of the
    // sixteen reference vectors, so that a row reads one contiguous 16 x dsub block of the codebook.
    // The dot products run over k in order; the row's argmax keeps the smallest index among equal
    // values, as a scan in index order would.
    const u32 j = (u32)lane & 15u, row = (u32)lane >> 4;
    for (u32 l0 = 0; l0 < L.P; l0 += 4) {
        const u32 l = l0 + row;
        const bool live = l < L.P;
        const u32 lc = live ? l : 0u;
        const float* r = cb + ((u64)lc * PAG_NCODE + j) * L.dsub;
        double acc = 0.0;
        for (u32 k = 0; k < L.dsub; ++k) acc = __builtin_fma((double)r[k], (double)diff[lc * L.dsub + k], acc);
        double bv = acc;
        u32 bj = j;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            const double ov = __shfl_xor(bv, o, 64);
            const u32 oj = (u32)__shfl_xor((int)bj, o, 64);
            if (ov > bv || (ov == bv && oj < bj)) { bv = ov; bj = oj; }
        }
        if (live && j == 0) {
            const float* rb = cb + ((u64)l * PAG_NCODE + bj) * L.dsub;
            double o = 0.0;
            for (u32 k = 0; k < L.dsub; ++k) o = __builtin_fma((double)rb[k], (double)uu[l * L.dsub + k], o);
            best[l] = bv; offs[l] = o; code[l] = bj;
        }
    }
    __syncthreads();
    if ((u32)lane < L.cw) {
        u32 wd = 0;
        for (u32 t = 0; t < 8; ++t) wd |= (code[lane * 8 + t] & 15u) << (4 * t);
        cw_out[lane] = wd;
    }
    if (lane == 0) {
        double maxsum = 0.0, off = 0.0;
        for (u32 l = 0; l < L.P; ++l) { maxsum += best[l]; off += offs[l]; }
        double a = 0.0, c = 0.0;
        if (e2 > 0.0) {
            const double e = sqrt(e2);
            double cosb = maxsum / e;
            if (cosb < 1e-6) cosb = 1e-6;
            a = e / cosb;
            c = e2 + 2.0 * a * off;
        }
        ((float*)(rec + L.off_a))[slot] = (float)a;
        ((float*)(rec + L.off_c))[slot] = (float)c;
        e2_row[slot] = (float)e2;
    }
}

// Diagnostic: how fast can this GPU deliver whole rows of the vector store?  Every wave reads rows
// (four in flight) and folds them into a checksum; `stride` = 0 walks the store in order, otherwise
// row = (counter * stride) mod n visits it in a scattered order.  No arithmetic of the method.
__global__ void __launch_bounds__(64) k_row_reads(const uint4* __restrict__ vec, u64 row_chunks, u64 n, u64 rows,
                                                  u64 stride, u32* __restrict__ sink) {
    const int lane = threadIdx.x;
    u32 acc = 0;
    for (u64 r0 = (u64)blockIdx.x * 4; r0 < rows; r0 += (u64)gridDim.x * 4) {
        uint4 v[4];
        u64 row[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) row[g] = stride ? ((r0 + g) * stride) % n : (r0 + g) % n;
        for (u64 c = lane; c < row_chunks; c += 64) {
#pragma unroll
            for (int g = 0; g < 4; ++g) v[g] = vec[row[g] * row_chunks + c];
#pragma unroll
            for (int g = 0; g < 4; ++g) acc ^= v[g].x ^ v[g].y ^ v[g].z ^ v[g].w;
        }
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;     // practically never: keeps the loads alive
}

__device__ __forceinline__ u64 mix64(u64 x) {
    x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33;
    return x;
}

// Diagnostic: the memory traffic of one hop of a long search without any of its arithmetic.  Per
// "hop": one adjacency record, seven random rows of the vector store (four, then three in flight),
// eight random words of the wave's seen-set bitmap read and seven random bits of it set -- the mix
// the search kernel produces at about seven admitted neighbours per hop.  No step of the method.
__global__ void __launch_bounds__(64) k_hop_traffic(const uint4* __restrict__ vec, u64 row_chunks, const uint4* __restrict__ rec,
                                                    u64 rec_chunks, u64 n, u64 hops, u32* __restrict__ bitmap,
                                                    u64 bitmap_words, u32* __restrict__ sink) {
    const int lane = threadIdx.x;
    u32 acc = 0;
    u32* bm = bitmap + (u64)blockIdx.x * bitmap_words;
    for (u64 h = blockIdx.x; h < hops; h += gridDim.x) {
        const u64 u = mix64(h * 2654435761ull) % n;
        for (u64 c = lane; c < rec_chunks; c += 64) { const uint4 t = rec[u * rec_chunks + c]; acc ^= t.x ^ t.y ^ t.z ^ t.w; }
        if (lane < 8) acc ^= __hip_atomic_load(&bm[mix64(h * 977 + lane) % bitmap_words], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        u64 row[7];
#pragma unroll
        for (int g = 0; g < 7; ++g) row[g] = mix64(h * 7 + g + 12345) % n;
        for (int g0 = 0; g0 < 7; g0 += 4) {
            for (u64 c = lane; c < row_chunks; c += 64) {
                uint4 v[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) v[g] = vec[row[g0 + g < 7 ? g0 + g : 6] * row_chunks + c];
#pragma unroll
                for (int g = 0; g < 4; ++g) acc ^= v[g].x ^ v[g].y ^ v[g].z ^ v[g].w;
            }
        }
        if (lane < 7) atomicOr(&bm[mix64(h * 31 + lane + 99) % bitmap_words], 1u << (lane & 31));
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;
}

u32 edge_info_lds(const pag_layout& L) { return 2 * L.d * 4 + 2 * L.P * 8 + L.Ppad * 4; }

}  // namespace

int pag_launch_exact(hipStream_t s, const pag_index* ix, const float* qrot, u64 nq, const u32* ids, u32 m,
                     float* keys) {
    const u64 pairs = nq * m;
    if (pairs == 0) return PAG_OK;
    if (pairs > 0x7FFFFFFFull) { pag_set_error("pag_exact_distances: more than 2^31-1 pairs"); return PAG_EINVAL; }
    hipLaunchKernelGGL(k_exact, dim3((unsigned)pairs), dim3(64), 0, s, pag_vecs_of(ix), qrot, nq, ix->L.d, ix->n, ids, m, keys);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_screen(hipStream_t s, const pag_index* ix, const float* tables, u64 nq, const u32* u,
                      const float* Du, float* est) {
    if (nq == 0) return PAG_OK;
    hipLaunchKernelGGL(k_screen, dim3((unsigned)nq), dim3(64), ix->L.Ppad * PAG_NCODE * 4, s, ix->rec, ix->L,
                       ix->n, tables, nq, u, Du, est);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_edge_info_nodes(hipStream_t s, const pag_index* ix, u64 node_begin, u64 node_end, uint8_t* recs,
                               float* e2, u64 out_base) {
    if (node_end <= node_begin) return PAG_OK;
    const u64 total = (node_end - node_begin) * ix->L.deg;
    const u64 step = 1ull << 30;
    for (u64 o = 0; o < total; o += step) {
        // slabs of whole nodes so that blockIdx maps to (node, slot)
        const u64 nodes_per = step / ix->L.deg;
        const u64 nb = node_begin + (o / step) * nodes_per;
        const u64 ne = nb + nodes_per < node_end ? nb + nodes_per : node_end;
        if (nb >= node_end) break;
        hipLaunchKernelGGL(k_edge_info, dim3((unsigned)((ne - nb) * ix->L.deg)), dim3(64), edge_info_lds(ix->L), s,
                           pag_vecs_of(ix), recs, e2, ix->L, ix->cb, (const u32*)nullptr, 0ull, (const u32*)nullptr, nb, out_base);
    }
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_edge_info_list(hipStream_t s, const pag_index* ix, const u32* edge_list, u64 n_edges) {
    if (n_edges == 0) return PAG_OK;
    hipLaunchKernelGGL(k_edge_info, dim3((unsigned)n_edges), dim3(64), edge_info_lds(ix->L), s, pag_vecs_of(ix), ix->rec,
                       ix->e2, ix->L, ix->cb, edge_list, n_edges, (const u32*)nullptr, 0ull, 0ull);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_edge_info_of(hipStream_t s, const pag_index* ix, const u32* nodes, u64 m) {
    if (m == 0) return PAG_OK;
    hipLaunchKernelGGL(k_edge_info, dim3((unsigned)(m * ix->L.deg)), dim3(64), edge_info_lds(ix->L), s, pag_vecs_of(ix), ix->rec,
                       ix->e2, ix->L, ix->cb, (const u32*)nullptr, 0ull, nodes, 0ull, 0ull);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_hop_traffic(hipStream_t s, const pag_index* ix, u64 hops, u32* bitmap, u64 bitmap_words, u32* sink, int grid) {
    const u64 row_chunks = (u64)ix->L.d * (ix->vec_half ? 2 : 4) / 16;
    hipLaunchKernelGGL(k_hop_traffic, dim3((unsigned)grid), dim3(64), 0, s, (const uint4*)ix->vec, row_chunks,
                       (const uint4*)ix->rec, (u64)ix->L.rec_bytes / 16, ix->n, hops, bitmap, bitmap_words, sink);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}

int pag_launch_row_reads(hipStream_t s, const pag_index* ix, u64 rows, u64 stride, u32* sink, int grid) {
    const u64 row_chunks = (u64)ix->L.d * (ix->vec_half ? 2 : 4) / 16;
    hipLaunchKernelGGL(k_row_reads, dim3((unsigned)grid), dim3(64), 0, s, (const uint4*)ix->vec, row_chunks, ix->n, rows,
                       stride, sink);
    PAG_HIP(hipGetLastError());
    return PAG_OK;
}
